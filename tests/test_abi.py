"""CPU-side checks of the boundary: the shared library loads without a GPU and exports exactly
the entry points include/strait.h declares; the binding marshals the same names."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared():
    text = open(os.path.join(ROOT, "include", "strait.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(strait_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(os.path.join(ROOT, "paper_2604_28175_amd", "libstrait.so"))
    names = declared()
    assert len(names) >= 25
    for n in names:
        assert hasattr(lib, n), f"{n} declared in strait.h but not exported"


def test_binding_covers_the_header():
    import paper_2604_28175_amd as strait
    assert sorted(strait.EXPORTS) == declared()
    assert strait.lib.strait_version() == 1


def test_error_paths_without_gpu():
    import paper_2604_28175_amd as strait
    assert strait.lib.strait_ctx_create(None, None) == strait.E_INVALID
    assert "null" in strait.last_error()
    assert strait.lib.strait_model_free(None) == strait.E_INVALID
    assert strait.lib.strait_wait(None, None) == strait.E_INVALID
