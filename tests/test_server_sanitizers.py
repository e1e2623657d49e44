"""The serving front end under ThreadSanitizer and Address/UndefinedBehaviour sanitizers (host code only).

A host-only program (tests/native/server_race.cpp) links the front end's sources with stubs for the GPU-side entry
points and drives it with a fake executor from six client threads plus a polling thread, then stops it with work in
flight.  Any sanitizer report fails the test.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2604_28175_amd", "csrc")
CLANG = "/opt/rocm/llvm/bin/clang++"
HOST_SOURCES = ["server.cpp", "sched.cpp", "intf.cpp", "link.cpp"]


@pytest.mark.skipif(not os.path.exists(CLANG), reason="ROCm clang++ not found")
@pytest.mark.parametrize("sanitizer", ["thread", "address,undefined"])
def test_front_end_clean_under_sanitizer(tmp_path, sanitizer):
    exe = str(tmp_path / "server_race")
    cmd = [CLANG, "-std=c++17", "-O1", "-g", "-fsanitize=" + sanitizer, "-fno-sanitize-recover=all",
           "-I/opt/rocm/include", "-I" + os.path.join(ROOT, "include"), "-D__HIP_PLATFORM_AMD__",
           os.path.join(ROOT, "tests", "native", "server_race.cpp")]
    cmd += [os.path.join(CSRC, s) for s in HOST_SOURCES] + ["-o", exe, "-lpthread"]
    build = subprocess.run(cmd, capture_output=True, text=True, timeout=300)
    assert build.returncode == 0, build.stderr[-2000:]
    env = dict(os.environ, TSAN_OPTIONS="halt_on_error=1 exitcode=66", ASAN_OPTIONS="detect_leaks=1 exitcode=66")
    run = subprocess.run([exe], capture_output=True, text=True, timeout=120, env=env)
    assert "Sanitizer" not in run.stderr and "runtime error" not in run.stderr, run.stderr[-3000:]
    assert run.returncode == 0, (run.returncode, run.stdout[-500:], run.stderr[-2000:])
    assert "idle rc 0" in run.stdout
    shutil.rmtree(tmp_path, ignore_errors=True)
