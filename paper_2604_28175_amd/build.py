"""Compile the HIP kernels and the C-ABI runtime into paper_2604_28175_amd/libstrait.so (gfx950)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libstrait.so")
SOURCES = ["conv_igemm.hip", "elementwise.hip", "attention.hip", "stem_pool.hip", "noalloc.hip", "pointwise_pair.hip", "stem3x3.hip", "expand_dw.hip", "plan.cpp", "api.cpp", "link.cpp", "intf.cpp", "sched.cpp", "server.cpp"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
COMMON = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-Wall", "-Wno-unused-result",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-mf16c"]
# The BatchNorm fold on the host must round its product before the subtraction (two IEEE
# operations, as the specification of the fold says), so the host-only sources disable contraction.
HOST_ONLY = ["-ffp-contract=off"]


def _compile(src: str) -> str:
    obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC] + COMMON + (HOST_ONLY if src.endswith(".cpp") else []) + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build() -> str:
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    r = subprocess.run([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs + ["-lpthread"],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    for o in objs:
        os.remove(o)
    # the stand-alone ceilings program (MFMA, LDS-fed MFMA, streaming and host-link rates of the machine)
    r = subprocess.run([HIPCC] + COMMON + [os.path.join(CSRC, "ceilings.hip"), "-o", os.path.join(HERE, "ceilings")],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on ceilings.hip:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build())
