"""Compile the oracle's C loops (ops.c) into oracle/liboracle.so with gcc.

Two instantiations are linked into one library: `_f64` (the oracle proper) and `_f32`
(used only to measure the oracle's own rounding error against the fp64 build)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "liboracle.so")


def build(force: bool = True) -> str:
    src = os.path.join(HERE, "ops.c")
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(src):
        return LIB
    base = ["gcc", "-O2", "-ftree-vectorize", "-mavx2", "-mfma", "-fopenmp", "-fPIC", "-std=c11", "-c", src]
    o64 = os.path.join(HERE, "ops_f64.o")
    o32 = os.path.join(HERE, "ops_f32.o")
    subprocess.check_call(base + ["-DREAL=double", "-DSUFFIX=f64", "-DORACLE_COMMON", "-o", o64])
    subprocess.check_call(base + ["-DREAL=float", "-DSUFFIX=f32", "-o", o32])
    subprocess.check_call(["gcc", "-shared", "-fopenmp", "-o", LIB, o64, o32, "-lm"])
    os.remove(o64)
    os.remove(o32)
    return LIB


if __name__ == "__main__":
    print(build())
