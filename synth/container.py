"""The weight container handed to the GPU library (`STRW`, version 1).

Layout (little endian):
  header, 48 B : magic "STRW", u32 version (=1), u32 arch, u32 n_tensors, u32 hyper[8]
  n_tensors entries, 80 B each:
                 char name[40] (NUL padded), u32 dtype (0 = fp16), u32 ndim,
                 u32 shape[4], u64 offset (from the start of the blob, 64-B aligned),
                 u64 nbytes
  tensor data, each tensor contiguous, row-major, in the shape given.
Conv weights are OIHW, linear weights [out, in].  Pure serialisation: no arithmetic.
"""
from __future__ import annotations

import struct

import numpy as np

from .models import ModelData

MAGIC = b"STRW"
VERSION = 1
HEADER_BYTES = 48
ENTRY_BYTES = 80


def pack(md: ModelData) -> bytes:
    names = list(md.tensors.keys())
    n = len(names)
    hyper = list(md.hyper) + [0] * (8 - len(md.hyper))
    off = HEADER_BYTES + ENTRY_BYTES * n
    off = (off + 63) // 64 * 64
    entries, chunks = [], []
    for nm in names:
        t = md.tensors[nm]
        assert t.dtype == np.float16 and t.ndim <= 4 and len(nm) < 40
        shape = list(t.shape) + [1] * (4 - t.ndim)
        nbytes = t.size * 2
        entries.append(struct.pack("<40sII4IQQ", nm.encode(), 0, t.ndim, *shape, off, nbytes))
        pad = (-nbytes) % 64
        chunks.append(t.tobytes() + b"\0" * pad)
        off += nbytes + pad
    head = struct.pack("<4sIII8I", MAGIC, VERSION, md.arch, n, *hyper)
    body = head + b"".join(entries)
    body += b"\0" * ((-len(body)) % 64)
    return body + b"".join(chunks)
