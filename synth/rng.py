"""Counter-based seeded random numbers for the synthetic workloads.

Every draw is a pure function of (seed, stream name, element index): the
64-bit SplitMix64 finaliser (Steele, Lea & Flood, "Fast splittable
pseudorandom number generators", OOPSLA 2014) applied to
``key + (index + 1) * GOLDEN``, where ``key`` mixes the seed with an FNV-1a
hash of the stream name.  Nothing here is part of the served models'
arithmetic; both the CPU oracle and the GPU library only ever see the
generated numbers.
"""
from __future__ import annotations

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _mix(z: np.ndarray) -> np.ndarray:
    z = z.astype(np.uint64, copy=True)
    z ^= z >> np.uint64(30)
    z *= _M1
    z ^= z >> np.uint64(27)
    z *= _M2
    z ^= z >> np.uint64(31)
    return z


def _fnv1a(name: str) -> int:
    h = 0xCBF29CE484222325
    for b in name.encode("utf-8"):
        h ^= b
        h = (h * 0x100000001B3) & 0xFFFFFFFFFFFFFFFF
    return h


def stream_key(seed: int, name: str) -> np.uint64:
    with np.errstate(over="ignore"):
        k = _mix(np.array([(seed & 0xFFFFFFFFFFFFFFFF) ^ _fnv1a(name)], dtype=np.uint64))
    return k[0]


def bits(seed: int, name: str, n: int, offset: int = 0) -> np.ndarray:
    """n 64-bit words of stream (seed, name), starting at element `offset`."""
    key = stream_key(seed, name)
    with np.errstate(over="ignore"):
        idx = np.arange(offset + 1, offset + n + 1, dtype=np.uint64)
        return _mix(key + idx * _GOLDEN)


def uniform(seed: int, name: str, n: int, lo: float = 0.0, hi: float = 1.0) -> np.ndarray:
    """n doubles uniform on [lo, hi): the top 53 bits of each word."""
    u = (bits(seed, name, n) >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)
    return lo + (hi - lo) * u


def normal(seed: int, name: str, n: int, mean: float = 0.0, std: float = 1.0) -> np.ndarray:
    """n doubles N(mean, std^2) by Box-Muller; element i uses words 2i and 2i+1."""
    w = bits(seed, name, 2 * n)
    u1 = (w[0::2] >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)
    u2 = (w[1::2] >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)
    r = np.sqrt(-2.0 * np.log1p(-u1))          # 1-u1 in (0,1]
    return mean + std * r * np.cos(2.0 * np.pi * u2)


def integers(seed: int, name: str, n: int, lo: int, hi: int) -> np.ndarray:
    """n int64 uniform on {lo..hi} inclusive (multiply-shift on the top 32 bits)."""
    w = bits(seed, name, n) >> np.uint64(32)
    span = np.uint64(hi - lo + 1)
    return (lo + ((w * span) >> np.uint64(32)).astype(np.int64)).astype(np.int64)


def exponential(seed: int, name: str, n: int, rate: float) -> np.ndarray:
    """n doubles Exp(rate): -ln(1-u)/rate."""
    return -np.log1p(-uniform(seed, name, n)) / rate
