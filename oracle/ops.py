"""CPU oracle: the operators of a served batch's kernel sequence, as plain definitions.

TEST INFRASTRUCTURE ONLY.  Nothing under `oracle/` is imported by the served path; it exists
to check the GPU library (tests, the smoke check and the CPU-baseline leg of the benchmark).

The paper (Section 2; Section 3.2, step (2) "kernel execution") fixes only that a batch runs a
sequence of dependent kernels; which operators those are follows from the public architectures
being served (Table 1 lists ResNet-50 at 4.09 G multiply-accumulates).  Every operator below is
its textbook definition in fp64, activations NHWC:

  conv2d / dwconv2d / maxpool2d   nested loops in ops.c
  everything else                 a few numpy lines each

A float32 build of the convolution loops is exposed as `conv2d(..., f32=True)` only so that a
test can bound the oracle's own rounding error.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np
from scipy.special import erf as _erf

from .build import LIB, build

if not os.path.exists(LIB):
    build()
_lib = ctypes.CDLL(LIB)
_P = ctypes.c_void_p
_I = ctypes.c_int


def _ptr(a):
    return None if a is None else a.ctypes.data_as(_P)


def num_threads() -> int:
    """OpenMP threads the C loops run on."""
    return int(_lib.oracle_num_threads())


def out_size(h: int, k: int, stride: int, pad: int) -> int:
    return (h + 2 * pad - k) // stride + 1


def conv2d(x, w_oihw, b=None, stride=1, pad=0, f32=False):
    """x [N,H,W,C]; w_oihw [K,C,R,S]; b [K] -> y [N,P,Q,K].  Cross-correlation, zero padding."""
    real = np.float32 if f32 else np.float64
    x = np.ascontiguousarray(x, dtype=real)
    n, h, wd, c = x.shape
    k, c2, r, s = w_oihw.shape
    assert c2 == c
    w_rsck = np.ascontiguousarray(np.transpose(np.asarray(w_oihw, dtype=np.float32), (2, 3, 1, 0)))
    bb = None if b is None else np.ascontiguousarray(b, dtype=real)
    y = np.empty((n, out_size(h, r, stride, pad), out_size(wd, s, stride, pad), k), dtype=real)
    fn = _lib.oracle_conv2d_f32 if f32 else _lib.oracle_conv2d_f64
    fn(_ptr(x), _I(n), _I(h), _I(wd), _I(c), _ptr(w_rsck), _ptr(bb), _I(k), _I(r), _I(s),
       _I(stride), _I(pad), _ptr(y))
    return y


def dwconv2d(x, w_c1rs, b=None, stride=1, pad=0):
    """Depthwise: x [N,H,W,C]; w [C,1,R,S]; b [C] -> y [N,P,Q,C]."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    n, h, wd, c = x.shape
    c2, one, r, s = w_c1rs.shape
    assert c2 == c and one == 1
    w_rsc = np.ascontiguousarray(np.transpose(np.asarray(w_c1rs, dtype=np.float32)[:, 0], (1, 2, 0)))
    bb = None if b is None else np.ascontiguousarray(b, dtype=np.float64)
    y = np.empty((n, out_size(h, r, stride, pad), out_size(wd, s, stride, pad), c), dtype=np.float64)
    _lib.oracle_dwconv2d_f64(_ptr(x), _I(n), _I(h), _I(wd), _I(c), _ptr(w_rsc), _ptr(bb), _I(r), _I(s),
                             _I(stride), _I(pad), _ptr(y))
    return y


def maxpool2d(x, k=3, stride=2, pad=1):
    x = np.ascontiguousarray(x, dtype=np.float64)
    n, h, wd, c = x.shape
    y = np.empty((n, out_size(h, k, stride, pad), out_size(wd, k, stride, pad), c), dtype=np.float64)
    _lib.oracle_maxpool2d_f64(_ptr(x), _I(n), _I(h), _I(wd), _I(c), _I(k), _I(stride), _I(pad), _ptr(y))
    return y


def relu(x):
    return np.maximum(x, 0.0)


def relu6(x):
    return np.minimum(np.maximum(x, 0.0), 6.0)


def global_avg_pool(x):
    """[N,H,W,C] -> [N,C]: mean over the H*W positions."""
    n, h, w, c = x.shape
    return x.reshape(n, h * w, c).sum(axis=1) / float(h * w)


def linear(x, w, b=None):
    """x [..., in]; w [out, in]; y = x w^T + b."""
    y = np.asarray(x, dtype=np.float64) @ np.asarray(w, dtype=np.float64).T
    return y if b is None else y + np.asarray(b, dtype=np.float64)


def softmax(x):
    """Row-wise over the last axis: exp(x - max) / sum."""
    x = np.asarray(x, dtype=np.float64)
    e = np.exp(x - x.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def argmax_first(x):
    """Index of the maximum over the last axis, lowest index on exact ties, int32."""
    return np.argmax(x, axis=-1).astype(np.int32)


def gelu(x):
    """Exact (erf) GELU: 0.5 x (1 + erf(x / sqrt 2))."""
    x = np.asarray(x, dtype=np.float64)
    return 0.5 * x * (1.0 + _erf(x / np.sqrt(2.0)))


def layernorm(x, gamma, beta, eps=1e-12):
    """Over the last axis, biased variance."""
    x = np.asarray(x, dtype=np.float64)
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * np.asarray(gamma, np.float64) + np.asarray(beta, np.float64)


def attention(q, k, v, valid_len, heads):
    """Multi-head scaled dot-product attention with a key-padding mask.

    q, k, v [B,S,hidden]; valid_len [B].  For sequence b only keys j < valid_len[b] take part
    (masked keys get probability exactly zero).  Every query row is computed."""
    q = np.asarray(q, np.float64)
    k = np.asarray(k, np.float64)
    v = np.asarray(v, np.float64)
    bsz, s, hid = q.shape
    d = hid // heads
    out = np.zeros_like(q)
    for b in range(bsz):
        L = int(valid_len[b])
        for h in range(heads):
            sl = slice(h * d, (h + 1) * d)
            sc = (q[b, :, sl] @ k[b, :L, sl].T) / np.sqrt(float(d))
            out[b, :, sl] = softmax(sc) @ v[b, :L, sl]
    return out


def fold_bn(w, gamma, beta, mean, var, eps=1e-5):
    """BatchNorm folded into the preceding convolution, in fp32:
         scale = gamma / sqrt(var + eps);  w' = fp16(w * scale[k]);  b' = beta - mean * scale (fp32).
    The folded weight is rounded to fp16 once (round-to-nearest-even), as the GPU stores it."""
    f = np.float32
    scale = gamma.astype(f) / np.sqrt(var.astype(f) + f(eps))
    wf = (w.astype(f) * scale.reshape(-1, 1, 1, 1)).astype(np.float16)
    bf = beta.astype(f) - mean.astype(f) * scale
    return wf, bf.astype(f)
