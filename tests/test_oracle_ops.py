"""Pins of the CPU oracle's operators against things other than the oracle itself:
hand-worked fixtures, closed forms, invariants, and independent library formulations
(pad + sliding windows + tensordot instead of bounds-checked loops)."""
import os

import numpy as np
import pytest
from numpy.lib.stride_tricks import sliding_window_view

from oracle import ops

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
R = np.random.default_rng(1234)


def _table(path, section):
    rows, on = [], False
    for line in open(path):
        line = line.strip()
        if not line or line[0] == "#":
            continue
        if line[0].isalpha():
            on = line == section
            continue
        if on:
            rows.append([float(v) for v in line.split()])
    return np.array(rows)


def conv_by_windows(x, w, b, stride, pad):
    """Independent formulation: explicit zero padding, all windows, one tensordot."""
    xp = np.pad(np.asarray(x, np.float64), ((0, 0), (pad, pad), (pad, pad), (0, 0)))
    win = sliding_window_view(xp, (w.shape[2], w.shape[3]), axis=(1, 2))[:, ::stride, ::stride]  # N,P,Q,C,R,S
    y = np.tensordot(win, np.asarray(w, np.float64), axes=([3, 4, 5], [1, 2, 3]))
    return y if b is None else y + b


# ------------------------------------------------------------------ conv2d
def test_conv_hand_worked_sobel():
    x = (np.arange(16, dtype=np.float64) + 1).reshape(1, 4, 4, 1)
    w = np.array([[1, 0, -1], [2, 0, -2], [1, 0, -1]], np.float32).reshape(1, 1, 3, 3)
    p = os.path.join(GOLDEN, "sobel_4x4.txt")
    assert np.array_equal(ops.conv2d(x, w, None, 1, 1)[0, :, :, 0], _table(p, "stride1"))
    assert np.array_equal(ops.conv2d(x, w, None, 2, 1)[0, :, :, 0], _table(p, "stride2"))


def test_conv_identity_and_shift_kernels():
    x = R.standard_normal((2, 6, 7, 3))
    for (r, s) in [(1, 1), (0, 1), (1, 2), (2, 0)]:
        w = np.zeros((3, 3, 3, 3), np.float32)
        for c in range(3):
            w[c, c, r, s] = 1.0
        y = ops.conv2d(x, w, None, 1, 1)
        # y[p,q] = x[p + r - 1, q + s - 1] where inside, else 0
        want = np.zeros_like(x)
        dh, dw = r - 1, s - 1
        hs = slice(max(0, -dh), 6 - max(0, dh))
        ws = slice(max(0, -dw), 7 - max(0, dw))
        want[:, hs, ws] = x[:, hs.start + dh:hs.stop + dh, ws.start + dw:ws.stop + dw]
        assert np.array_equal(y, want), (r, s)


def test_conv_tap_counts_all_ones():
    for stride, hw in [(1, 5), (2, 6), (2, 7)]:
        y = ops.conv2d(np.ones((1, hw, hw, 1)), np.ones((1, 1, 3, 3), np.float32), None, stride, 1)[0, :, :, 0]
        P = (hw + 2 - 3) // stride + 1
        assert y.shape == (P, P)
        cnt = lambda i: sum(0 <= i * stride + r - 1 < hw for r in range(3))
        want = np.array([[cnt(i) * cnt(j) for j in range(P)] for i in range(P)], float)
        assert np.array_equal(y, want)
    assert ops.conv2d(np.ones((1, 5, 5, 1)), np.ones((1, 1, 3, 3), np.float32), None, 1, 1)[0, 0, 0, 0] == 4
    assert ops.conv2d(np.ones((1, 5, 5, 1)), np.ones((1, 1, 3, 3), np.float32), None, 1, 1)[0, 0, 2, 0] == 6
    assert ops.conv2d(np.ones((1, 5, 5, 1)), np.ones((1, 1, 3, 3), np.float32), None, 1, 1)[0, 2, 2, 0] == 9


def test_conv_1x1_is_matmul():
    x = R.standard_normal((2, 5, 4, 16))
    w = R.standard_normal((8, 16, 1, 1)).astype(np.float32)
    b = R.standard_normal(8)
    y = ops.conv2d(x, w, b)
    want = x.reshape(-1, 16) @ w[:, :, 0, 0].astype(np.float64).T + b
    assert np.allclose(y.reshape(-1, 8), want, rtol=1e-13, atol=1e-13)
    # strided 1x1 picks every other pixel
    y2 = ops.conv2d(x, w, b, stride=2)
    assert np.allclose(y2, y[:, ::2, ::2], rtol=0, atol=0)


@pytest.mark.parametrize("k,stride,pad,hw,c,co", [(3, 1, 1, 9, 5, 7), (3, 2, 1, 10, 4, 6), (7, 2, 3, 17, 3, 8),
                                                    (3, 2, 1, 9, 6, 3), (1, 2, 0, 8, 6, 4), (3, 1, 0, 6, 2, 2)])
def test_conv_matches_window_formulation(k, stride, pad, hw, c, co):
    x = R.standard_normal((2, hw, hw + 1, c))
    w = R.standard_normal((co, c, k, k)).astype(np.float32)
    b = R.standard_normal(co)
    y = ops.conv2d(x, w, b, stride, pad)
    want = conv_by_windows(x, w, b, stride, pad)
    assert y.shape == want.shape
    assert np.allclose(y, want, rtol=1e-12, atol=1e-12)


def test_conv_not_symmetric_in_rs():
    """A transposed (r,s) or flipped kernel must fail: asymmetric kernel, asymmetric image."""
    x = np.zeros((1, 5, 5, 1)); x[0, 1, 3, 0] = 1.0
    w = np.arange(9, dtype=np.float32).reshape(1, 1, 3, 3)
    y = ops.conv2d(x, w, None, 1, 1)[0, :, :, 0]
    # impulse at (1,3): y[p,q] = w[1-p+1, 3-q+1]
    for p in range(5):
        for q in range(5):
            r, s = 1 - p + 1, 3 - q + 1
            want = w[0, 0, r, s] if 0 <= r < 3 and 0 <= s < 3 else 0.0
            assert y[p, q] == want


def test_conv_linearity():
    x1, x2 = R.standard_normal((1, 6, 6, 4)), R.standard_normal((1, 6, 6, 4))
    w = R.standard_normal((5, 4, 3, 3)).astype(np.float32)
    a, b = 0.5, -2.0
    lhs = ops.conv2d(a * x1 + b * x2, w, None, 2, 1)
    rhs = a * ops.conv2d(x1, w, None, 2, 1) + b * ops.conv2d(x2, w, None, 2, 1)
    assert np.allclose(lhs, rhs, rtol=1e-12, atol=1e-12)


def test_conv_f32_build_bounds_own_rounding():
    x = R.standard_normal((1, 14, 14, 256))
    w = (R.standard_normal((64, 256, 3, 3)) * (2.0 / 2304) ** 0.5).astype(np.float16).astype(np.float32)
    y64 = ops.conv2d(x.astype(np.float16), w, None, 1, 1)
    y32 = ops.conv2d(x.astype(np.float16), w, None, 1, 1, f32=True)
    assert np.abs(y64 - y32).max() <= 1e-5 * np.abs(y64).max()


# ------------------------------------------------------------------ depthwise
def test_dwconv_is_per_channel_correlation():
    x = R.standard_normal((2, 9, 8, 6))
    w = R.standard_normal((6, 1, 3, 3)).astype(np.float32)
    b = R.standard_normal(6)
    for stride in (1, 2):
        y = ops.dwconv2d(x, w, b, stride, 1)
        for c in range(6):
            want = conv_by_windows(x[..., c:c + 1], w[c:c + 1], b[c:c + 1], stride, 1)
            assert np.allclose(y[..., c:c + 1], want, rtol=1e-12, atol=1e-12)


def test_dwconv_equals_block_diagonal_conv():
    x = R.standard_normal((1, 7, 7, 4))
    w = R.standard_normal((4, 1, 3, 3)).astype(np.float32)
    full = np.zeros((4, 4, 3, 3), np.float32)
    for c in range(4):
        full[c, c] = w[c, 0]
    assert np.allclose(ops.dwconv2d(x, w, None, 2, 1), ops.conv2d(x, full, None, 2, 1), rtol=1e-13, atol=1e-13)


# ------------------------------------------------------------------ BN fold
def test_bn_fold_matches_unfused_batchnorm():
    x = R.standard_normal((1, 6, 6, 8)).astype(np.float16)
    w = (R.standard_normal((5, 8, 3, 3)) * 0.2).astype(np.float16)
    g = R.uniform(0.8, 1.2, 5).astype(np.float16); be = (R.standard_normal(5) * .05).astype(np.float16)
    mu = (R.standard_normal(5) * .05).astype(np.float16); var = R.uniform(0.8, 1.2, 5).astype(np.float16)
    wf, bf = ops.fold_bn(w, g, be, mu, var)
    assert wf.dtype == np.float16 and bf.dtype == np.float32
    fused = ops.conv2d(x, wf, bf, 1, 1)
    conv = conv_by_windows(x, w.astype(np.float64), None, 1, 1)
    unfused = (conv - mu.astype(np.float64)) / np.sqrt(var.astype(np.float64) + 1e-5) * g.astype(np.float64) + be.astype(np.float64)
    # only difference: the folded weight is rounded to fp16 (2^-11 relative per weight)
    assert np.abs(fused - unfused).max() < 3e-3 * np.abs(unfused).max()
    # and in exact arithmetic (no fp16 rounding of w') it is an identity to fp32 precision
    scale = g.astype(np.float64) / np.sqrt(var.astype(np.float64) + 1e-5)
    exact = conv_by_windows(x, w.astype(np.float64) * scale[:, None, None, None], be - mu * scale, 1, 1)
    assert np.allclose(exact, unfused, rtol=1e-10, atol=1e-10)


# ------------------------------------------------------------------ pools, activations
def test_maxpool_ramp_negative_and_sizes():
    x = np.arange(7 * 7, dtype=np.float64).reshape(1, 7, 7, 1)
    y = ops.maxpool2d(x, 3, 2, 1)[0, :, :, 0]
    assert y.shape == (4, 4)
    # strictly increasing ramp: the bottom-right in-bounds tap wins
    want = np.array([[x[0, min(2 * p + 1, 6), min(2 * q + 1, 6), 0] for q in range(4)] for p in range(4)])
    assert np.array_equal(y, want)
    neg = -np.ones((1, 6, 6, 2)) - R.uniform(0, 1, (1, 6, 6, 2))
    yn = ops.maxpool2d(neg, 3, 2, 1)
    assert yn.max() < 0          # zero padding never selected
    xp = np.pad(neg, ((0, 0), (1, 1), (1, 1), (0, 0)), constant_values=-np.inf)
    win = sliding_window_view(xp, (3, 3), axis=(1, 2))[:, ::2, ::2]
    assert np.array_equal(yn, win.max(axis=(-1, -2)))


def test_gap_relu6():
    assert np.array_equal(ops.global_avg_pool(np.full((2, 7, 7, 5), 3.25)), np.full((2, 5), 3.25))
    x = R.standard_normal((1, 4, 4, 3))
    assert np.allclose(ops.global_avg_pool(x)[0], x.reshape(16, 3).mean(0))
    v = np.array([-1.0, -0.0, 0.0, 0.5, 6.0, 6.5, 100.0])
    assert np.array_equal(ops.relu6(v), [0, 0, 0, 0.5, 6, 6, 6])
    assert np.array_equal(ops.relu(v), [0, 0, 0, 0.5, 6, 6.5, 100])


def test_linear_is_1x1_conv_and_identity():
    x = R.standard_normal((3, 12))
    w = R.standard_normal((7, 12)).astype(np.float32)
    b = R.standard_normal(7)
    y = ops.linear(x, w, b)
    yc = ops.conv2d(x.reshape(3, 1, 1, 12), w.reshape(7, 12, 1, 1), b).reshape(3, 7)
    assert np.allclose(y, yc, rtol=1e-13, atol=1e-13)
    assert np.array_equal(ops.linear(x, np.eye(12)), x)


# ------------------------------------------------------------------ softmax, LN, GELU
def test_softmax_pins():
    x = R.standard_normal((5, 1000)) * 5
    p = ops.softmax(x)
    assert np.abs(p.sum(-1) - 1).max() < 1e-12
    assert np.allclose(p, ops.softmax(x + 123.0), rtol=1e-12)
    assert np.allclose(ops.softmax(np.full((2, 10), 7.0)), 0.1)
    assert np.array_equal(p.argmax(-1), x.argmax(-1))
    assert np.allclose(ops.softmax(np.log(np.array([[1.0, 2.0, 5.0]]))), [[0.125, 0.25, 0.625]])
    assert np.isfinite(ops.softmax(np.array([[1e4, 0.0]]))).all()
    assert ops.argmax_first(np.array([[1.0, 3.0, 3.0, 2.0]]))[0] == 1


def test_layernorm_pins():
    x = R.standard_normal((6, 768)) * 3 + 2
    y = ops.layernorm(x, np.ones(768), np.zeros(768))
    assert np.abs(y.mean(-1)).max() < 1e-12 and np.abs(y.var(-1) - 1).max() < 1e-9
    assert np.allclose(ops.layernorm(2.5 * x + 7.0, np.ones(768), np.zeros(768)), y, atol=1e-9)
    g, b = R.uniform(0.8, 1.2, 768), R.standard_normal(768)
    assert np.allclose(ops.layernorm(x, g, b), y * g + b)
    # two-element row: (x - mean)/std = +-1
    assert np.allclose(ops.layernorm(np.array([[1.0, 3.0]]), np.ones(2), np.zeros(2)), [[-1, 1]])


def test_gelu_pins():
    from math import erf, sqrt
    assert ops.gelu(np.array([0.0]))[0] == 0
    x = np.linspace(-6, 6, 101)
    assert np.allclose(ops.gelu(x) - ops.gelu(-x), x, atol=1e-14)
    assert abs(ops.gelu(np.array([10.0]))[0] - 10.0) < 1e-12 and abs(ops.gelu(np.array([-10.0]))[0]) < 1e-12
    # Phi(1) = 0.841344746068543 (standard normal CDF table)
    assert abs(ops.gelu(np.array([1.0]))[0] - 0.841344746068543) < 1e-13
    assert abs(ops.gelu(np.array([0.7]))[0] - 0.35 * (1 + erf(0.7 / sqrt(2)))) < 1e-15


# ------------------------------------------------------------------ attention
def test_attention_hand_worked():
    ln2 = np.log(2.0)
    q = np.array([[[np.sqrt(2) * ln2, 0], [0, 0], [0.3, -0.2], [9, 9]]])
    k = np.array([[[1.0, 0], [0, 0], [-1, 0], [50, 50]]])
    v = np.array([[[7.0, 0], [0, 7], [7, 7], [1e3, -1e3]]])
    out = ops.attention(q, k, v, np.array([3]), heads=1)
    assert np.allclose(out[0, 0], [5, 3], atol=1e-12)
    assert np.allclose(out[0, 1], [14 / 3, 14 / 3], atol=1e-12)


def test_attention_onehot_v_returns_probabilities():
    S, d = 8, 8
    q, k = R.standard_normal((1, S, d)), R.standard_normal((1, S, d))
    v = np.eye(S)[None]
    out = ops.attention(q, k, v, np.array([S]), heads=1)
    want = ops.softmax(q[0] @ k[0].T / np.sqrt(d))
    assert np.allclose(out[0], want, atol=1e-12)


def test_attention_equal_scores_mean_of_valid_values():
    S, hid, heads = 16, 32, 4
    q = np.zeros((2, S, hid)); k = R.standard_normal((2, S, hid)); v = R.standard_normal((2, S, hid))
    vl = np.array([5, 16])
    out = ops.attention(q, k, v, vl, heads)
    for b in range(2):
        assert np.allclose(out[b], np.broadcast_to(v[b, :vl[b]].mean(0), (S, hid)), atol=1e-12)


def test_attention_mask_and_permutation_invariance():
    S, hid, heads = 12, 24, 3
    q, k, v = (R.standard_normal((2, S, hid)) for _ in range(3))
    vl = np.array([7, 12])
    base = ops.attention(q, k, v, vl, heads)
    k2, v2 = k.copy(), v.copy()
    k2[0, 7:] = 1e3 * R.standard_normal((5, hid)); v2[0, 7:] = -1e3
    assert np.array_equal(ops.attention(q, k2, v2, vl, heads), base)       # padded keys never matter
    perm = R.permutation(7)
    k3, v3 = k.copy(), v.copy()
    k3[0, :7], v3[0, :7] = k[0, perm], v[0, perm]
    assert np.allclose(ops.attention(q, k3, v3, vl, heads)[0], base[0], atol=1e-12)
    # heads are independent: changing head 2's slice leaves heads 0,1 alone
    q4 = q.copy(); q4[..., 16:] += 1.0
    assert np.array_equal(ops.attention(q4, k, v, vl, heads)[..., :16], base[..., :16])
