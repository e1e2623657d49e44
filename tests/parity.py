"""Comparison rules shared by the GPU parity tests.

End-to-end bar (from the build's stated tolerance): max |gpu - oracle| over the pre-softmax
logits of the whole batch <= 2e-2 * max |oracle logit|; probabilities within 2e-2 absolute;
top-1 indices identical.  A sample whose oracle top-1/top-2 margin is below twice the measured
error is a numerical tie: there either of the oracle's two best classes is accepted, and the
number of such samples is reported.

Per-kernel bar: one fp16 rounding of the output (2^-11 relative) plus fp32 accumulation noise,
written as |err| <= 2^-10 |ref| + 1e-3 max|ref| -- an order of magnitude below the end-to-end
budget, so that a wrong tap, index or operand cannot hide in it.
"""
import numpy as np

E2E_REL = 2e-2


def check_logits(gpu_logits, ref_logits, gpu_top1, what=""):
    gpu_logits = np.asarray(gpu_logits, np.float64)
    scale = float(np.abs(ref_logits).max())
    err = float(np.abs(gpu_logits - ref_logits).max())
    assert np.isfinite(gpu_logits).all(), f"{what}: non-finite logits"
    assert err <= E2E_REL * scale, f"{what}: max|err| {err:.4e} > {E2E_REL} * {scale:.4e}"
    order = np.argsort(-ref_logits, axis=-1, kind="stable")
    best, second = order[..., 0], order[..., 1]
    margin = np.take_along_axis(ref_logits, best[..., None], -1)[..., 0] - np.take_along_axis(ref_logits, second[..., None], -1)[..., 0]
    ties = 0
    for i in range(len(best)):
        if gpu_top1[i] == best[i]:
            continue
        assert margin[i] < 2 * err and gpu_top1[i] == second[i], \
            f"{what}: sample {i} top-1 {gpu_top1[i]} != oracle {best[i]} (margin {margin[i]:.3e}, err {err:.3e})"
        ties += 1
    return err, scale, ties


def check_kernel(got, ref, what="", rel=2.0 ** -10, abs_rel=1e-3):
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, f"{what}: shape {got.shape} vs {ref.shape}"
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    tol = rel * np.abs(ref) + abs_rel * max(float(np.abs(ref).max()), 1e-30)
    bad = np.abs(got - ref) > tol
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} elements off; worst {np.abs(got - ref).max():.4e} (max|ref| {np.abs(ref).max():.4e})"
    return float(np.abs(got - ref).max())
