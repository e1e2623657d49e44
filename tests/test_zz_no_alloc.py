"""The GEMM entry point that allocates nothing (split-K workspace in a static device array) against the
allocating one: same kernels, so the outputs must agree bit for bit, on two calls in a row, the second smaller;
both are also held to the per-kernel bar against the CPU oracle."""
import numpy as np
import pytest

from oracle import ops
from parity import check_kernel

pytestmark = pytest.mark.gpu
R = np.random.default_rng(77)


def operands(torch, M, N, K, use_res):
    x = (R.standard_normal((M, K))).astype(np.float16)
    w = (R.standard_normal((N, K)) * K ** -0.5).astype(np.float16)
    b = (R.standard_normal(N) * 0.1).astype(np.float32)
    res = R.standard_normal((M, N)).astype(np.float16) if use_res else None
    ref = ops.linear(x, w, b)
    if use_res:
        ref = ref + res.astype(np.float64)
    dev = lambda a: None if a is None else torch.from_numpy(a).cuda()
    return dev(x), dev(w), dev(b), dev(res), ref


def test_gemm_noalloc_equals_gemm_two_calls_in_a_row():
    import torch
    import paper_2604_28175_amd as S
    assert torch.cuda.is_available()
    # (M, N, K, residual, fp32 out): split reductions (few tiles, long K) first large then smaller, then a product
    # that does not split at all
    for M, N, K, use_res, out_f32 in ((64, 1000, 2048, False, True), (5, 768, 3072, True, False),
                                      (8, 1000, 4096, False, True), (3, 64, 512, False, False),
                                      (128, 4096, 64, False, False)):
        x, w, b, res, ref = operands(torch, M, N, K, use_res)
        want = S.k_gemm(x, w, b, S.ACT_NONE, res, out_f32)
        y = torch.full((M, N), float("nan"), dtype=torch.float32 if out_f32 else torch.float16, device="cuda")
        before = torch.cuda.memory_allocated()
        S.k_gemm_noalloc(x, w, b, y, S.ACT_NONE, res, out_f32)
        assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        assert torch.equal(y, want), f"gemm_noalloc {M}x{N}x{K} differs from gemm"
        check_kernel(y.float().cpu().numpy(), ref, f"gemm_noalloc {M}x{N}x{K}")


def test_gemm_noalloc_rejects_sizes_beyond_its_workspace():
    import torch
    import paper_2604_28175_amd as S
    x = torch.zeros((129, 64), dtype=torch.float16, device="cuda")
    w = torch.zeros((4096, 64), dtype=torch.float16, device="cuda")
    y = torch.zeros((129, 4096), dtype=torch.float16, device="cuda")
    with pytest.raises(S.StraitError) as e:
        S.k_gemm_noalloc(x, w, None, y)
    assert e.value.status == S.E_SHAPE and "exceeds" in str(e.value)
