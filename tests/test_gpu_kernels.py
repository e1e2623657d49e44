"""GPU parity, kernel by kernel: each library kernel, called through the C ABI's kernel-level
entry points on the oracle's own operands, against the oracle's operator."""
import numpy as np
import pytest

from oracle import ops
from parity import check_kernel

pytestmark = pytest.mark.gpu
R = np.random.default_rng(20260428)


@pytest.fixture(scope="module")
def S():
    import torch
    import paper_2604_28175_amd as strait
    assert torch.cuda.is_available()
    strait.torch = torch
    return strait


def dev(S, a, dtype=None):
    t = S.torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def f16(a):
    return np.asarray(a).astype(np.float16)


def act_ref(y, act):
    return {0: y, 1: ops.relu(y), 2: ops.relu6(y), 3: ops.gelu(y)}[act]


CONV_CASES = [
    # N, H, W, C, K, R, stride, pad, act, residual, out_f32     (what it exercises)
    (2, 14, 14, 64, 64, 3, 1, 1, 1, False, False),      # gather path, exact tiles in K
    (3, 15, 13, 32, 96, 3, 2, 1, 1, False, False),      # stride 2, ragged M, ragged N tile
    (2, 9, 9, 16, 40, 3, 1, 1, 0, True, False),         # C = 16: a 32-wide slice straddles taps; residual
    (1, 10, 10, 24, 72, 3, 2, 1, 2, False, False),      # C = 24, ReLU6
    (2, 12, 12, 128, 256, 1, 1, 0, 1, True, False),     # 1x1 GEMM path + residual + ReLU
    (2, 12, 12, 64, 128, 1, 2, 0, 0, False, False),     # strided 1x1 (projection shortcut)
    (2, 20, 20, 3, 16, 7, 2, 3, 1, False, False),       # C = 3: scalar gather path, 7x7
    (1, 8, 8, 5, 10, 3, 1, 1, 0, False, False),         # odd C and K: scalar gather, direct epilogue
    (4, 1, 1, 64, 10, 1, 1, 0, 0, False, True),         # FC as 1x1 conv, fp32 logits
    (1, 40, 40, 64, 64, 3, 1, 1, 1, False, False),      # several 128-pixel tiles and a ragged tail (M = 1600)
    (1, 7, 7, 512, 512, 3, 1, 1, 1, False, False),      # long reduction (K = 4608), small M
    (11, 56, 56, 64, 256, 1, 1, 0, 1, True, False),     # 64 -> 256 pointwise with residual, M = 34496: many tiles, ragged tail, residual requested early
    # wide 3x3 stride-1 layers with enough output tiles not to split the reduction: the kernel that keeps an input patch in LDS
    (3, 56, 56, 64, 64, 3, 1, 1, 1, False, False),      # 64 channels out: 256-pixel tiles, two input slices
    (6, 28, 28, 32, 128, 3, 1, 1, 1, False, False),     # 128 channels out: 128-pixel tiles, a single input slice, smallest patch
    (1, 37, 112, 64, 128, 3, 1, 1, 0, False, False),    # wider rows (larger patch), ragged height, no activation
    (2, 24, 224, 32, 64, 3, 1, 1, 1, False, False),     # widest rows served: the largest patch
    (2, 40, 100, 96, 192, 3, 1, 1, 2, False, False),    # three channel tiles, three input slices, ReLU6
    # enough 256 x 128 tiles (768 or more) for the eight-wave form of that kernel, in both of its patch sizes
    (64, 56, 56, 32, 256, 3, 1, 1, 1, False, False),    # 1626 tiles, three patch transfers per wave, two channel tiles
    (16, 112, 112, 64, 128, 3, 1, 1, 1, False, False),  # rows cut into two strips of 56; two input slices
    (48, 64, 64, 32, 128, 3, 1, 1, 0, False, False),    # 64-pixel rows: four patch transfers per wave
    (12, 128, 128, 32, 128, 3, 1, 1, 2, False, False),  # two strips of 64: four transfers per wave with real pixels on the strips' sides
    # 64 channels out, at most 128 in and 1024 or more 256-pixel tiles: workgroups that walk over several tiles each
    (81, 56, 56, 64, 64, 3, 1, 1, 1, False, False),     # 1028 tiles, two input slices
    (24, 112, 112, 32, 64, 3, 1, 1, 2, False, False),   # one slice: every slice is a tile's last; rows in two strips
    (320, 28, 28, 128, 64, 3, 1, 1, 0, False, False),   # four slices
    # few tiles and a reduction worth splitting two to eight ways: two groups of wavefronts in one workgroup, half the slices each
    (8, 14, 14, 1024, 256, 1, 1, 0, 1, False, False),   # pointwise, 64-wide slices, 16 of them
    (2, 14, 14, 512, 256, 1, 1, 0, 1, True, False),     # pointwise with residual
    (8, 14, 14, 256, 256, 3, 1, 1, 1, False, False),    # 3x3: 72 slices of 32
    (1, 10, 10, 264, 64, 1, 1, 0, 0, False, False),     # nine 32-wide slices, the last one ragged: the second group's fifth slice is empty
    (3, 9, 9, 160, 96, 3, 2, 1, 2, False, False),       # stride 2, ragged tiles in both directions, 45 slices
]


@pytest.mark.parametrize("case", CONV_CASES, ids=lambda c: "x".join(map(str, c[:8])))
def test_conv2d(S, case):
    N, H, W, C, K, Rk, stride, pad, act, use_res, out_f32 = case
    x = f16(R.standard_normal((N, H, W, C)))
    w = f16(R.standard_normal((K, C, Rk, Rk)) * (2.0 / (C * Rk * Rk)) ** 0.5)
    b = R.standard_normal(K).astype(np.float32)
    ref = ops.conv2d(x, w, b, stride, pad)
    res = f16(R.standard_normal(ref.shape)) if use_res else None
    if use_res:
        ref = ref + res.astype(np.float64)
    ref = act_ref(ref, act)
    w_krsc = np.ascontiguousarray(np.transpose(w, (0, 2, 3, 1)))
    y = S.k_conv2d(dev(S, x), dev(S, w_krsc), dev(S, b), stride, pad, act, None if res is None else dev(S, res), out_f32)
    S.torch.cuda.synchronize()
    check_kernel(y.float().cpu().numpy(), ref, f"conv {case}")


def test_conv2d_split_in_the_workgroup_integer_data_is_bit_exact(S):
    """The reduction split over two groups of wavefronts of one workgroup (few tiles, 9 to 32 slices), pointwise and 3x3:
    exact on integer data, partial sums and their hand-over included."""
    for (N, H, W, C, K, Rk, stride, pad) in ((4, 14, 14, 512, 128, 1, 1, 0), (1, 10, 10, 264, 64, 1, 1, 0), (2, 14, 14, 96, 64, 3, 1, 1)):
        x = R.integers(-2, 3, (N, H, W, C)).astype(np.float16)
        w = (R.integers(-1, 2, (K, C, Rk, Rk)) * (R.random((K, C, Rk, Rk)) < 0.2)).astype(np.float16)
        b = R.integers(-5, 6, K).astype(np.float32)
        ref = ops.conv2d(x, w, b, stride, pad)
        assert np.abs(ref).max() < 2048
        y = S.k_conv2d(dev(S, x), dev(S, np.ascontiguousarray(np.transpose(w, (0, 2, 3, 1)))), dev(S, b), stride, pad)
        assert np.array_equal(y.float().cpu().numpy().astype(np.float64), ref), (N, H, W, C, K, Rk)


def test_conv2d_integer_data_is_bit_exact(S):
    """Small integers are exact in fp16 and fp32, so the GPU must reproduce the oracle exactly."""
    x = R.integers(-3, 4, (2, 11, 9, 16)).astype(np.float16)
    w = R.integers(-2, 3, (24, 16, 3, 3)).astype(np.float16)
    b = R.integers(-5, 6, 24).astype(np.float32)
    for stride in (1, 2):
        ref = ops.conv2d(x, w, b, stride, 1)
        assert np.abs(ref).max() < 2048
        y = S.k_conv2d(dev(S, x), dev(S, np.ascontiguousarray(np.transpose(w, (0, 2, 3, 1)))), dev(S, b), stride, 1)
        assert np.array_equal(y.float().cpu().numpy().astype(np.float64), ref)


@pytest.mark.parametrize("N,H,W,C,K", [(4, 40, 60, 32, 64),      # 256-pixel tiles, one strip per row
                                       (2, 36, 128, 32, 128),    # rows cut into two strips of 64: the strips' side borders are real pixels
                                       (1, 29, 224, 64, 64),     # four strips of 56, two input slices
                                       (40, 15, 14, 32, 64),     # the narrowest rows served, odd height: shared borders everywhere
                                       (30, 19, 17, 32, 128),    # odd width and height
                                       (2, 70, 65, 32, 64),      # an odd width above 64 stays one strip
                                       (2, 40, 130, 32, 64),     # two strips of odd width 65
                                       (3, 21, 200, 32, 64),     # four strips of 50
                                       # the eight-wave 256 x 128 tile (768 tiles or more): three and four patch transfers per wave
                                       (64, 56, 56, 32, 256), (16, 112, 112, 32, 128), (48, 64, 64, 32, 128), (12, 128, 128, 64, 128),
                                       # workgroups that walk over tiles (64 channels out, 1024 tiles or more): two slices, one slice,
                                       # three slices (the patch buffers swap roles from tile to tile), two strips of odd width 65
                                       (81, 56, 56, 64, 64), (72, 60, 60, 32, 64), (300, 30, 30, 96, 64), (50, 40, 130, 32, 64),
                                       (6, 224, 224, 64, 64)])   # and four strips of 56
def test_conv2d_wide_3x3_integer_data_is_bit_exact(S, N, H, W, C, K):
    """The wide 3x3 stride-1 layers run from an input patch in LDS, addressed through the bordered image: with
    integer data every border, strip seam and tile seam must come out exactly."""
    x = R.integers(-3, 4, (N, H, W, C)).astype(np.float16)
    w = R.integers(-2, 3, (K, C, 3, 3)).astype(np.float16)
    b = R.integers(-5, 6, K).astype(np.float32)
    ref = ops.conv2d(x, w, b, 1, 1)
    assert np.abs(ref).max() < 2048
    y = S.k_conv2d(dev(S, x), dev(S, np.ascontiguousarray(np.transpose(w, (0, 2, 3, 1)))), dev(S, b), 1, 1)
    assert np.array_equal(y.float().cpu().numpy().astype(np.float64), ref)


def test_conv2d_tap_count_pattern(S):
    y = S.k_conv2d(dev(S, np.ones((1, 6, 6, 8), np.float16)), dev(S, np.ones((8, 3, 3, 8), np.float16)), None, 2, 1)
    got = y.float().cpu().numpy()[0, :, :, 0] / 8
    cnt = lambda i: sum(0 <= 2 * i + r - 1 < 6 for r in range(3))
    assert np.array_equal(got, [[cnt(i) * cnt(j) for j in range(3)] for i in range(3)])


@pytest.mark.parametrize("M,N,K,act,use_res,out_f32", [(256, 768, 768, 0, True, False), (130, 3072, 768, 3, False, False),
                                                        (64, 768, 3072, 0, True, False), (5, 1000, 2048, 0, False, True),
                                                        (300, 2304, 768, 0, False, False)])
def test_gemm(S, M, N, K, act, use_res, out_f32):
    x = f16(R.standard_normal((M, K)))
    w = f16(R.standard_normal((N, K)) * K ** -0.5)
    b = (R.standard_normal(N) * 0.1).astype(np.float32)
    ref = ops.linear(x, w, b)
    res = f16(R.standard_normal(ref.shape)) if use_res else None
    if use_res:
        ref = ref + res.astype(np.float64)
    ref = act_ref(ref, act)
    y = S.k_gemm(dev(S, x), dev(S, w), dev(S, b), act, None if res is None else dev(S, res), out_f32)
    check_kernel(y.float().cpu().numpy(), ref, f"gemm {M}x{N}x{K}")


@pytest.mark.parametrize("M,K1,N1,N2,use_res", [(9001, 64, 256, 64, True),       # many 32-pixel tiles and a ragged tail
                                                 (5000, 64, 256, 128, True),      # the seam into the next stage: twice as wide
                                                 (70, 64, 256, 64, True),         # fewer tiles than one workgroup has wavefronts
                                                 (97001, 64, 256, 64, True),      # every wavefront of the full grid walks over several tiles
                                                 (70003, 64, 256, 128, True)])
def test_pointwise_pair(S, M, K1, N1, N2, use_res):
    """y = relu(x W3^T + b3 + res), z = relu(fp16(y) W1^T + b1) in one launch: against the oracle's operators, and bit
    for bit against the same two layers as two launches."""
    x = f16(R.standard_normal((M, K1)))
    w3 = f16(R.standard_normal((N1, K1)) * (0.5 / K1) ** 0.5)
    b3 = (R.standard_normal(N1) * 0.1).astype(np.float32)
    res = f16(R.standard_normal((M, N1))) if use_res else None
    w1 = f16(R.standard_normal((N2, N1)) * (2.0 / N1) ** 0.5)
    b1 = (R.standard_normal(N2) * 0.1).astype(np.float32)
    y_ref = ops.linear(x, w3, b3)
    if use_res:
        y_ref = y_ref + res.astype(np.float64)
    y_ref = ops.relu(y_ref)
    z_ref = ops.relu(ops.linear(y_ref.astype(np.float16), w1, b1))      # the second layer reads the fp16 tensor
    dx, dw3, db3, dw1, db1 = dev(S, x), dev(S, w3), dev(S, b3), dev(S, w1), dev(S, b1)
    dres = None if res is None else dev(S, res)
    y, z = S.k_pointwise_pair(dx, dw3, db3, dres, dw1, db1)
    S.torch.cuda.synchronize()
    check_kernel(y.float().cpu().numpy(), y_ref, f"pair y {M}x{K1}x{N1}")
    check_kernel(z.float().cpu().numpy(), z_ref, f"pair z {M}x{N1}x{N2}", rel=2.0 ** -9)
    y2 = S.k_gemm(dx, dw3, db3, S.ACT_RELU, dres)
    assert S.torch.equal(y, y2)
    if -(-M // 64) * -(-N2 // 64) > 256:   # (with fewer tiles the stand-alone kernel splits its reduction and adds in another order)
        assert S.torch.equal(z, S.k_gemm(y2, dw1, db1, S.ACT_RELU))


def test_pointwise_pair_integer_data_is_bit_exact(S):
    M, K1, N1, N2 = 777, 64, 256, 64
    x = R.integers(-2, 3, (M, K1)).astype(np.float16)
    w3 = R.integers(-1, 2, (N1, K1)).astype(np.float16)
    b3 = R.integers(-3, 4, N1).astype(np.float32)
    res = R.integers(-4, 5, (M, N1)).astype(np.float16)
    w1 = (R.integers(-1, 2, (N2, N1)) * (R.random((N2, N1)) < 0.1)).astype(np.float16)     # sparse: sums stay exact in fp16
    b1 = R.integers(-3, 4, N2).astype(np.float32)
    y_ref = ops.relu(ops.linear(x, w3, b3) + res.astype(np.float64))
    z_ref = ops.relu(ops.linear(y_ref, w1, b1))
    assert np.abs(y_ref).max() < 2048 and np.abs(z_ref).max() < 2048
    y, z = S.k_pointwise_pair(dev(S, x), dev(S, w3), dev(S, b3), dev(S, res), dev(S, w1), dev(S, b1))
    assert np.array_equal(y.float().cpu().numpy().astype(np.float64), y_ref)
    assert np.array_equal(z.float().cpu().numpy().astype(np.float64), z_ref)


def test_pointwise_pair_rejects_other_shapes(S):
    t = S.torch.zeros((256, 96), dtype=S.torch.float16, device="cuda")
    w3 = S.torch.zeros((256, 96), dtype=S.torch.float16, device="cuda")
    w1 = S.torch.zeros((64, 256), dtype=S.torch.float16, device="cuda")
    res = S.torch.zeros((256, 256), dtype=S.torch.float16, device="cuda")
    with pytest.raises(S.StraitError) as e:
        S.k_pointwise_pair(t, w3, None, res, w1, None)             # 96 input channels
    assert e.value.status == S.E_SHAPE
    with pytest.raises(S.StraitError) as e:
        S.k_pointwise_pair(S.torch.zeros((256, 128), dtype=S.torch.float16, device="cuda"),
                           S.torch.zeros((512, 128), dtype=S.torch.float16, device="cuda"), None,
                           S.torch.zeros((256, 512), dtype=S.torch.float16, device="cuda"),
                           S.torch.zeros((128, 512), dtype=S.torch.float16, device="cuda"), None)   # weights that do not fit in LDS
    assert e.value.status == S.E_SHAPE
    with pytest.raises(S.StraitError) as e:
        S.k_pointwise_pair(t[:, :64].contiguous(), w3[:, :64].contiguous(), None, None, w1, None)   # no residual tensor
    assert e.value.status == S.E_INVALID


@pytest.mark.parametrize("N,P,Q,C,H2,W2,K2,s2,Cout", [(2, 14, 14, 128, 28, 28, 256, 2, 512),      # few tiles: the reduction is split
                                                        (16, 28, 28, 128, 56, 56, 256, 2, 512),    # 128-wide tiles
                                                        (3, 7, 7, 512, 14, 14, 1024, 2, 2048),     # ragged rows, long second part
                                                        (5, 8, 9, 64, 15, 17, 64, 2, 256),         # odd second tensor
                                                        (4, 20, 20, 64, 20, 20, 64, 1, 256),       # stride 1
                                                        (44, 28, 28, 128, 56, 56, 256, 2, 512)])   # enough tiles for the 256 x 128 shape
def test_conv1x1_proj(S, N, P, Q, C, H2, W2, K2, s2, Cout):
    """A pointwise convolution with a subsampling pointwise projection of a second tensor inside its reduction, against
    the oracle's two convolutions added in fp64."""
    x = f16(R.standard_normal((N, P, Q, C)))
    x2 = f16(R.standard_normal((N, H2, W2, K2)))
    w3 = f16(R.standard_normal((Cout, C)) * (0.5 / C) ** 0.5)
    wd = f16(R.standard_normal((Cout, K2)) * (0.5 / K2) ** 0.5)
    bias = (R.standard_normal(Cout) * 0.1).astype(np.float32)
    sub = x2[:, ::s2, ::s2][:, :P, :Q]
    ref = ops.relu(ops.linear(x, w3, None) + ops.linear(sub, wd, None) + bias.astype(np.float64))
    wcat = np.ascontiguousarray(np.concatenate([w3, wd], axis=1))
    y = S.k_conv1x1_proj(dev(S, x), dev(S, x2), s2, dev(S, wcat), dev(S, bias), S.ACT_RELU)
    check_kernel(y.float().cpu().numpy(), ref, f"conv1x1+proj {N}x{P}x{Q}x{C}+{K2}->{Cout}")


def test_conv1x1_proj_integer_data_and_errors(S):
    N, P, Q, C, K2, Cout = 3, 9, 10, 64, 128, 72
    x = R.integers(-2, 3, (N, P, Q, C)).astype(np.float16)
    x2 = R.integers(-2, 3, (N, 2 * P, 2 * Q, K2)).astype(np.float16)
    wcat = (R.integers(-1, 2, (Cout, C + K2)) * (R.random((Cout, C + K2)) < 0.5)).astype(np.float16)
    bias = R.integers(-3, 4, Cout).astype(np.float32)
    ref = ops.linear(np.concatenate([x, x2[:, ::2, ::2]], axis=-1), wcat, bias)
    assert np.abs(ref).max() < 2048
    y = S.k_conv1x1_proj(dev(S, x), dev(S, x2), 2, dev(S, wcat), dev(S, bias))
    assert np.array_equal(y.float().cpu().numpy().astype(np.float64), ref)
    with pytest.raises(S.StraitError) as e:                      # a first part that is not whole 64-wide slices
        S.k_conv1x1_proj(dev(S, x[..., :32].copy()), dev(S, x2), 2, dev(S, wcat[:, 32:].copy()), dev(S, bias))
    assert e.value.status == S.E_SHAPE
    with pytest.raises(S.StraitError) as e:                      # second tensor too small for the last output pixel
        S.k_conv1x1_proj(dev(S, x), dev(S, x2[:, :2 * P - 2].copy()), 2, dev(S, wcat), dev(S, bias))
    assert e.value.status == S.E_SHAPE


@pytest.mark.parametrize("M", [9001, 70, 97001])
def test_pointwise_pair_proj(S, M):
    """The pair whose shortcut is a 1x1 projection of a second tensor: y = relu(x W3^T + x2 Wd^T + b3 + bd) with the two
    products in one reduction, z = relu(fp16(y) W1^T + b1): against the oracle's operators, and bit for bit against one
    product over the concatenated inputs."""
    K1 = K2 = 64; N1, N2 = 256, 64
    x, x2 = f16(R.standard_normal((M, K1))), f16(R.standard_normal((M, K2)))
    w3 = f16(R.standard_normal((N1, K1)) * (0.5 / K1) ** 0.5)
    wd = f16(R.standard_normal((N1, K2)) * (0.5 / K2) ** 0.5)
    b3 = (R.standard_normal(N1) * 0.1).astype(np.float32)
    bd = (R.standard_normal(N1) * 0.1).astype(np.float32)
    w1 = f16(R.standard_normal((N2, N1)) * (2.0 / N1) ** 0.5)
    b1 = (R.standard_normal(N2) * 0.1).astype(np.float32)
    bsum = b3 + bd
    y_ref = ops.relu(ops.linear(x, w3, None) + ops.linear(x2, wd, None) + bsum.astype(np.float64))
    z_ref = ops.relu(ops.linear(y_ref.astype(np.float16), w1, b1))
    wcat = np.ascontiguousarray(np.concatenate([w3, wd], axis=1))
    dx, dx2, dw, db, dw1, db1 = dev(S, x), dev(S, x2), dev(S, wcat), dev(S, bsum), dev(S, w1), dev(S, b1)
    y, z = S.k_pointwise_pair_proj(dx, dx2, dw, db, dw1, db1)
    S.torch.cuda.synchronize()
    check_kernel(y.float().cpu().numpy(), y_ref, f"pair-proj y {M}")
    check_kernel(z.float().cpu().numpy(), z_ref, f"pair-proj z {M}", rel=2.0 ** -9)
    if M * N1 > 128 * 4096:           # (below that the stand-alone kernel splits its reduction and adds in another order)
        xcat = S.torch.cat([dx, dx2], dim=1).contiguous()
        assert S.torch.equal(y, S.k_gemm(xcat, dw, db, S.ACT_RELU))


def test_pointwise_pair_proj_integer_data_and_errors(S):
    M, N1, N2 = 777, 256, 64
    x = R.integers(-2, 3, (M, 64)).astype(np.float16)
    x2 = R.integers(-2, 3, (M, 64)).astype(np.float16)
    wcat = R.integers(-1, 2, (N1, 128)).astype(np.float16)
    b = R.integers(-3, 4, N1).astype(np.float32)
    w1 = (R.integers(-1, 2, (N2, N1)) * (R.random((N2, N1)) < 0.1)).astype(np.float16)     # sparse: sums stay exact in fp16
    b1 = R.integers(-3, 4, N2).astype(np.float32)
    y_ref = ops.relu(ops.linear(np.concatenate([x, x2], axis=1), wcat, b))
    z_ref = ops.relu(ops.linear(y_ref, w1, b1))
    assert np.abs(y_ref).max() < 2048 and np.abs(z_ref).max() < 2048
    y, z = S.k_pointwise_pair_proj(dev(S, x), dev(S, x2), dev(S, wcat), dev(S, b), dev(S, w1), dev(S, b1))
    assert np.array_equal(y.float().cpu().numpy().astype(np.float64), y_ref)
    assert np.array_equal(z.float().cpu().numpy().astype(np.float64), z_ref)
    with pytest.raises(S.StraitError) as e:                      # the next stage's 128 channels do not fit beside the wider weights
        S.k_pointwise_pair_proj(dev(S, x), dev(S, x2), dev(S, wcat), dev(S, b), S.torch.zeros((128, 256), dtype=S.torch.float16, device="cuda"), None)
    assert e.value.status == S.E_SHAPE
    with pytest.raises(S.StraitError) as e:
        S.k_pointwise_pair_proj(dev(S, x), None, dev(S, wcat), dev(S, b), dev(S, w1), dev(S, b1))
    assert e.value.status == S.E_INVALID


@pytest.mark.parametrize("N,H,W,C,stride", [(2, 14, 14, 96, 1), (2, 15, 13, 144, 2), (1, 7, 7, 960, 1), (3, 28, 28, 32, 2), (1, 9, 10, 8, 1),
                                            # stride 1 with enough work for the column kernel: few channels, ragged height, many channels
                                            (6, 56, 56, 32, 1), (5, 30, 27, 144, 1), (16, 7, 7, 960, 1)])
def test_dwconv3x3(S, N, H, W, C, stride):
    x = f16(R.standard_normal((N, H, W, C)) * 2)
    w = f16(R.standard_normal((C, 1, 3, 3)) * 0.47)
    b = R.standard_normal(C).astype(np.float32)
    ref = ops.relu6(ops.dwconv2d(x, w, b, stride, 1))
    w_rsc = np.ascontiguousarray(np.transpose(w[:, 0], (1, 2, 0)))
    y = S.k_dwconv3x3(dev(S, x), dev(S, w_rsc), dev(S, b), stride, S.ACT_RELU6)
    check_kernel(y.float().cpu().numpy(), ref, "dwconv")
    assert (ref == 6).any() and (ref == 0).any()


def test_pools_bit_exact_and_avg(S):
    x = f16(R.standard_normal((2, 13, 12, 64)) - 3.0)      # mostly negative: padding must never win
    y = S.k_maxpool3x3s2(dev(S, x))
    assert np.array_equal(y.cpu().numpy().astype(np.float64), ops.maxpool2d(x, 3, 2, 1))
    g = S.k_global_avgpool(dev(S, x))
    check_kernel(g.float().cpu().numpy(), ops.global_avg_pool(x.astype(np.float64)), "gap")
    c = S.k_global_avgpool(dev(S, np.full((1, 7, 7, 8), 3.25, np.float16)))
    assert np.array_equal(c.cpu().numpy(), np.full((1, 8), 3.25, np.float16))


@pytest.mark.parametrize("rows,n", [(4, 10), (33, 1000), (1, 7), (5, 64)])
def test_softmax_top1(S, rows, n):
    x = (R.standard_normal((rows, n)) * 4).astype(np.float32)
    x[0, min(3, n - 1)] = x[0].max() + 1.0
    x[-1, 0] = x[-1, n - 1] = x[-1].max() + 2.0             # exact tie: lowest index wins
    p, t = S.k_softmax_top1(dev(S, x))
    ref = ops.softmax(x)
    assert np.abs(p.cpu().numpy() - ref).max() < 1e-5
    assert np.abs(p.cpu().numpy().sum(-1) - 1).max() < 1e-5
    assert np.array_equal(t.cpu().numpy(), ops.argmax_first(x))
    assert t.cpu().numpy()[-1] == 0


@pytest.mark.parametrize("rows,n", [(7, 768), (130, 768), (3, 64), (2, 3072), (5, 256), (13, 512), (9, 1024)])
def test_layernorm(S, rows, n):
    x = f16(R.standard_normal((rows, n)) * 3 + 1)
    g = R.uniform(0.8, 1.2, n).astype(np.float32)
    b = (R.standard_normal(n) * 0.02).astype(np.float32)
    y = S.k_layernorm(dev(S, x), dev(S, g), dev(S, b), 1e-12)
    check_kernel(y.float().cpu().numpy(), ops.layernorm(x, g, b, 1e-12), "layernorm")


@pytest.mark.parametrize("B,Sq,heads,lens", [(3, 128, 12, (128, 32, 77)), (2, 64, 2, (64, 5)), (4, 32, 1, (1, 16, 31, 32)),
                                             (2, 128, 4, (33, 100)),
                                             # lengths that are no multiple of the 32-row blocks, and more than 128 keys
                                             (3, 197, 12, (197, 197, 150)), (2, 37, 2, (37, 20)), (3, 17, 1, (17, 1, 16)),
                                             (2, 256, 2, (256, 129)), (2, 129, 3, (129, 128)), (2, 255, 1, (255, 97))])
def test_attention(S, B, Sq, heads, lens):
    hid = heads * 64
    qkv = f16(R.standard_normal((B, Sq, 3 * hid)))
    vl = np.array(lens, np.int32)
    ref = ops.attention(qkv[..., :hid], qkv[..., hid:2 * hid], qkv[..., 2 * hid:], vl, heads)
    out = S.k_attention(dev(S, qkv), dev(S, vl), heads).float().cpu().numpy()
    for b in range(B):
        L = int(vl[b])
        check_kernel(out[b, :L], ref[b, :L], f"attention seq {b}", rel=2.0 ** -9, abs_rel=2e-3)
        assert np.isfinite(out[b]).all()
    # padded keys never matter: scribble over them (including non-finite values) and compare bit for bit
    qkv2 = qkv.copy()
    for b in range(B):
        qkv2[b, vl[b]:, hid:] = np.float16(np.inf)
    out2 = S.k_attention(dev(S, qkv2), dev(S, vl), heads).float().cpu().numpy()
    for b in range(B):
        assert np.array_equal(out2[b, :vl[b]], out[b, :vl[b]])


def stem_pool_weights(w_oihw):
    """[64,3,7,7] -> the fused stem kernel's [64][176] layout (strait.h, strait_k_stem_pool)."""
    wf = np.zeros((64, 22 * 8), np.float16)
    for r in range(7):
        for s in range(7):
            for c in range(3):
                wf[:, r * 24 + 1 + s * 3 + c] = w_oihw[:, c, r, s]
    return wf


@pytest.mark.parametrize("n,h,w", [(2, 64, 64), (1, 224, 224), (3, 50, 38), (2, 7, 8), (1, 33, 66), (2, 1, 2), (1, 130, 226)])
def test_stem_pool(S, n, h, w):
    x = f16(R.standard_normal((n, h, w, 3)))
    wt = f16(R.standard_normal((64, 3, 7, 7)) * (2.0 / 147) ** 0.5)
    b = (R.standard_normal(64) * 0.5).astype(np.float32)
    ref = ops.maxpool2d(ops.relu(ops.conv2d(x, wt, b, 2, 3)), 3, 2, 1)
    y = S.k_stem_pool(dev(S, x), dev(S, stem_pool_weights(wt)), dev(S, b)).float().cpu().numpy()
    assert y.shape == ref.shape
    check_kernel(y, ref, f"stem+pool {n}x{h}x{w}")


def stem3_weights(w_oihw):
    """[K,3,3,3] -> the direct 3x3/2 stem's [32][48] layout (strait.h, strait_k_stem3x3s2)."""
    wf = np.zeros((32, 48), np.float16)
    k = w_oihw.shape[0]
    for r in range(3):
        for s in range(3):
            for c in range(3):
                wf[:k, r * 16 + 1 + s * 3 + c] = w_oihw[:, c, r, s]
    return wf


@pytest.mark.parametrize("n,h,w,k,act", [(2, 64, 64, 32, 2), (1, 224, 224, 32, 2), (3, 51, 38, 32, 1), (2, 7, 8, 16, 0), (1, 33, 66, 24, 2),
                                         (2, 1, 2, 8, 0), (1, 130, 226, 32, 2), (5, 18, 130, 32, 2), (40, 96, 96, 32, 2)])
def test_stem3x3s2(S, n, h, w, k, act):
    x = f16(R.standard_normal((n, h, w, 3)))
    wt = f16(R.standard_normal((k, 3, 3, 3)) * (2.0 / 27) ** 0.5)
    b = (R.standard_normal(k) * 0.5).astype(np.float32)
    ref = act_ref(ops.conv2d(x, wt, b, 2, 1), act)
    y = S.k_stem3x3s2(dev(S, x), dev(S, stem3_weights(wt)), dev(S, b), k, act=act).float().cpu().numpy()
    assert y.shape == ref.shape
    check_kernel(y, ref, f"stem 3x3/2 {n}x{h}x{w}->{k}")


def test_stem3x3s2_integer_data_and_errors(S):
    # small integers: every product and partial sum is exact in fp16 and fp32, so any order of summation gives the same bits
    x = R.integers(-3, 4, (3, 45, 70, 3)).astype(np.float16)
    wt = R.integers(-2, 3, (32, 3, 3, 3)).astype(np.float16)
    b = R.integers(-4, 5, 32).astype(np.float32)
    y = S.k_stem3x3s2(dev(S, x), dev(S, stem3_weights(wt)), dev(S, b), 32, act=2).float().cpu().numpy()
    assert np.array_equal(y, ops.relu6(ops.conv2d(x, wt, b, 2, 1)))
    with pytest.raises(S.StraitError):       # odd width
        S.k_stem3x3s2(dev(S, x[:, :, :69]), dev(S, stem3_weights(wt)), dev(S, b), 32)
    with pytest.raises(S.StraitError):       # a channel count the kernel does not take
        S.k_stem3x3s2(dev(S, x), dev(S, stem3_weights(wt)), dev(S, b), 12)


@pytest.mark.parametrize("n,h,w", [(2, 64, 64), (1, 224, 224), (3, 51, 38), (2, 7, 8), (2, 1, 2), (1, 130, 226), (5, 18, 122), (40, 96, 96)])
def test_stem3x3s2_dw(S, n, h, w):
    """Stem 3x3/2 (3 -> 32) + depthwise 3x3 as one launch: against the oracle's two operators, and bit for bit against the
    two stand-alone kernels."""
    x = f16(R.standard_normal((n, h, w, 3)))
    wt = f16(R.standard_normal((32, 3, 3, 3)) * (2.0 / 27) ** 0.5)
    b = (R.standard_normal(32) * 0.5).astype(np.float32)
    wd = f16(R.standard_normal((32, 1, 3, 3)) * 0.47)
    bd = R.standard_normal(32).astype(np.float32)
    ref = ops.relu6(ops.dwconv2d(ops.relu6(ops.conv2d(x, wt, b, 2, 1)), wd, bd, 1, 1))
    wf_d, wd_d = dev(S, stem3_weights(wt)), dev(S, np.ascontiguousarray(np.transpose(wd[:, 0], (1, 2, 0))))
    y = S.k_stem3x3s2_dw(dev(S, x), wf_d, dev(S, b), wd_d, dev(S, bd))
    y2 = S.k_dwconv3x3(S.k_stem3x3s2(dev(S, x), wf_d, dev(S, b), 32, act=2), wd_d, dev(S, bd), 1, 2)
    S.torch.cuda.synchronize()
    assert tuple(y.shape) == ref.shape
    assert S.torch.equal(y, y2), f"fused differs from the two launches {n}x{h}x{w}"
    check_kernel(y.float().cpu().numpy(), ref, f"stem + dw {n}x{h}x{w}")
    with pytest.raises(S.StraitError):       # odd width
        S.k_stem3x3s2_dw(dev(S, x[:, :, :w - 1]), wf_d, dev(S, b), wd_d, dev(S, bd))


EXPAND_DW_CASES = [
    # N, H, W, Cin, Chid, stride      (MobileNetV2's blocks at their real shapes, then ragged ones)
    (2, 112, 112, 16, 96, 2), (2, 56, 56, 24, 144, 1), (2, 56, 56, 24, 144, 2), (3, 28, 28, 32, 192, 1), (3, 28, 28, 32, 192, 2),
    (4, 14, 14, 64, 384, 1), (4, 14, 14, 96, 576, 1), (4, 14, 14, 96, 576, 2), (5, 7, 7, 160, 960, 1),
    (2, 15, 13, 40, 88, 1),       # 40 input channels in a 64-wide reduction, 88 = 2 groups of 32 and 24 channels, odd image
    (1, 9, 10, 8, 8, 2),          # one group with 8 channels, the smallest of everything
    (2, 37, 45, 48, 200, 2),      # stride 2 with ragged tiles in both directions, a ragged last group
    (70, 14, 14, 64, 384, 1),     # enough tiles that a workgroup takes all twelve groups
    (1, 20, 70, 160, 64, 2),      # 160 input channels at stride 2: only the smallest tile fits LDS
]


@pytest.mark.parametrize("case", EXPAND_DW_CASES, ids=lambda c: "x".join(map(str, c)))
def test_expand_dw(S, case):
    """1x1 expansion + depthwise 3x3 as one launch: against the oracle's two operators, and bit for bit against the two
    stand-alone kernels."""
    N, H, W, Cin, Chid, stride = case
    x = f16(R.standard_normal((N, H, W, Cin)))
    w1 = f16(R.standard_normal((Chid, Cin, 1, 1)) * (2.0 / Cin) ** 0.5)
    b1 = R.standard_normal(Chid).astype(np.float32)
    wd = f16(R.standard_normal((Chid, 1, 3, 3)) * 0.47)
    bd = R.standard_normal(Chid).astype(np.float32)
    hid = ops.relu6(ops.conv2d(x, w1, b1, 1, 0))
    ref = ops.relu6(ops.dwconv2d(hid, wd, bd, stride, 1))
    w1_d = dev(S, np.ascontiguousarray(w1[:, :, 0, 0]))
    wd_d = dev(S, np.ascontiguousarray(np.transpose(wd[:, 0], (1, 2, 0))))
    y = S.k_expand_dw(dev(S, x), w1_d, dev(S, b1), wd_d, dev(S, bd), stride)
    t = S.k_conv2d(dev(S, x), w1_d.reshape(Chid, 1, 1, Cin), dev(S, b1), 1, 0, 2)
    y2 = S.k_dwconv3x3(t, wd_d, dev(S, bd), stride, 2)
    S.torch.cuda.synchronize()
    assert tuple(y.shape) == ref.shape
    assert S.torch.equal(y, y2), f"fused differs from the two launches {case}"
    check_kernel(y.float().cpu().numpy(), ref, f"expand+dw {case}")


def test_expand_dw_errors(S):
    x = dev(S, np.zeros((1, 8, 8, 12), np.float16))
    with pytest.raises(S.StraitError):       # Cin % 8 != 0
        S.k_expand_dw(x, dev(S, np.zeros((16, 12), np.float16)), None, dev(S, np.zeros((3, 3, 16), np.float16)), None, 1)
    x = dev(S, np.zeros((1, 8, 8, 16), np.float16))
    with pytest.raises(S.StraitError):       # stride 3
        S.k_expand_dw(x, dev(S, np.zeros((16, 16), np.float16)), None, dev(S, np.zeros((3, 3, 16), np.float16)), None, 3)


@pytest.mark.parametrize("n,h,w,c", [(2, 8, 6, 16), (3, 14, 14, 512), (1, 224, 224, 64)])
def test_maxpool2x2(S, n, h, w, c):
    x = f16(R.standard_normal((n, h, w, c)))
    y = S.k_maxpool2x2s2(dev(S, x)).float().cpu().numpy()
    assert np.array_equal(y, ops.maxpool2d(x, 2, 2, 0))          # selection only: bit-exact


@pytest.mark.parametrize("n,t,d", [(2, 9, 64), (3, 196, 768)])
def test_vit_tokens(S, n, t, d):
    patch = f16(R.standard_normal((n, t, d)))
    cls = f16(R.standard_normal(d) * 0.02).astype(np.float32)
    pos = f16(R.standard_normal((t + 1, d)) * 0.02).astype(np.float32)
    z = S.k_vit_tokens(dev(S, patch), dev(S, cls), dev(S, pos)).float().cpu().numpy()
    ref = np.concatenate([np.broadcast_to(cls.astype(np.float64), (n, 1, d)), patch.astype(np.float64)], axis=1) + pos.astype(np.float64)
    check_kernel(z, ref, "vit tokens", rel=2.0 ** -10, abs_rel=1e-3)


def test_argmax_f16(S):
    x = f16(R.standard_normal((6, 16, 768)))
    x[2, 0, 5] = x[2, 0, 700] = 50.0
    t = S.k_argmax_f16(dev(S, x), 768, 16 * 768, 6)
    assert np.array_equal(t.cpu().numpy(), ops.argmax_first(x[:, 0, :].astype(np.float64)))


def test_launchers_reject_bad_shapes(S):
    x = dev(S, np.zeros((1, 8, 8, 12), np.float16))
    with pytest.raises(S.StraitError):
        S.k_dwconv3x3(x, dev(S, np.zeros((3, 3, 12), np.float16)), None, 1)       # C % 8 != 0
    with pytest.raises(S.StraitError):
        S.k_attention(dev(S, np.zeros((1, 300, 192), np.float16)), dev(S, np.array([300], np.int32)), 1)   # more than 256 keys
    with pytest.raises(S.StraitError):
        S.k_layernorm(dev(S, np.zeros((2, 12), np.float16)), dev(S, np.ones(12, np.float32)), dev(S, np.zeros(12, np.float32)), 1e-5)


SPLITK_CASES = [
    # N, H, W, C, K, R, stride, pad, act, residual, out_f32   (few output tiles + long reduction: split-K path)
    (1, 7, 7, 512, 512, 3, 1, 1, 1, True, False),       # 49 pixels, K = 4608, residual + ReLU in the finishing kernel
    (2, 14, 14, 256, 256, 3, 2, 1, 1, False, False),    # strided 3x3, slices start in the middle of the tap sequence
    (1, 7, 7, 1024, 512, 1, 1, 0, 2, False, False),     # 1x1, ReLU6
    (8, 1, 1, 2048, 1000, 1, 1, 0, 0, False, True),     # classifier head: fp32 logits out of the finishing kernel
    (3, 9, 11, 64, 72, 3, 1, 1, 0, False, False),       # ragged M and N tiles, uneven split of the 18 slices
]


@pytest.mark.parametrize("case", SPLITK_CASES, ids=lambda c: "x".join(map(str, c[:8])))
def test_conv2d_split_k(S, case):
    N, H, W, C, K, Rk, stride, pad, act, use_res, out_f32 = case
    x = f16(R.standard_normal((N, H, W, C)))
    w = f16(R.standard_normal((K, C, Rk, Rk)) * (2.0 / (C * Rk * Rk)) ** 0.5)
    b = R.standard_normal(K).astype(np.float32)
    ref = ops.conv2d(x, w, b, stride, pad)
    res = f16(R.standard_normal(ref.shape)) if use_res else None
    if use_res:
        ref = ref + res.astype(np.float64)
    ref = act_ref(ref, act)
    w_krsc = np.ascontiguousarray(np.transpose(w, (0, 2, 3, 1)))
    args = (dev(S, x), dev(S, w_krsc), dev(S, b), stride, pad, act, None if res is None else dev(S, res), out_f32)
    y1 = S.k_conv2d(*args).float().cpu().numpy()
    check_kernel(y1, ref, f"split-K conv {case}")
    # slabs are reduced in a fixed order: a second launch gives the same bits
    y2 = S.k_conv2d(*args).float().cpu().numpy()
    assert np.array_equal(y1, y2)


def test_gemm_gelu_and_ragged_k(S):
    """GELU epilogue of the pipelined kernel and a reduction that is not a multiple of the slice."""
    for (M, N, K, act) in [(512, 768, 776, 3), (1000, 256, 40, 0), (4096, 3072, 768, 3)]:
        x = f16(R.standard_normal((M, K)))
        w = f16(R.standard_normal((N, K)) * K ** -0.5)
        b = (R.standard_normal(N) * 0.1).astype(np.float32)
        ref = act_ref(ops.linear(x, w, b), act)
        y = S.k_gemm(dev(S, x), dev(S, w), dev(S, b), act)
        check_kernel(y.float().cpu().numpy(), ref, f"gemm {M}x{N}x{K} act {act}")

