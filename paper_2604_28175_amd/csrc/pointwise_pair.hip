// Two chained pointwise (1x1) convolutions in one launch, for gfx950 (CDNA4), NHWC fp16 activations:
//
//     y[m, 0:N1] = act1(x[m, 0:K1] W3^T + b3 + res[m, 0:N1])        written out (it is the next block's shortcut)
//     z[m, 0:N2] = act2(y[m, 0:N1] W1^T + b1)                       written out
//
// This is the seam between two residual bottlenecks of a served ResNet (paper Section 3.2 step (2): a batch is a
// sequence of dependent kernels; which kernels is ours to choose): the block-closing 1x1 with its residual add, and
// the next block's opening 1x1, which reads nothing but the tensor the first one has just produced.  At large batches
// both layers are bound by HBM traffic, and y is the largest tensor of the block; computing z from the y tile while
// it is still on the chip removes one full read of y from HBM and one launch.
//
// Built for 64 input channels and 256 channels in between (the first residual stage), where both weight matrices fit
// in LDS together (32 KB + N2 x 512 bytes).  A workgroup loads them once; each of its wavefronts then carries 32-pixel
// tiles through both layers on its own, with no barrier in the loop:
//   - input fragments come straight from global memory in MFMA operand layout (lane = pixel, 8 consecutive channels),
//     weight fragments (the A operand) from the shared copy in LDS, whose 16-byte chunks are XOR-swizzled by row so
//     that 16 consecutive rows read at one logical chunk hit 16 distinct bank groups;
//   - y is produced in chunks of 64 channels: MFMA, + bias, rounded to fp16, written to a 4.5 KB LDS region that
//     belongs to the wavefront alone as [pixel][channel], read back as 16-byte row segments to add the residual, clamp
//     and store; the finished values are put back in place and are at once the B operand (k = channel) of the second
//     product, whose accumulators stay in registers across the chunks;
//   - LDS operations of one wavefront execute in order, so the hand-overs between lanes need no synchronisation; the
//     wavefronts of a compute unit drift apart and hide each other's memory latency;
//   - the residual of the chunk after next and the input fragments of the next tile are requested ahead, across tile
//     boundaries, and always before the stores of the current chunk (returns are counted in issue order: a load issued
//     behind a store is not seen to arrive before that store is acknowledged);
//     with 128 output channels the accumulators leave no registers for a second set of input fragments, and the next
//     tile's are requested at the end of the current tile instead of at its start (with the early request the compiler
//     spilled 23 registers per lane: 155 -> 124 us at batch 128);
//   - rounding points are those of the two separate launches (fp32 accumulate, + bias, one rounding to fp16, residual
//     add and clamp in fp16), and the second product reduces over the channels in ascending order in 16-wide MFMA
//     steps like the stand-alone kernel, so the results are the same bit for bit.
//
// DUAL: in the first block of the stage the shortcut is not a tensor but a 1x1 projection of the block input x2
// [M][64].  A projection added to a pointwise convolution is one product over the two inputs side by side,
//     y = act1([x | x2] [W3 | Wd]^T + (b3 + bd)),
// so this instantiation reduces over 128 channels (the loader stores the two weight matrices side by side, 64 KB in
// LDS, and one summed bias), takes its second half of input fragments from x2, and reads no residual: the projection's
// own launch and the tensor it would write and this kernel read back do not exist.  The sum is rounded to fp16 once
// (separate launches round the projection first).
//
// (A version with one 128-pixel tile per workgroup, the y chunk shared by four wavefronts and weight fragments fetched
// from L2 per wavefront was measured first: three barriers per chunk and the weight traffic held it to 121-132 us on
// the first stage's shape, against 111 us for this one and 158 us for the two separate launches; with 128 input
// channels, where the weights do not fit in LDS, it took 95 us against 75 us for two launches, so that shape is left to
// the two launches.)
#include <atomic>

#include "kernels.hpp"

namespace strait {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

template <int N1, int N2, int NW, bool DUAL>
__global__ void __launch_bounds__(64 * NW, 1) pointwise_pair_wave_kernel(const PairParams p) {
    // DUAL: the block's shortcut is a 1x1 projection of a second 64-channel tensor.  Its product joins the first
    // one's reduction (K1 = 64 + 64, the two weight matrices side by side) instead of arriving as a residual tensor.
    constexpr int K1 = DUAL ? 128 : 64, KS1 = K1 / 16, CH = 64, NC = N1 / CH, NB2 = N2 / 32, LDC = CH + 8;
    constexpr int W3B = N1 * K1 * 2, W1B = N2 * N1 * 2, BIASB = (N1 + N2) * 4, PRIV = 32 * LDC * 2;
    static_assert(NC % 2 == 0 && N1 % 128 == 0 && (N2 == 64 || N2 == 128), "unsupported shape");
    static_assert(W3B + W1B + BIASB + NW * PRIV <= 160 * 1024, "LDS limit");
    extern __shared__ __attribute__((aligned(16))) char smem[];
    half_t* W3s = (half_t*)smem;                       // [N1][K1], chunk c of row r at c ^ swz3(r)
    auto swz3 = [](int r) { return K1 == 64 ? (r >> 1) & 7 : r & 15; };
    half_t* W1s = (half_t*)(smem + W3B);               // [N2][N1], chunk c of row r at c ^ (r & 15)
    float* b3s = (float*)(smem + W3B + W1B);
    float* b1s = b3s + N1;

    if (p.hp) __builtin_amdgcn_s_setprio(3);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, lh = lane >> 5;
    half_t* Cs = (half_t*)(smem + W3B + W1B + BIASB + wave * PRIV);   // this wavefront's own [32][LDC]

    for (int id = tid; id < N1 * (K1 / 8); id += 64 * NW) {
        const int row = id / (K1 / 8), c = id % (K1 / 8);
        *(uint4*)(W3s + row * K1 + ((c ^ swz3(row)) * 8)) = *(const uint4*)(p.w3 + (long long)row * K1 + c * 8);
    }
    for (int id = tid; id < N2 * (N1 / 8); id += 64 * NW) {
        const int row = id / (N1 / 8), c = id % (N1 / 8);
        *(uint4*)(W1s + row * N1 + ((c ^ (row & 15)) * 8)) = *(const uint4*)(p.w1 + (long long)row * N1 + c * 8);
    }
    for (int i = tid; i < N1; i += 64 * NW) b3s[i] = p.b3 ? p.b3[i] : 0.f;
    for (int i = tid; i < N2; i += 64 * NW) b1s[i] = p.b1 ? p.b1[i] : 0.f;

    const long long mlast = (long long)p.M - 1;
    const long long ntiles = ((long long)p.M + 31) / 32;
    const long long stride = (long long)gridDim.x * NW;
    long long t = (long long)blockIdx.x * NW + wave;

    const half_t lo1 = (p.act1 == ACT_RELU || p.act1 == ACT_RELU6) ? (half_t)0.f : (half_t)-INFINITY;
    const half_t hi1 = p.act1 == ACT_RELU6 ? (half_t)6.f : (half_t)INFINITY;
    const half8 lo8 = {lo1, lo1, lo1, lo1, lo1, lo1, lo1, lo1}, hi8 = {hi1, hi1, hi1, hi1, hi1, hi1, hi1, hi1};
    const half_t lo2 = (p.act2 == ACT_RELU || p.act2 == ACT_RELU6) ? (half_t)0.f : (half_t)-INFINITY;
    const half_t hi2 = p.act2 == ACT_RELU6 ? (half_t)6.f : (half_t)INFINITY;
    const half4 lz4 = {lo2, lo2, lo2, lo2}, hz4 = {hi2, hi2, hi2, hi2};

    // row-segment pass of a 32 x 64 chunk: lane -> (row, 8-channel segment), four per lane
    const int rrow = lane >> 3, rc8 = lane & 7;        // segment i of this lane: row rrow + 8 i
    // Lanes exchange data through the wavefront's LDS region.  The hardware executes one wavefront's LDS operations in
    // order; this keeps the compiler from moving them across the hand-over points.
    auto wave_sync = [] { __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront"); __builtin_amdgcn_wave_barrier(); };
    auto clampm = [&](long long m) { return m < mlast ? m : mlast; };
    // operands requested ahead: input fragments of a tile, residual segments of a chunk
    auto load_x = [&](long long tile, half8 (&xf)[KS1]) {
        const long long off = clampm(tile * 32 + l32) * 64 + lh * 8;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) xf[ks] = *(const half8*)(p.x + off + ks * 16);
        if constexpr (DUAL) {
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) xf[4 + ks] = *(const half8*)(p.x2 + off + ks * 16);
        }
    };
    auto load_res = [&](long long tile, int j, half8 (&rv)[4]) {
        if constexpr (!DUAL) {
#pragma unroll
            for (int i = 0; i < 4; ++i) rv[i] = *(const half8*)(p.res + clampm(tile * 32 + rrow + 8 * i) * N1 + j * CH + rc8 * 8);
        }
    };
    constexpr bool XPRE = N2 <= 64;                     // with 128 outputs the next tile's fragments do not fit in registers beside the accumulators
    half8 xf[KS1], xn[XPRE ? KS1 : 1], rvA[4], rvB[4];
    const long long t0 = t < ntiles ? t : ntiles - 1;   // a wavefront with no tile still issues valid loads
    load_x(t0, xf);
    load_res(t0, 0, rvA);
    load_res(t0, 1, rvB);
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();                                   // weights and biases are in LDS; the only barrier

    for (; t < ntiles; t += stride) {
        const long long tn = t + stride < ntiles ? t + stride : t;     // past the end: this tile again, unused
        const long long pix0 = t * 32;
        floatx16 acc2[NB2];
#pragma unroll
        for (int a = 0; a < NB2; ++a)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc2[a][v] = 0.f;
        if constexpr (XPRE) load_x(tn, xn);
        __builtin_amdgcn_sched_barrier(0);

        auto chunk = [&](int j, half8 (&rv)[4]) {
            // ---- first product: 64 channels x 32 pixels ----------------------------------------------
            floatx16 acc1[2];
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc1[a][v] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS1; ++ks)
#pragma unroll
                for (int a = 0; a < 2; ++a) {
                    const int row = j * CH + a * 32 + l32;
                    const half8 wf = *(const half8*)(W3s + row * K1 + (((ks * 2 + lh) ^ swz3(row)) * 8));
                    acc1[a] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wf, xf[ks], acc1[a], 0, 0, 0);
                }
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const float4 b4 = *(const float4*)(b3s + j * CH + a * 32 + 8 * g + 4 * lh);
                    const float bv[4] = {b4.x, b4.y, b4.z, b4.w};
                    half4 h;
#pragma unroll
                    for (int e = 0; e < 4; ++e) h[e] = (half_t)(acc1[a][4 * g + e] + bv[e]);
                    *(half4*)(Cs + l32 * LDC + a * 32 + 8 * g + 4 * lh) = h;
                }
            wave_sync();
            // ---- row segments: + residual, clamp, back into LDS as the next operand, store y -------------
            half8 vout[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                half8 v = *(const half8*)(Cs + (rrow + 8 * i) * LDC + rc8 * 8);
                if constexpr (!DUAL) v = v + rv[i];
                v = __builtin_elementwise_min(__builtin_elementwise_max(v, lo8), hi8);
                *(half8*)(Cs + (rrow + 8 * i) * LDC + rc8 * 8) = v;
                vout[i] = v;
            }
            __builtin_amdgcn_sched_barrier(0);
            if (j + 2 < NC) load_res(t, j + 2, rv); else load_res(tn, j + 2 - NC, rv);   // ahead of the stores below
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (pix0 + rrow + 8 * i <= mlast) *(half8*)(p.y + (pix0 + rrow + 8 * i) * N1 + j * CH + rc8 * 8) = vout[i];
            wave_sync();
            // ---- second product: N2 channels x 32 pixels, reduction over this chunk's 64 channels ------------
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const half8 yf = *(const half8*)(Cs + l32 * LDC + ks * 16 + lh * 8);
#pragma unroll
                for (int a = 0; a < NB2; ++a) {
                    const int row = a * 32 + l32;
                    const half8 wf = *(const half8*)(W1s + row * N1 + (((j * 8 + ks * 2 + lh) ^ (row & 15)) * 8));
                    acc2[a] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wf, yf, acc2[a], 0, 0, 0);
                }
            }
            wave_sync();
        };
#pragma unroll
        for (int j = 0; j < NC; j += 2) {
            chunk(j, rvA);
            chunk(j + 1, rvB);
        }
        // ---- z: bias, clamp, through the wavefront's LDS region 64 channels at a time, row segments out ----
#pragma unroll
        for (int h2 = 0; h2 < N2 / 64; ++h2) {
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const float4 b4 = *(const float4*)(b1s + h2 * 64 + a * 32 + 8 * g + 4 * lh);
                    const float bz[4] = {b4.x, b4.y, b4.z, b4.w};
                    half4 h;
#pragma unroll
                    for (int e = 0; e < 4; ++e) h[e] = (half_t)(acc2[h2 * 2 + a][4 * g + e] + bz[e]);
                    h = __builtin_elementwise_min(__builtin_elementwise_max(h, lz4), hz4);
                    *(half4*)(Cs + l32 * LDC + a * 32 + 8 * g + 4 * lh) = h;
                }
            wave_sync();
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const half8 v = *(const half8*)(Cs + (rrow + 8 * i) * LDC + rc8 * 8);
                if (pix0 + rrow + 8 * i <= mlast) *(half8*)(p.z + (pix0 + rrow + 8 * i) * N2 + h2 * 64 + rc8 * 8) = v;
            }
            wave_sync();
        }
#pragma unroll
        for (int ks = 0; ks < KS1; ++ks) { if constexpr (XPRE) xf[ks] = xn[ks]; }
        if constexpr (!XPRE) { if (t + stride < ntiles) load_x(t + stride, xf); }
    }
}

template <int N1, int N2, int NW, bool DUAL>
static int launch_pair_wave(const PairParams& p, hipStream_t stream) {
    constexpr unsigned lds = N1 * (DUAL ? 128 : 64) * 2 + N2 * N1 * 2 + (N1 + N2) * 4 + NW * 32 * 72 * 2;
    auto kernel = pointwise_pair_wave_kernel<N1, N2, NW, DUAL>;
    static std::atomic<bool> configured{false};
    if (!configured.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) { set_error("pointwise pair: cannot reserve %u bytes of LDS: %s", lds, hipGetErrorString(e)); return -2; }
        configured.store(true, std::memory_order_release);
    }
    // one workgroup per compute unit, each wavefront walking over tiles; fewer when there are fewer tiles
    const long long tiles = ((long long)p.M + 31) / 32;
    long long wgs = (tiles + NW - 1) / NW;
    if (wgs > 256) wgs = 256;
    hipLaunchKernelGGL(kernel, dim3((unsigned)wgs), dim3(64 * NW), lds, stream, p);
    return 0;
}

bool pointwise_pair_supported(int K1, int N1, int N2) { return K1 == 64 && N1 == 256 && (N2 == 64 || N2 == 128); }
bool pointwise_pair_proj_supported(int K1, int K2, int N1, int N2) { return K1 == 64 && K2 == 64 && N1 == 256 && N2 == 64; }

int launch_pointwise_pair(const PairParams& p, hipStream_t stream) {
    const bool dual = p.x2 != nullptr;
    if (!p.x || !p.w3 || (dual ? p.res != nullptr : !p.res) || !p.y || !p.w1 || !p.z || p.M <= 0) {
        set_error("pointwise pair: invalid parameters (a residual tensor or a second input, not both, not neither)");
        return -1;
    }
    if (dual ? !pointwise_pair_proj_supported(p.K1, p.K2, p.N1, p.N2) : !pointwise_pair_supported(p.K1, p.N1, p.N2)) {
        set_error("pointwise pair: unsupported shape (K1 %d, K2 %d, N1 %d, N2 %d)", p.K1, dual ? p.K2 : 0, p.N1, p.N2);
        return -5;
    }
    if ((reinterpret_cast<uintptr_t>(p.x) | reinterpret_cast<uintptr_t>(p.w3) | reinterpret_cast<uintptr_t>(p.y) |
         reinterpret_cast<uintptr_t>(p.w1) | reinterpret_cast<uintptr_t>(p.z) | reinterpret_cast<uintptr_t>(p.res) |
         reinterpret_cast<uintptr_t>(p.x2)) & 15) {
        set_error("pointwise pair: pointers must be 16-byte aligned");
        return -1;
    }
    const int rc = dual ? launch_pair_wave<256, 64, 8, true>(p, stream)
                 : p.N2 == 64 ? launch_pair_wave<256, 64, 8, false>(p, stream) : launch_pair_wave<256, 128, 8, false>(p, stream);
    if (rc) return rc;
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_error("pointwise pair launch: %s", hipGetErrorString(e)); return -2; }
    return 0;
}

}  // namespace strait
