// ResNet stem in one launch for gfx950: 7x7 convolution of stride 2 and padding 3 on a 3-channel fp16 image,
// bias, ReLU, then 3x3 max pooling of stride 2 and padding 1.  (Paper Section 3.2 step (2): the first two
// members of ResNet-50's kernel sequence.)
//
// The unfused path writes the 64-channel convolution output (1.6 MB per image) and reads it back for the
// pooling, and needs a packed copy of the input before it; here the image is read once and only the pooled
// result (0.4 MB per image) is written.
//
// A workgroup (4 wavefronts) produces 8 x 7 pooled positions of one image at a time and walks over tiles in
// a grid-stride loop (the 64 x 176 weight matrix stays in registers across tiles):
//   1. the 39 x 35-pixel input patch the tile depends on goes to LDS as it lies in memory (3 halfs per pixel),
//      zeros outside the image;
//   2. the 17 x 15 convolution positions under the tile are 8 blocks of 32 rows of an implicit GEMM whose
//      reduction runs over 7 filter rows x 24 halfs: the 21 halfs of a filter row's 7 taps are contiguous in
//      the patch, preceded by one half and followed by two that meet zero weights, which makes every 8-half
//      operand fragment start on a 4-byte boundary.  v_mfma_f32_32x32x16_f16, weights as the A operand, so a
//      lane ends up with 16 channels of one position per 32-channel block;
//   3. bias + ReLU, positions outside the convolution's output set to 0 (never above a real ReLU output,
//      and every pooling window holds a real one), fp16 tile in LDS;
//   4. each pooled value is the maximum of 9 LDS vectors of 8 channels.
// With non-finite pixels the three zero-weight neighbours of a window can turn a finite result into NaN;
// finite inputs give exactly the sum the definition gives.
#include "kernels.hpp"

namespace strait {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t uint32x4 __attribute__((ext_vector_type(4)));

constexpr int SP_TP = 8, SP_TQ = 7;                       // pooled tile
constexpr int SP_CR = 2 * SP_TP + 1, SP_CC = 2 * SP_TQ + 1;   // convolution positions under it: 17 x 15
constexpr int SP_POS = SP_CR * SP_CC;                     // 255 (the 256th row of the GEMM is a dummy)
constexpr int SP_IR = 2 * SP_CR + 5;                      // input rows: 39
constexpr int SP_USED_DW = 54;                            // dwords of a patch row: 6 * 14 + 24 = 108 halfs
constexpr int SP_ROW_DW = 56;                             // its pitch
constexpr int SP_LDC = 72;                                // convolution tile pitch (halfs)
constexpr int SP_K = 64;                                  // output channels
constexpr int SP_STEPS = 11;                              // MFMA steps of 16: 22 fragments of 8 (21 in use)

__global__ void __launch_bounds__(256, 3)
stem_pool_kernel(const half_t* __restrict__ x, const half_t* __restrict__ wf, const float* __restrict__ bias, int N, int H, int W,
                 int P, int Q, int P2, int Q2, int tiles_p, int tiles_q, half_t* __restrict__ y, int hp) {
    __shared__ __attribute__((aligned(16))) uint32_t patch[SP_IR * SP_ROW_DW];
    __shared__ __attribute__((aligned(16))) half_t ctile[256 * SP_LDC];
    if (hp) __builtin_amdgcn_s_setprio(3);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, lh = lane >> 5;

    half8 wreg[2][SP_STEPS];
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
        for (int t = 0; t < SP_STEPS; ++t) wreg[ni][t] = *(const half8*)(wf + (ni * 32 + l32) * (SP_STEPS * 16) + (2 * t + lh) * 8);

    const long long total = (long long)N * tiles_p * tiles_q;
    const int row_elems = W * 3;
    for (long long tile = blockIdx.x; tile < total; tile += gridDim.x) {
        const int tq = (int)(tile % tiles_q);
        const long long rest = tile / tiles_q;
        const int tp = (int)(rest % tiles_p), n = (int)(rest / tiles_p);
        const int P0 = tp * SP_TP, Q0 = tq * SP_TQ;
        const int ih0 = 4 * P0 - 5, e0 = 12 * Q0 - 16;        // first input row / first (even) element of a row in the patch
        const half_t* img = x + (long long)n * H * row_elems;

        for (int idx = tid; idx < SP_IR * SP_USED_DW; idx += 256) {
            const int row = idx / SP_USED_DW, dw = idx - row * SP_USED_DW;
            const int ih = ih0 + row, e = e0 + 2 * dw;
            uint32_t v = 0;
            if ((unsigned)ih < (unsigned)H && e >= 0 && e < row_elems) v = *(const uint32_t*)(img + (long long)ih * row_elems + e);
            patch[row * SP_ROW_DW + dw] = v;
        }
        __syncthreads();

#pragma unroll 1
        for (int mi = 0; mi < 2; ++mi) {
            const int pos = (wave + 4 * mi) * 32 + l32;
            const int pc = pos < SP_POS ? pos : SP_POS - 1;
            const int cr = pc / SP_CC, cc = pc - cr * SP_CC;
            const uint32_t* abase = patch + (2 * cr) * SP_ROW_DW + 3 * cc;
            floatx16 acc[2];
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[ni][v] = 0.f;
#pragma unroll
            for (int t = 0; t < SP_STEPS; ++t) {
                // fragment 2t + lh = (filter row, third of its 24 halfs); the 22nd fragment meets zero weights
                const int f0 = 2 * t, f1 = 2 * t + 1 < 21 ? 2 * t + 1 : 20;
                const int off0 = (f0 / 3) * SP_ROW_DW + (f0 % 3) * 4, off1 = (f1 / 3) * SP_ROW_DW + (f1 % 3) * 4;
                const uint32_t* ap = abase + (lh ? off1 : off0);
                const uint32x4 au = {ap[0], ap[1], ap[2], ap[3]};
                const half8 a = __builtin_bit_cast(half8, au);
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wreg[0][t], a, acc[0], 0, 0, 0);
                acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wreg[1][t], a, acc[1], 0, 0, 0);
            }
            const int gr = 2 * P0 - 1 + cr, gc = 2 * Q0 - 1 + cc;
            const bool ok = pos < SP_POS && (unsigned)gr < (unsigned)P && (unsigned)gc < (unsigned)Q;
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int c0 = ni * 32 + 8 * g + 4 * lh;
                    const float4 b4 = *(const float4*)(bias + c0);
                    half4 h;
                    h[0] = (half_t)fmaxf(acc[ni][4 * g + 0] + b4.x, 0.f);
                    h[1] = (half_t)fmaxf(acc[ni][4 * g + 1] + b4.y, 0.f);
                    h[2] = (half_t)fmaxf(acc[ni][4 * g + 2] + b4.z, 0.f);
                    h[3] = (half_t)fmaxf(acc[ni][4 * g + 3] + b4.w, 0.f);
                    if (!ok) h = half4{(half_t)0, (half_t)0, (half_t)0, (half_t)0};
                    *(half4*)(ctile + pos * SP_LDC + c0) = h;
                }
        }
        __syncthreads();

        for (int item = tid; item < SP_TP * SP_TQ * 8; item += 256) {
            const int c8 = item & 7, pix = item >> 3;
            const int pp = pix / SP_TQ, pq = pix - pp * SP_TQ;
            const int gp = P0 + pp, gq = Q0 + pq;
            if (gp < P2 && gq < Q2) {
                const half_t* src = ctile + ((2 * pp) * SP_CC + 2 * pq) * SP_LDC + c8 * 8;
                half8 m = *(const half8*)src;
#pragma unroll
                for (int dr = 0; dr < 3; ++dr)
#pragma unroll
                    for (int dc = 0; dc < 3; ++dc)
                        if (dr | dc) m = __builtin_elementwise_max(m, *(const half8*)(src + (dr * SP_CC + dc) * SP_LDC));
                *(half8*)(y + (((long long)n * P2 + gp) * Q2 + gq) * SP_K + c8 * 8) = m;
            }
        }
        // The next tile's fill touches only `patch`, which nobody reads between the barrier above and the one after
        // the fill; `ctile` is rewritten only after that second barrier, when every thread has left the pooling loop.
    }
}

int launch_stem_pool(const half_t* x, const half_t* wf, const float* bias, int N, int H, int W, half_t* y, int hp,
                     hipStream_t stream) {
    if (!x || !wf || !bias || !y || N <= 0 || H < 1 || W < 2 || W % 2 != 0) { set_error("stem+pool: needs an even image width"); return -5; }
    const int P = (H - 1) / 2 + 1, Q = (W - 1) / 2 + 1;          // 7x7, stride 2, pad 3
    const int P2 = (P - 1) / 2 + 1, Q2 = (Q - 1) / 2 + 1;        // 3x3, stride 2, pad 1
    const int tiles_p = (P2 + SP_TP - 1) / SP_TP, tiles_q = (Q2 + SP_TQ - 1) / SP_TQ;
    const long long total = (long long)N * tiles_p * tiles_q;
    if ((long long)H * W * 3 > 0x7fffffffLL || total > 0x7fffffffLL) { set_error("stem+pool: image or grid too large"); return -5; }
    const unsigned blocks = (unsigned)(total < 768 ? total : 768);     // 3 workgroups on each of 256 compute units
    hipLaunchKernelGGL(stem_pool_kernel, dim3(blocks), dim3(256), 0, stream, x, wf, bias, N, H, W, P, Q, P2, Q2, tiles_p, tiles_q, y, hp);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_error("stem+pool launch: %s", hipGetErrorString(e)); return -2; }
    return 0;
}

}  // namespace strait
