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
//      zeros outside the image; it was fetched into registers while the previous tile was being computed;
//   2. the 17 x 15 convolution positions under the tile are 8 blocks of 32 rows of an implicit GEMM whose
//      reduction runs over 7 filter rows x 24 halfs: the 21 halfs of a filter row's 7 taps are contiguous in
//      the patch, preceded by one half and followed by two that meet zero weights, which makes every 8-half
//      operand fragment start on a 4-byte boundary.  v_mfma_f32_32x32x16_f16, weights as the A operand, so a
//      lane ends up with 16 channels of one position per 32-channel block;
//   3. bias + ReLU, positions outside the convolution's output set to 0 (never above a real ReLU output,
//      and every pooling window holds a real one), fp16 tile in LDS;
//   4. each pooled value is the maximum of 9 LDS vectors of 8 channels.
//   5. optionally the 1x1 convolution that follows in a residual network (64 -> 64 channels, + bias, ReLU: the first
//      block's opening layer): the pooled tile, which the pooling pass also leaves in LDS, is the B operand of four more
//      MFMA steps per wavefront, and the layer's own launch, with its read of the pooled tensor, goes away.  Same
//      instruction, reduction order and rounding points as the stand-alone kernel: bit-identical.
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
constexpr int SP_PLD = 72;                                // pooled tile pitch (halfs)

__global__ void __launch_bounds__(256, 2)
stem_pool_kernel(const half_t* __restrict__ x, const half_t* __restrict__ wf, const float* __restrict__ bias, int N, int H, int W,
                 int P, int Q, int P2, int Q2, int tiles_p, int tiles_q, half_t* __restrict__ y, int hp,
                 const half_t* __restrict__ w1, const float* __restrict__ b1, half_t* __restrict__ t1) {
    __shared__ __attribute__((aligned(16))) uint32_t patch[SP_IR * SP_ROW_DW];
    __shared__ __attribute__((aligned(16))) half_t ctile[256 * SP_LDC];
    __shared__ __attribute__((aligned(16))) half_t ptile[64 * SP_PLD];      // pooled tile (56 pixels in use) for step 5
    if (hp) __builtin_amdgcn_s_setprio(3);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, lh = lane >> 5;

    __shared__ __attribute__((aligned(16))) float bias_s[SP_K];
    if (tid < SP_K) bias_s[tid] = bias[tid];          // visible after the first barrier of the tile loop
    half8 wreg[2][SP_STEPS];
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
        for (int t = 0; t < SP_STEPS; ++t) {
            wreg[ni][t] = *(const half8*)(wf + (ni * 32 + l32) * (SP_STEPS * 16) + (2 * t + lh) * 8);
            // Keep the fragment in registers: re-loading it inside the tile loop would put a wait for all older loads,
            // the prefetched patch among them, in front of every MFMA.
            asm volatile("" : "+v"(wreg[ni][t]));
        }

    // step 5: this wavefront's 32 of the 64 pooled pixels (pb) and 32 of the 64 output channels (cb)
    const int pb = wave & 1, cb = wave >> 1;
    half8 w1f[4];
    float b1v[4][4];
    if (w1) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) w1f[ks] = *(const half8*)(w1 + (cb * 32 + l32) * 64 + ks * 16 + lh * 8);
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int e = 0; e < 4; ++e) b1v[g][e] = b1 ? b1[cb * 32 + 8 * g + 4 * lh + e] : 0.f;
    }

    const int total = N * tiles_p * tiles_q;          // the launcher checks that this fits
    const int row_elems = W * 3;
    // Patch traffic: thread (fr, fd) = (tid / 54, tid % 54) of the first 216 moves dword fd of patch rows fr, fr + 4,
    // ..., so a row step is one pointer increment.  The next tile's patch is fetched into registers while this tile
    // is computed.
    constexpr int SP_NF = (SP_IR + 3) / 4;                 // 10 rows per thread (the last pass covers 3 rows)
    const int fr = tid / SP_USED_DW, fd = tid - fr * SP_USED_DW;
    const bool mover = tid < 4 * SP_USED_DW;
    uint32_t pre[SP_NF], pre_in = 0;
    auto fetch_patch = [&](int tile) {
        pre_in = 0;
        const int tq = tile % tiles_q, rest = tile / tiles_q;
        const int tp = rest % tiles_p, n = rest / tiles_p;
        const int ih0 = 4 * tp * SP_TP - 5 + fr;           // first input row of this thread
        const int e = 12 * tq * SP_TQ - 16 + 2 * fd;       // its (even) element within an image row
        const bool col_in = mover && e >= 0 && e < row_elems;
        const half_t* img = x + (long long)n * H * row_elems;
        const half_t* src = img + (long long)ih0 * row_elems + e;
#pragma unroll
        for (int i = 0; i < SP_NF; ++i) {
            const int ih = ih0 + 4 * i;
            // every lane loads (the image's first dword when its element lies outside) and then selects: no branches
            const bool in = col_in && (unsigned)ih < (unsigned)H && (4 * i + fr) < SP_IR;
            pre[i] = *(const uint32_t*)(in ? src + (long long)(4 * i) * row_elems : img);
            pre_in |= in ? 1u << i : 0u;       // the selection waits until the value is used, one tile later
        }
    };
    if ((int)blockIdx.x < total) fetch_patch((int)blockIdx.x);
    uint32_t* const pdst = patch + fr * SP_ROW_DW + fd;
    for (int tile = (int)blockIdx.x; tile < total; tile += (int)gridDim.x) {
        const int tq = tile % tiles_q, rest = tile / tiles_q;
        const int tp = rest % tiles_p, n = rest / tiles_p;
        const int P0 = tp * SP_TP, Q0 = tq * SP_TQ;
        if (mover) {
#pragma unroll
            for (int i = 0; i < SP_NF; ++i)
                if (4 * i + fr < SP_IR) pdst[4 * i * SP_ROW_DW] = (pre_in >> i & 1u) ? pre[i] : 0u;
        }
        __syncthreads();
        if (tile + (int)gridDim.x < total) fetch_patch(tile + (int)gridDim.x);

#pragma unroll 1
        for (int mi = 0; mi < 2; ++mi) {
            const int pos = (wave + 4 * mi) * 32 + l32;
            const int pc = pos < SP_POS ? pos : SP_POS - 1;
            const int cr = pc / SP_CC, cc = pc - cr * SP_CC;
            // Fragment 2t + lh = (filter row, third of its 24 halfs).  The upper half-wave reads the fragment after the
            // lower one's: 4 dwords further on in the same filter row, or at the start of the next one (56 - 8 dwords
            // further); the 22nd fragment meets zero weights and re-reads the 21st.  Three lane-dependent bases, and every
            // step's own offset is a constant.
            const uint32_t* abase = patch + (2 * cr) * SP_ROW_DW + 3 * cc;
            const uint32_t* base_same = abase + (lh ? 4 : 0);
            const uint32_t* base_next = abase + (lh ? SP_ROW_DW - 8 : 0);
            floatx16 acc[2];
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                for (int g = 0; g < 4; ++g) {          // the accumulators start from the bias
                    const float4 b4 = *(const float4*)(bias_s + ni * 32 + 8 * g + 4 * lh);
                    acc[ni][4 * g + 0] = b4.x; acc[ni][4 * g + 1] = b4.y; acc[ni][4 * g + 2] = b4.z; acc[ni][4 * g + 3] = b4.w;
                }
#pragma unroll
            for (int t = 0; t < SP_STEPS; ++t) {
                const int f0 = 2 * t;
                const int off0 = (f0 / 3) * SP_ROW_DW + (f0 % 3) * 4;
                const uint32_t* ap = (t == SP_STEPS - 1 ? abase : (f0 % 3 == 2 ? base_next : base_same)) + off0;
                const uint32x4 au = {ap[0], ap[1], ap[2], ap[3]};
                const half8 a = __builtin_bit_cast(half8, au);
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wreg[0][t], a, acc[0], 0, 0, 0);
                acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wreg[1][t], a, acc[1], 0, 0, 0);
            }
            const int gr = 2 * P0 - 1 + cr, gc = 2 * Q0 - 1 + cc;
            const bool ok = pos < SP_POS && (unsigned)gr < (unsigned)P && (unsigned)gc < (unsigned)Q;
            const half4 zero4 = {(half_t)0, (half_t)0, (half_t)0, (half_t)0};
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    half4 h;
#pragma unroll
                    for (int j = 0; j < 4; ++j) h[j] = (half_t)acc[ni][4 * g + j];
                    h = __builtin_elementwise_max(h, zero4);        // ReLU after rounding gives the same fp16 value
                    if (!ok) h = zero4;
                    *(half4*)(ctile + pos * SP_LDC + ni * 32 + 8 * g + 4 * lh) = h;
                }
        }
        __syncthreads();

        for (int item = tid; item < SP_TP * SP_TQ * 8; item += 256) {
            const int c8 = item & 7, pix = item >> 3;
            const int pp = pix / SP_TQ, pq = pix - pp * SP_TQ;
            const int gp = P0 + pp, gq = Q0 + pq;
            if (gp < P2 && gq < Q2) {
                const half_t* src = ctile + ((2 * pp) * SP_CC + 2 * pq) * SP_LDC + c8 * 8;
                half8 v[9];
#pragma unroll
                for (int k = 0; k < 9; ++k) v[k] = *(const half8*)(src + ((k / 3) * SP_CC + k % 3) * SP_LDC);
                half8 m = v[0];
#pragma unroll
                for (int k = 1; k < 9; ++k) m = __builtin_elementwise_max(m, v[k]);
                *(half8*)(y + (((long long)n * P2 + gp) * Q2 + gq) * SP_K + c8 * 8) = m;
                if (w1) *(half8*)(ptile + pix * SP_PLD + c8 * 8) = m;
            } else if (w1) {
                const half8 z = {0, 0, 0, 0, 0, 0, 0, 0};
                *(half8*)(ptile + pix * SP_PLD + c8 * 8) = z;     // outside the pooled image: multiplied, never stored
            }
        }
        if (w1) {
            __syncthreads();
            floatx16 a1;
#pragma unroll
            for (int v = 0; v < 16; ++v) a1[v] = 0.f;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const half8 pf = *(const half8*)(ptile + (pb * 32 + l32) * SP_PLD + ks * 16 + lh * 8);
                a1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(w1f[ks], pf, a1, 0, 0, 0);
            }
            const int pix = pb * 32 + l32;
            const int pp = pix / SP_TQ, pq = pix - pp * SP_TQ;
            const int gp = P0 + pp, gq = Q0 + pq;
            if (pix < SP_TP * SP_TQ && gp < P2 && gq < Q2) {
                half_t* dst = t1 + (((long long)n * P2 + gp) * Q2 + gq) * SP_K + cb * 32 + 4 * lh;
                const half4 zero4 = {(half_t)0, (half_t)0, (half_t)0, (half_t)0};
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    half4 h;
#pragma unroll
                    for (int e = 0; e < 4; ++e) h[e] = (half_t)(a1[4 * g + e] + b1v[g][e]);
                    *(half4*)(dst + 8 * g) = __builtin_elementwise_max(h, zero4);
                }
            }
        }
        // The next tile's patch is written to LDS after this point: nobody reads `patch` between the barrier above and
        // the one after that write; `ctile` is rewritten only after that second barrier, when every thread has left
        // the pooling loop.
    }
}

int launch_stem_pool(const half_t* x, const half_t* wf, const float* bias, int N, int H, int W, half_t* y, int hp,
                     hipStream_t stream, const half_t* w1, const float* b1, half_t* t1) {
    if (!x || !wf || !bias || !y || N <= 0 || H < 1 || W < 2 || W % 2 != 0) { set_error("stem+pool: needs an even image width"); return -5; }
    if ((w1 != nullptr) != (t1 != nullptr) || ((reinterpret_cast<uintptr_t>(w1) | reinterpret_cast<uintptr_t>(t1)) & 15)) {
        set_error("stem+pool: the following 1x1 convolution needs its weights and its output, 16-byte aligned"); return -1;
    }
    const int P = (H - 1) / 2 + 1, Q = (W - 1) / 2 + 1;          // 7x7, stride 2, pad 3
    const int P2 = (P - 1) / 2 + 1, Q2 = (Q - 1) / 2 + 1;        // 3x3, stride 2, pad 1
    const int tiles_p = (P2 + SP_TP - 1) / SP_TP, tiles_q = (Q2 + SP_TQ - 1) / SP_TQ;
    const long long total = (long long)N * tiles_p * tiles_q;
    if ((long long)H * W * 3 > 0x7fffffffLL || total > 0x7fffffffLL) { set_error("stem+pool: image or grid too large"); return -5; }
    const unsigned blocks = (unsigned)(total < 512 ? total : 512);     // 2 workgroups on each of 256 compute units
    hipLaunchKernelGGL(stem_pool_kernel, dim3(blocks), dim3(256), 0, stream, x, wf, bias, N, H, W, P, Q, P2, Q2, tiles_p, tiles_q, y, hp, w1, b1, t1);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_error("stem+pool launch: %s", hipGetErrorString(e)); return -2; }
    return 0;
}

}  // namespace strait
