// 3x3 convolution of stride 2 and padding 1 on a 3-channel fp16 image, + bias + activation: the stem of MobileNetV2
// (paper Section 3.2 step (2): the first member of that network's kernel sequence), in one launch for gfx950.
//
// The generic path packs the image into a zero-bordered, channel-padded copy (one launch, 26 MB written at batch 64)
// and runs the convolution as a GEMM over it (K = 96 of which 27 are real).  Here the image is read as it lies in
// memory and nothing but the result is written.
//
// A workgroup (4 wavefronts) produces 4 x 32 output positions of one image at a time and walks over tiles in a
// grid-stride loop:
//   1. the 9 rows x 65 pixels the tile depends on go to LDS as they lie in memory (3 halfs per pixel), zeros outside
//      the image, starting S3_LEAD halfs to the left of the first window's first tap (which puts every window on a 4-byte
//      boundary: neighbouring output positions are two pixels, 12 bytes, apart).  Image widths that are multiples of 8
//      make every 16-byte piece of a patch row lie inside or outside the image as a whole (a row is 6 W bytes, a tile
//      starts 384 bytes after the one before, the patch 16 bytes before that), so those move as 16-byte pieces; other
//      even widths move 4 bytes at a time;
//   2. an output row of the tile is 32 rows of an implicit GEMM whose reduction runs over 3 filter rows x 16 halfs: the
//      9 halfs of a filter row's three taps are contiguous in the patch, preceded by one half and followed by six that
//      meet zero weights.  v_mfma_f32_32x32x16_f16, weights as the A operand (in registers for the whole launch), so a
//      lane ends up with 16 output channels of one position;
//   3. + bias, activation, fp16; a wavefront turns its row of 32 positions round in a piece of LDS of its own and stores
//      it as the run of 16-byte pieces it is in memory.
// With non-finite pixels the zero-weight neighbours of a window can turn a finite result into NaN; finite inputs
// give exactly the sum the definition gives.
#include "kernels.hpp"

namespace strait {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t uint32x4 __attribute__((ext_vector_type(4)));

constexpr int S3_TP = 4, S3_TQ = 32;                      // output tile
constexpr int S3_IR = 2 * S3_TP + 1;                      // input rows under it: 9
constexpr int S3_LEAD = 8;                                // halfs in a patch row before the first window's first tap
constexpr int S3_WIN0 = (S3_LEAD - 4) / 2;                // dword of a patch row the first window starts at (one pixel + one half before the tap)
constexpr int S3_USED_DW = S3_WIN0 + 3 * (S3_TQ - 1) + 8; // dwords of a patch row in use: 103
constexpr int S3_ROW_DW = 104;                            // its pitch: 26 pieces of 16 bytes
constexpr int S3_OPITCH = 40;                             // halfs between positions of the output staging: 64 bytes of channels + 16
static_assert(S3_USED_DW <= S3_ROW_DW && S3_ROW_DW % 4 == 0, "patch row");

template <bool V16>
__global__ void __launch_bounds__(256)
stem3x3s2_kernel(const half_t* __restrict__ x, const half_t* __restrict__ wf, const float* __restrict__ bias, int N, int H, int W,
                 int P, int Q, int tiles_p, int tiles_q, int Kout, int act, half_t* __restrict__ y, int hp) {
    __shared__ __attribute__((aligned(16))) uint32_t patch[S3_IR * S3_ROW_DW];
    __shared__ __attribute__((aligned(16))) half_t ostage[4 * (S3_TQ + 1) * S3_OPITCH];
    if (hp) __builtin_amdgcn_s_setprio(3);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, lh = lane >> 5;

    half8 wreg[3];
#pragma unroll
    for (int r = 0; r < 3; ++r) wreg[r] = *(const half8*)(wf + l32 * 48 + r * 16 + lh * 8);
    float bv[4][4];
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int c = 8 * g + 4 * lh + e;
            bv[g][e] = (bias && c < Kout) ? bias[c] : 0.f;
        }
    const half_t lo = (act == ACT_RELU || act == ACT_RELU6) ? (half_t)0.f : (half_t)-INFINITY;
    const half_t hi = act == ACT_RELU6 ? (half_t)6.f : (half_t)INFINITY;
    const half4 lo4 = {lo, lo, lo, lo}, hi4 = {hi, hi, hi, hi};

    // the 16-byte pieces of an output row this lane stores: piece lane + 64 j of 4 Kout; position and place within it
    half_t* mine = ostage + wave * ((S3_TQ + 1) * S3_OPITCH);
    const int kp = Kout >> 3;
    int opx[2], opart[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int i = lane + 64 * j;
        opx[j] = i / kp;                                   // S3_TQ or more: no such piece (fewer than 32 channels)
        opart[j] = i - opx[j] * kp;
        if (opx[j] >= S3_TQ) { opx[j] = S3_TQ; opart[j] = 0; }
    }
    const int total = N * tiles_p * tiles_q;              // the launcher checks that this fits
    const int row_elems = W * 3;
    for (int tile = (int)blockIdx.x; tile < total; tile += (int)gridDim.x) {
        const int tq = tile % tiles_q, rest = tile / tiles_q;
        const int tp = rest % tiles_p, n = rest / tiles_p;
        const int P0 = tp * S3_TP, Q0 = tq * S3_TQ;
        const half_t* img = x + (long long)n * H * row_elems;
        const int e0 = 6 * Q0 - S3_LEAD;                   // element (half) of an image row that patch dword 0 starts at
        if (V16) {
            constexpr int PIECES = S3_ROW_DW / 4;
            for (int id = tid; id < S3_IR * PIECES; id += 256) {
                const int row = id / PIECES, d = id - row * PIECES;
                const int ih = 2 * P0 - 1 + row, e = e0 + 8 * d;
                uint32x4 v = {0u, 0u, 0u, 0u};
                if ((unsigned)ih < (unsigned)H && e >= 0 && e < row_elems) v = *(const uint32x4*)(img + (long long)ih * row_elems + e);
                *(uint32x4*)(patch + row * S3_ROW_DW + 4 * d) = v;
            }
        } else {
            for (int id = tid; id < S3_IR * S3_USED_DW; id += 256) {
                const int row = id / S3_USED_DW, d = id - row * S3_USED_DW;
                const int ih = 2 * P0 - 1 + row, e = e0 + 2 * d;
                uint32_t v = 0;
                if ((unsigned)ih < (unsigned)H && e >= 0 && e < row_elems) v = *(const uint32_t*)(img + (long long)ih * row_elems + e);
                patch[row * S3_ROW_DW + d] = v;
            }
        }
        __syncthreads();
#pragma unroll
        for (int part = 0; part < S3_TP / 4; ++part) {
            const int rb = wave + 4 * part;                // this wavefront's output row of the tile
            floatx16 acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
            for (int r = 0; r < 3; ++r) {
                const uint32_t* ap = patch + (2 * rb + r) * S3_ROW_DW + S3_WIN0 + 3 * l32 + (lh ? 4 : 0);
                const uint32x4 au = {ap[0], ap[1], ap[2], ap[3]};
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(wreg[r], __builtin_bit_cast(half8, au), acc, 0, 0, 0);
            }
            // this lane: channels 8 g + 4 lh + (0..3) of position l32.  Through this wavefront's own piece of LDS the row
            // of 32 positions becomes what it is in memory, one run of 32 Kout halfs, which the lanes store 16 bytes each.
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                half4 h;
#pragma unroll
                for (int e = 0; e < 4; ++e) h[e] = (half_t)(acc[4 * g + e] + bv[g][e]);
                *(half4*)(mine + l32 * S3_OPITCH + 8 * g + 4 * lh) = __builtin_elementwise_min(__builtin_elementwise_max(h, lo4), hi4);
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            const int gp = P0 + rb;
            half_t* dst = y + (((long long)n * P + gp) * Q + Q0) * Kout;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const uint32x4 v = *(const uint32x4*)(mine + opx[j] * S3_OPITCH + 8 * opart[j]);
                if (gp < P && opx[j] < S3_TQ && Q0 + opx[j] < Q) *(uint32x4*)(dst + opx[j] * Kout + 8 * opart[j]) = v;
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
        __syncthreads();                                   // the next tile's patch overwrites this one
    }
}

// The same stem with the stride-1 depthwise 3x3 of a network's first block behind it (MobileNetV2: 32 channels, + bias +
// activation each): the stem's output, the largest tensor the two layers touch, stays in LDS.  A workgroup takes 8 x 30
// positions of the depthwise layer's output: the 10 x 32 stem positions under them and their rim are computed as above
// (21 rows of input, the same row layout with the patch starting SD_LEAD halfs before the first window's first tap, moved in
// 8- or 4-byte pieces, several requested before the first is waited for), written to LDS as [position][32 channels] with
// zeros where the position lies outside the stem's output (the depthwise layer pads that tensor), and the depthwise taps are
// added from there: a thread owns 8 channels of a column of 4 outputs, fp32, in the order of the stand-alone kernels.
// Bit-identical to the two launches.
constexpr int SD_TP = 8, SD_TQ = 30;                      // depthwise outputs per tile
constexpr int SD_SR = SD_TP + 2, SD_SC = 32;              // stem positions under them: 10 x 32
constexpr int SD_PR = 2 * SD_SR + 1;                      // input rows: 21
constexpr int SD_LEAD = 10;                               // halfs before the first window's first tap: windows on dword 3 + 3 c
constexpr int SD_WIN0 = (SD_LEAD - 4) / 2;
constexpr int SD_ROW_DW = 104;                            // 3 + 3 * 31 + 8
constexpr int SD_HP = 40;                                 // halfs between positions of the stem tile
static_assert(SD_WIN0 + 3 * (SD_SC - 1) + 8 <= SD_ROW_DW, "patch row");

template <bool V8>
__global__ void __launch_bounds__(256)
stem3x3s2_dw_kernel(const half_t* __restrict__ x, const half_t* __restrict__ wf, const float* __restrict__ bias, int act1,
                    const half_t* __restrict__ wd, const float* __restrict__ bd, int act2, int N, int H, int W, int P, int Q,
                    int tiles_p, int tiles_q, half_t* __restrict__ y, int hp) {
    __shared__ __attribute__((aligned(16))) uint32_t patch[SD_PR * SD_ROW_DW];
    __shared__ __attribute__((aligned(16))) half_t hs[SD_SR * SD_SC * SD_HP];
    if (hp) __builtin_amdgcn_s_setprio(3);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, lh = lane >> 5;

    half8 wreg[3];
#pragma unroll
    for (int r = 0; r < 3; ++r) wreg[r] = *(const half8*)(wf + l32 * 48 + r * 16 + lh * 8);
    float bv[4][4];
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int e = 0; e < 4; ++e) bv[g][e] = bias ? bias[8 * g + 4 * lh + e] : 0.f;
    const half_t lo = (act1 == ACT_RELU || act1 == ACT_RELU6) ? (half_t)0.f : (half_t)-INFINITY;
    const half_t hi = act1 == ACT_RELU6 ? (half_t)6.f : (half_t)INFINITY;
    const half4 lo4 = {lo, lo, lo, lo}, hi4 = {hi, hi, hi, hi};
    const half4 zero4 = {(half_t)0.f, (half_t)0.f, (half_t)0.f, (half_t)0.f};
    // depthwise: this thread's 8 channels, column and strip of 4 rows
    const int c8 = tid & 3, col = (tid >> 2) & 31, strip = tid >> 7;
    half8 wv[9];
#pragma unroll
    for (int k = 0; k < 9; ++k) wv[k] = *(const half8*)(wd + k * 32 + 8 * c8);
    float bdv[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) bdv[j] = bd ? bd[8 * c8 + j] : 0.f;
#pragma unroll
    for (int k = 0; k < 9; ++k) asm volatile("" : "+v"(wv[k]));   // in registers before the tile loop

    const int total = N * tiles_p * tiles_q;
    const int row_elems = W * 3;
    constexpr int PW = V8 ? 2 : 1;                         // dwords per piece of the patch
    constexpr int PIECES = SD_ROW_DW / PW, TOTAL = SD_PR * PIECES, NIT = (TOTAL + 255) / 256;
    uint32_t pv[NIT][2];                                   // this thread's pieces of a tile's patch, on their way to LDS
    bool pok[NIT];
    // requests the pieces of a tile's patch (all before any is waited for; each from an address inside the image, those
    // outside it turned into zeros when they are written to LDS)
    auto request_patch = [&](int tile) __attribute__((always_inline)) {
        const int tq = tile % tiles_q, rest = tile / tiles_q;
        const int tp = rest % tiles_p, n = rest / tiles_p;
        const half_t* img = x + (long long)n * H * row_elems;
        const int ih0 = 2 * (tp * SD_TP - 1) - 1;          // input row of patch row 0
        const int e0 = 6 * (tq * SD_TQ - 1) - SD_LEAD;     // element of an image row that patch dword 0 starts at
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int id = tid + it * 256;
            const int row = id / PIECES, d = id - row * PIECES;
            const int ih = ih0 + row, e = e0 + 2 * PW * d;
            pok[it] = id < TOTAL && (unsigned)ih < (unsigned)H && e >= 0 && e < row_elems;
            const half_t* src = img + (pok[it] ? (long long)ih * row_elems + e : 0);
            if (V8) { const uint2 t = *(const uint2*)src; pv[it][0] = t.x; pv[it][1] = t.y; }
            else { pv[it][0] = *(const uint32_t*)src; pv[it][1] = 0u; }
        }
    };
    if ((int)blockIdx.x < total) request_patch((int)blockIdx.x);
    for (int tile = (int)blockIdx.x; tile < total; tile += (int)gridDim.x) {
        const int tq = tile % tiles_q, rest = tile / tiles_q;
        const int tp = rest % tiles_p, n = rest / tiles_p;
        const int P0 = tp * SD_TP, Q0 = tq * SD_TQ;
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int id = tid + it * 256;
            const int row = id / PIECES, d = id - row * PIECES;
            if (id < TOTAL) {
                patch[row * SD_ROW_DW + PW * d] = pok[it] ? pv[it][0] : 0u;
                if (V8) patch[row * SD_ROW_DW + PW * d + 1] = pok[it] ? pv[it][1] : 0u;
            }
        }
        __syncthreads();
        if (tile + (int)gridDim.x < total) request_patch(tile + (int)gridDim.x);   // under way while this tile is computed
        for (int rb = wave; rb < SD_SR; rb += 4) {         // this wavefront's rows of stem positions
            floatx16 acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
            for (int r = 0; r < 3; ++r) {
                const uint32_t* ap = patch + (2 * rb + r) * SD_ROW_DW + SD_WIN0 + 3 * l32 + (lh ? 4 : 0);
                const uint32x4 au = {ap[0], ap[1], ap[2], ap[3]};
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(wreg[r], __builtin_bit_cast(half8, au), acc, 0, 0, 0);
            }
            const bool inside = (unsigned)(P0 - 1 + rb) < (unsigned)P && (unsigned)(Q0 - 1 + l32) < (unsigned)Q;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                half4 h;
#pragma unroll
                for (int e = 0; e < 4; ++e) h[e] = (half_t)(acc[4 * g + e] + bv[g][e]);
                h = __builtin_elementwise_min(__builtin_elementwise_max(h, lo4), hi4);
                *(half4*)(hs + (rb * SD_SC + l32) * SD_HP + 8 * g + 4 * lh) = inside ? h : zero4;
            }
        }
        __syncthreads();
        {
            float acc[4][8];
#pragma unroll
            for (int o = 0; o < 4; ++o)
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[o][j] = bdv[j];
            const int colr = col < SD_TQ ? col : SD_TQ - 1;    // the two spare columns of threads read in bounds and store nothing
#pragma unroll
            for (int rr = 0; rr < 6; ++rr) {
                const int ir = strip * 4 + rr;
                if ((unsigned)(P0 - 1 + ir) >= (unsigned)P) continue;
                half8 xv[3];
#pragma unroll
                for (int sx = 0; sx < 3; ++sx) xv[sx] = *(const half8*)(hs + (ir * SD_SC + colr + sx) * SD_HP + 8 * c8);
#pragma unroll
                for (int o = 0; o < 4; ++o) {
                    const int fr = rr - o;
                    if (fr < 0 || fr > 2) continue;
#pragma unroll
                    for (int sx = 0; sx < 3; ++sx)
#pragma unroll
                        for (int j = 0; j < 8; ++j) acc[o][j] += (float)xv[sx][j] * (float)wv[fr * 3 + sx][j];
                }
            }
            const int gq = Q0 + col;
#pragma unroll
            for (int o = 0; o < 4; ++o) {
                const int gp = P0 + strip * 4 + o;
                if (gp < P && gq < Q && col < SD_TQ) {
                    half8 ov;
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        float t = acc[o][j];
                        if (act2 == ACT_RELU) t = fmaxf(t, 0.f);
                        if (act2 == ACT_RELU6) t = fminf(fmaxf(t, 0.f), 6.f);
                        ov[j] = (half_t)t;
                    }
                    *(half8*)(y + (((long long)n * P + gp) * Q + gq) * 32 + 8 * c8) = ov;
                }
            }
        }
        __syncthreads();                                   // the next tile overwrites the patch and the stem tile
    }
}

int launch_stem3x3s2_dw(const half_t* x, const half_t* wf, const float* bias, int act1, const half_t* wd_rsc, const float* bd, int act2,
                        int N, int H, int W, half_t* y, int hp, hipStream_t stream) {
    if (!x || !wf || !wd_rsc || !y || N <= 0 || H < 1 || W < 2 || W % 2 != 0 || act1 == ACT_GELU || act2 == ACT_GELU) {
        set_error("stem 3x3/2 + depthwise: needs an even image width"); return -5;
    }
    if ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(wf) | reinterpret_cast<uintptr_t>(wd_rsc) | reinterpret_cast<uintptr_t>(y) |
         reinterpret_cast<uintptr_t>(bias) | reinterpret_cast<uintptr_t>(bd)) & 15) {
        set_error("stem 3x3/2 + depthwise: pointers must be 16-byte aligned"); return -1;
    }
    const int P = (H - 1) / 2 + 1, Q = (W - 1) / 2 + 1;
    const int tiles_p = (P + SD_TP - 1) / SD_TP, tiles_q = (Q + SD_TQ - 1) / SD_TQ;
    const long long total = (long long)N * tiles_p * tiles_q;
    if ((long long)H * W * 3 > 0x7fffffffLL || total > 0x7fffffffLL) { set_error("stem 3x3/2 + depthwise: image or grid too large"); return -5; }
    const unsigned blocks = (unsigned)(total < 512 ? total : 512);    // two workgroups per compute unit, each walking over tiles
    if (W % 4 == 0)
        hipLaunchKernelGGL(stem3x3s2_dw_kernel<true>, dim3(blocks), dim3(256), 0, stream, x, wf, bias, act1, wd_rsc, bd, act2, N, H, W, P, Q, tiles_p, tiles_q, y, hp);
    else
        hipLaunchKernelGGL(stem3x3s2_dw_kernel<false>, dim3(blocks), dim3(256), 0, stream, x, wf, bias, act1, wd_rsc, bd, act2, N, H, W, P, Q, tiles_p, tiles_q, y, hp);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_error("stem 3x3/2 + depthwise launch: %s", hipGetErrorString(e)); return -2; }
    return 0;
}

int launch_stem3x3s2(const half_t* x, const half_t* wf, const float* bias, int N, int H, int W, int Kout, int act, half_t* y, int hp,
                     hipStream_t stream) {
    if (!x || !wf || !y || N <= 0 || H < 1 || W < 2 || W % 2 != 0 || Kout < 8 || Kout > 32 || Kout % 8 != 0 || act == ACT_GELU) {
        set_error("stem 3x3/2: needs an even image width and 8, 16, 24 or 32 output channels"); return -5;
    }
    if ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(wf) | reinterpret_cast<uintptr_t>(y) | reinterpret_cast<uintptr_t>(bias)) & 15) {
        set_error("stem 3x3/2: pointers must be 16-byte aligned"); return -1;
    }
    const int P = (H - 1) / 2 + 1, Q = (W - 1) / 2 + 1;          // 3x3, stride 2, pad 1
    const int tiles_p = (P + S3_TP - 1) / S3_TP, tiles_q = (Q + S3_TQ - 1) / S3_TQ;
    const long long total = (long long)N * tiles_p * tiles_q;
    if ((long long)H * W * 3 > 0x7fffffffLL || total > 0x7fffffffLL) { set_error("stem 3x3/2: image or grid too large"); return -5; }
    const unsigned blocks = (unsigned)(total < 8192 ? total : 8192);
    if (W % 8 == 0)
        hipLaunchKernelGGL(stem3x3s2_kernel<true>, dim3(blocks), dim3(256), 0, stream, x, wf, bias, N, H, W, P, Q, tiles_p, tiles_q, Kout, act, y, hp);
    else
        hipLaunchKernelGGL(stem3x3s2_kernel<false>, dim3(blocks), dim3(256), 0, stream, x, wf, bias, N, H, W, P, Q, tiles_p, tiles_q, Kout, act, y, hp);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_error("stem 3x3/2 launch: %s", hipGetErrorString(e)); return -2; }
    return 0;
}

}  // namespace strait
