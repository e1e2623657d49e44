// The first two layers of an inverted residual block in one launch for gfx950: a 1x1 convolution that expands Cin
// channels to Chid (+ bias + activation) and the depthwise 3x3 convolution of stride 1 or 2 and padding 1 behind it
// (+ bias + activation).  (Paper Section 3.2 step (2): two members of MobileNetV2's kernel sequence.)
//
// Run as two launches, the expanded tensor, six times the block's input and the largest tensor of the network, is
// written to memory and read back.  Here it exists only tile by tile in LDS: a workgroup (4 wavefronts) takes a tile of
// TP x TQ output positions of one image and
//   A. loads the input pixels under the tile and its one-pixel rim (all Cin channels, zeros outside the image) into
//      LDS once;
//   B. for each group of 32 expanded channels in turn
//      1. computes the group for every pixel of A: blocks of 32 pixels, v_mfma_f32_32x32x16_f16 with the weights as
//         the A operand (this lane's fragments in registers, those of the next group already requested), + bias,
//         activation, fp16, zero for pixels outside the image (the depthwise layer pads the expanded tensor, not the
//         input), into LDS as [pixel][32 channels];
//      2. depthwise: a thread owns 8 channels of a column of TH output positions and adds their nine taps in fp32
//         from LDS, in the order the stand-alone depthwise kernels use, + bias, activation, and stores 16 bytes per
//         position.
// Every arithmetic step is the one the two stand-alone kernels take, in the same order: results are bit-identical.
// Small images give few tiles, so the groups of a tile can be shared out over several workgroups (gridDim.y).
#include <atomic>

#include "kernels.hpp"

namespace strait {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int EDW_HP = 40;                                // halfs between pixels of the expanded tile: 32 channels + 8

struct ExpandDwParams {
    const half_t* x; int N, H, W, Cin;
    const half_t* w1; int ldw1; const float* b1; int Chid, act1;
    const half_t* wd; const float* bd; int act2;
    half_t* y; int P, Q, tiles_p, tiles_q, groups_per_block, hp;
};

__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

__device__ __forceinline__ float edw_act(float v, int act) {
    if (act == ACT_RELU) return fmaxf(v, 0.f);
    if (act == ACT_RELU6) return fminf(fmaxf(v, 0.f), 6.f);
    return v;
}

// KS: 16-channel steps of the expansion's reduction (Cin rounded up); STRIDE of the depthwise layer; the tile is
// TP x TQ outputs with TP = 256 / (4 TQ) * TH.
template <int KS, int STRIDE, int TQ, int TH>
__global__ void __launch_bounds__(256) expand_dw_kernel(const ExpandDwParams p) {
    constexpr int STRIPS = 256 / (4 * TQ), TP = STRIPS * TH;
    constexpr int IR = (TP - 1) * STRIDE + 3, IC = (TQ - 1) * STRIDE + 3;      // input pixels under the tile and its rim
    constexpr int NPX = IR * IC, NPB = (NPX + 31) / 32, ROWS = NPB * 32;
    constexpr int XP = KS * 16 + 8;                                            // halfs between pixels of the input tile
    extern __shared__ __attribute__((aligned(16))) half_t edw_smem[];
    half_t* xs = edw_smem;                                                     // [ROWS][XP]
    half_t* hs = edw_smem + ROWS * XP;                                         // [ROWS][EDW_HP]
    if (p.hp) __builtin_amdgcn_s_setprio(3);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, lh = lane >> 5;

    // A workgroup takes every gridDim.x-th tile.  Virtual workgroup v -> tile: every XCD takes a contiguous range of tiles
    // (neighbouring tiles share rim pixels through one L2); v mod 8 is this workgroup's XCD for every v it takes, because
    // a grid smaller than the number of tiles is a multiple of eight.
    const int ntiles = p.N * p.tiles_p * p.tiles_q;
    auto tile_of = [&](int v, int& n, int& P0, int& Q0) __attribute__((always_inline)) {
        const unsigned per = (unsigned)ntiles >> 3, rem = (unsigned)ntiles & 7, xcd = (unsigned)v & 7, idx = (unsigned)v >> 3;
        const int tile = (int)((xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per) + idx);
        const int tq = tile % p.tiles_q, rest = tile / p.tiles_q;
        Q0 = tq * TQ; P0 = (rest % p.tiles_p) * TP; n = rest / p.tiles_p;
    };
    const int groups = (p.Chid + 31) >> 5;
    const int g_begin = (int)blockIdx.y * p.groups_per_block;
    const int g_end = g_begin + p.groups_per_block < groups ? g_begin + p.groups_per_block : groups;

    // fragments of the expansion's weights and its bias for group g: output channel 32 g + l32, input channels 16 ks + 8 lh ..
    auto load_w1 = [&](int g, half8 (&wf)[KS], float (&bv)[4][4]) __attribute__((always_inline)) {
        const int row = 32 * g + l32;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            half8 v;
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = (half_t)0.f;
            if (g < groups && row < p.Chid && 16 * ks + 8 * lh < p.Cin) v = *(const half8*)(p.w1 + (long long)row * p.ldw1 + 16 * ks + 8 * lh);
            wf[ks] = v;
        }
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
            const int c = 32 * g + 8 * g4 + 4 * lh;
            float4 b = make_float4(0.f, 0.f, 0.f, 0.f);
            if (g < groups && p.b1 && c < p.Chid) b = *(const float4*)(p.b1 + c);
            bv[g4][0] = b.x; bv[g4][1] = b.y; bv[g4][2] = b.z; bv[g4][3] = b.w;
        }
    };
    // the depthwise layer's weights and bias of group g for this thread's 8 channels (c8)
    const int c8 = tid & 3, col = (tid >> 2) % TQ, strip = (tid >> 2) / TQ;
    auto load_wd = [&](int g, half8 (&wv)[9], float (&bdv)[8]) __attribute__((always_inline)) {
        const int cd = 32 * g + 8 * c8;
        const bool ok = g < groups && cd < p.Chid;
#pragma unroll
        for (int k = 0; k < 9; ++k) {
#pragma unroll
            for (int j = 0; j < 8; ++j) wv[k][j] = (half_t)0.f;
            if (ok) wv[k] = *(const half8*)(p.wd + (long long)k * p.Chid + cd);
        }
        float4 b0 = make_float4(0.f, 0.f, 0.f, 0.f), b1 = b0;
        if (ok && p.bd) { b0 = *(const float4*)(p.bd + cd); b1 = *(const float4*)(p.bd + cd + 4); }
        bdv[0] = b0.x; bdv[1] = b0.y; bdv[2] = b0.z; bdv[3] = b0.w; bdv[4] = b1.x; bdv[5] = b1.y; bdv[6] = b1.z; bdv[7] = b1.w;
    };
    // both layers' weights are requested a whole group ahead: a group is short, and a wait for them would be most of it
    half8 wf[KS], wf_next[KS], wv[9], wv_next[9];
    float bv[4][4], bv_next[4][4], bdv[8], bdv_next[8];
    load_w1(g_begin, wf, bv);
    load_wd(g_begin, wv, bdv);

    // ---- A: the input tile: its 16-byte pieces are requested into registers (every request from an address inside the
    // image, several before the first is waited for) and deposited in LDS, zeros where the piece lies outside the image.
    // Where a thread holds few enough of them, the next tile's are requested while this tile is computed.
    constexpr int CH = KS * 2;                                                 // 16-byte pieces per pixel, zero-padded
    constexpr int TOTAL = ROWS * CH, NIT = (TOTAL + 255) / 256;
    constexpr bool AHEAD = NIT <= 12;
    constexpr int BATCH = AHEAD ? NIT : 8;
    half8 xv[BATCH];
    bool xok[BATCH];
    auto request_tile = [&](int v, int it0) __attribute__((always_inline)) {
        int n, P0, Q0;
        tile_of(v, n, P0, Q0);
        const int ih0 = P0 * STRIDE - 1, iw0 = Q0 * STRIDE - 1;
        const half_t* img = p.x + (long long)n * p.H * p.W * p.Cin;
#pragma unroll
        for (int b = 0; b < BATCH; ++b) {
            const int id = tid + (it0 + b) * 256;
            const int px = id / CH, ch = id - px * CH;
            const int ir = px / IC, ic = px - ir * IC;
            const int ih = ih0 + ir, iw = iw0 + ic;
            xok[b] = id < TOTAL && px < NPX && (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W && ch * 8 < p.Cin;
            const long long off = xok[b] ? ((long long)ih * p.W + iw) * p.Cin + ch * 8 : 0;
            xv[b] = *(const half8*)(img + off);
        }
    };
    auto deposit_tile = [&](int it0) __attribute__((always_inline)) {
#pragma unroll
        for (int b = 0; b < BATCH; ++b) {
            const int id = tid + (it0 + b) * 256;
            const int px = id / CH, ch = id - px * CH;
            half8 z;
#pragma unroll
            for (int j = 0; j < 8; ++j) z[j] = xok[b] ? xv[b][j] : (half_t)0.f;
            if (id < TOTAL) *(half8*)(xs + px * XP + ch * 8) = z;
        }
    };
    const half_t lo1 = (p.act1 == ACT_RELU || p.act1 == ACT_RELU6) ? (half_t)0.f : (half_t)-INFINITY;
    const half_t hi1 = p.act1 == ACT_RELU6 ? (half_t)6.f : (half_t)INFINITY;
    const half4 lo4 = {lo1, lo1, lo1, lo1}, hi4 = {hi1, hi1, hi1, hi1};
    const half4 zero4 = {(half_t)0.f, (half_t)0.f, (half_t)0.f, (half_t)0.f};

    if (AHEAD) request_tile((int)blockIdx.x, 0);
    for (int v = (int)blockIdx.x; v < ntiles; v += (int)gridDim.x) {
    int n, P0, Q0;
    tile_of(v, n, P0, Q0);
    const int ih0 = P0 * STRIDE - 1, iw0 = Q0 * STRIDE - 1;
    if (AHEAD) {
        deposit_tile(0);
    } else {
#pragma unroll
        for (int it0 = 0; it0 < NIT; it0 += BATCH) { request_tile(v, it0); deposit_tile(it0); }
    }
    __syncthreads();                                                           // the input tile is in place
    if (AHEAD && v + (int)gridDim.x < ntiles) request_tile(v + (int)gridDim.x, 0);

    for (int g = g_begin; g < g_end; ++g) {
        const int cd = 32 * g + 8 * c8;
        const bool cd_ok = cd < p.Chid;
        // ---- B1: expansion of this group for every pixel of the tile ----------------------------------------------
        for (int blk = wave; blk < NPB; blk += 4) {
            const int px = blk * 32 + l32;
            floatx16 acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const half8 xf = *(const half8*)(xs + px * XP + 16 * ks + 8 * lh);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(wf[ks], xf, acc, 0, 0, 0);
            }
            const int ir = px / IC, ic = px - ir * IC;
            const bool inside = px < NPX && (unsigned)(ih0 + ir) < (unsigned)p.H && (unsigned)(iw0 + ic) < (unsigned)p.W;
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                half4 h;
#pragma unroll
                for (int e = 0; e < 4; ++e) h[e] = (half_t)(acc[4 * g4 + e] + bv[g4][e]);
                h = __builtin_elementwise_min(__builtin_elementwise_max(h, lo4), hi4);
                *(half4*)(hs + px * EDW_HP + 8 * g4 + 4 * lh) = inside ? h : zero4;
            }
        }
        const int g_next = g + 1 < g_end ? g + 1 : g_begin;                   // after a tile's last group: the next tile's first
        load_w1(g_next, wf_next, bv_next);                                    // requested while this group goes on
        load_wd(g_next, wv_next, bdv_next);
        lds_barrier();
        // ---- B2: depthwise 3x3 from the expanded tile --------------------------------------------------------------
        {
            float acc[TH][8];
#pragma unroll
            for (int o = 0; o < TH; ++o)
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[o][j] = bdv[j];
            constexpr int RR = (TH - 1) * STRIDE + 3;
#pragma unroll
            for (int rr = 0; rr < RR; ++rr) {
                const int ir = strip * TH * STRIDE + rr;
                if ((unsigned)(ih0 + ir) >= (unsigned)p.H) continue;            // a row of padding adds nothing
                half8 xv[3];
#pragma unroll
                for (int sx = 0; sx < 3; ++sx) xv[sx] = *(const half8*)(hs + (ir * IC + col * STRIDE + sx) * EDW_HP + 8 * c8);
#pragma unroll
                for (int o = 0; o < TH; ++o) {
                    const int fr = rr - o * STRIDE;
                    if (fr < 0 || fr > 2) continue;
#pragma unroll
                    for (int sx = 0; sx < 3; ++sx)
#pragma unroll
                        for (int j = 0; j < 8; ++j) acc[o][j] += (float)xv[sx][j] * (float)wv[fr * 3 + sx][j];
                }
            }
            const int gq = Q0 + col;
#pragma unroll
            for (int o = 0; o < TH; ++o) {
                const int gp = P0 + strip * TH + o;
                if (gp < p.P && gq < p.Q && cd_ok) {
                    half8 ov;
#pragma unroll
                    for (int j = 0; j < 8; ++j) ov[j] = (half_t)edw_act(acc[o][j], p.act2);
                    *(half8*)(p.y + (((long long)n * p.P + gp) * p.Q + gq) * p.Chid + cd) = ov;
                }
            }
        }
#pragma unroll
        for (int k = 0; k < 9; ++k) wv[k] = wv_next[k];
#pragma unroll
        for (int j = 0; j < 8; ++j) bdv[j] = bdv_next[j];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) wf[ks] = wf_next[ks];
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4)
#pragma unroll
            for (int e = 0; e < 4; ++e) bv[g4][e] = bv_next[g4][e];
        lds_barrier();                                                         // the next group overwrites the expanded tile
    }
    }
}

constexpr unsigned edw_lds_bytes(int ks, int stride, int tq, int th) {
    const int tp = 256 / (4 * tq) * th, ir = (tp - 1) * stride + 3, ic = (tq - 1) * stride + 3, rows = (ir * ic + 31) / 32 * 32;
    return (unsigned)(rows * (ks * 16 + 8 + EDW_HP) * 2);
}

template <int KS, int STRIDE, int TQ, int TH>
static int launch_edw_tile(const ExpandDwParams& q, hipStream_t stream) {
    constexpr int STRIPS = 256 / (4 * TQ), TP = STRIPS * TH;
    constexpr unsigned lds = edw_lds_bytes(KS, STRIDE, TQ, TH);
    static_assert(lds <= 160 * 1024, "LDS limit");
    ExpandDwParams p = q;
    p.tiles_p = (p.P + TP - 1) / TP;
    p.tiles_q = (p.Q + TQ - 1) / TQ;
    const long long tiles = (long long)p.N * p.tiles_p * p.tiles_q;
    if (tiles <= 0 || tiles > 0x7fffffffLL) { set_error("expand+depthwise: bad grid (%lld tiles)", tiles); return -5; }
    // few tiles: share the channel groups of a tile out over several workgroups (each loads the input tile again)
    const int groups = (p.Chid + 31) / 32;
    int split = 1;
    while (tiles * split < 256 && split * 2 <= groups) split *= 2;
    p.groups_per_block = (groups + split - 1) / split;
    const unsigned gy = (unsigned)((groups + p.groups_per_block - 1) / p.groups_per_block);
    auto kernel = expand_dw_kernel<KS, STRIDE, TQ, TH>;
    static std::atomic<bool> configured{false};
    if (!configured.load(std::memory_order_acquire) && lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) { set_error("expand+depthwise: cannot reserve %u bytes of LDS: %s", lds, hipGetErrorString(e)); return -2; }
    }
    configured.store(true, std::memory_order_release);
    // where the kernel requests a tile's input one tile ahead, two workgroups per compute unit walk over the tiles
    constexpr int IRr = (TP - 1) * STRIDE + 3, ICc = (TQ - 1) * STRIDE + 3, NITs = (((IRr * ICc + 31) / 32 * 32) * KS * 2 + 255) / 256;
    const unsigned gx = (NITs <= 12 && tiles > 512) ? 512u : (unsigned)tiles;
    hipLaunchKernelGGL(kernel, dim3(gx, gy), dim3(256), lds, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_error("expand+depthwise launch: %s", hipGetErrorString(e)); return -2; }
    return 0;
}

template <int KS>
static int launch_edw_ks(const ExpandDwParams& p, int stride, hipStream_t stream) {
    // tile by image width: 32 wide, 16 wide (14 x 14 maps as one tile), 8 wide (7 x 7)
    if (stride == 1) {
        if (p.Q > 16) return launch_edw_tile<KS, 1, 32, 4>(p, stream);
        if (p.Q > 8) return launch_edw_tile<KS, 1, 16, 4>(p, stream);
        return launch_edw_tile<KS, 1, 8, 1>(p, stream);
    }
    // stride 2 puts four input pixels under an output: with many input channels only the smallest tile fits LDS
    // (two workgroups per compute unit matter more than a tile's ratio of rim to area: half the height where the taller tile
    // would take more than half of LDS)
    if constexpr (edw_lds_bytes(KS, 2, 32, 2) <= 80 * 1024) {
        if (p.Q > 16) return launch_edw_tile<KS, 2, 32, 2>(p, stream);
    } else if constexpr (edw_lds_bytes(KS, 2, 32, 1) <= 160 * 1024) {
        if (p.Q > 16) return launch_edw_tile<KS, 2, 32, 1>(p, stream);
    }
    if constexpr (edw_lds_bytes(KS, 2, 16, 2) <= 80 * 1024) {
        if (p.Q > 8) return launch_edw_tile<KS, 2, 16, 2>(p, stream);
    } else if constexpr (edw_lds_bytes(KS, 2, 16, 1) <= 160 * 1024) {
        if (p.Q > 8) return launch_edw_tile<KS, 2, 16, 1>(p, stream);
    }
    return launch_edw_tile<KS, 2, 8, 1>(p, stream);
}

bool expand_dw_supported(int Cin, int Chid, int stride) {
    return Cin >= 8 && Cin % 8 == 0 && Cin <= 160 && Chid >= 8 && Chid % 8 == 0 && (stride == 1 || stride == 2);
}

int launch_expand_dw(const half_t* x, int N, int H, int W, int Cin, const half_t* w1, int ldw1, const float* b1, int Chid, int act1,
                     const half_t* wd_rsc, const float* bd, int stride, int act2, half_t* y, int hp, hipStream_t stream) {
    if (!x || !w1 || !wd_rsc || !y || N <= 0 || H <= 0 || W <= 0 || !expand_dw_supported(Cin, Chid, stride) || ldw1 < Cin || ldw1 % 8 != 0 ||
        act1 == ACT_GELU || act2 == ACT_GELU) {
        set_error("expand+depthwise: needs 8 to 160 input channels and a number of expanded channels that are multiples of 8, stride 1 or 2");
        return -5;
    }
    if ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(w1) | reinterpret_cast<uintptr_t>(wd_rsc) | reinterpret_cast<uintptr_t>(y) |
         reinterpret_cast<uintptr_t>(b1) | reinterpret_cast<uintptr_t>(bd)) & 15) {
        set_error("expand+depthwise: pointers must be 16-byte aligned"); return -1;
    }
    ExpandDwParams p{};
    p.x = x; p.N = N; p.H = H; p.W = W; p.Cin = Cin;
    p.w1 = w1; p.ldw1 = ldw1; p.b1 = b1; p.Chid = Chid; p.act1 = act1;
    p.wd = wd_rsc; p.bd = bd; p.act2 = act2; p.y = y; p.hp = hp;
    p.P = (H - 1) / stride + 1; p.Q = (W - 1) / stride + 1;      // 3x3, padding 1
    const int ks = (Cin + 15) / 16;
    if (ks <= 1) return launch_edw_ks<1>(p, stride, stream);
    if (ks <= 2) return launch_edw_ks<2>(p, stride, stream);
    if (ks <= 4) return launch_edw_ks<4>(p, stride, stream);
    if (ks <= 6) return launch_edw_ks<6>(p, stride, stream);
    return launch_edw_ks<10>(p, stride, stream);
}

}  // namespace strait
