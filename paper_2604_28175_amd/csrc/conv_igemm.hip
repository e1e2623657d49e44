// Implicit-GEMM convolution / GEMM on fp16 MFMA for gfx950 (CDNA4), NHWC activations.
//
// Computes the convolution layers (and, with R = S = 1, the linear layers) of a served batch's
// kernel sequence (paper Section 3.2, step (2)):
//     y[m, k] = act(bias[k] + sum_{r,s,c} x[n, p*stride+r-pad, q*stride+s-pad, c] * w[k, r, s, c] (+ res[m, k]))
// with m = (n, p, q) running over output pixels.
//
// Mapping to the machine
//   - a workgroup of 4 wavefronts (2 x 2) owns a BM-pixel x BN-channel output tile and walks the
//     reduction (r, s, c) in slices of BK = 32;
//   - each slice of the gathered input ("X", BM x 32) and of the weights ("W", BN x 32) is staged
//     in LDS with an 80-byte row pitch, which makes the 16-byte MFMA operand reads conflict free;
//     the next slice is fetched from global memory into registers while the current one feeds
//     v_mfma_f32_32x32x16_f16, and two LDS buffers alternate so one barrier per slice suffices;
//   - the weights are the MFMA "A" operand (rows = channels) and the pixels the "B" operand
//     (columns), so a lane ends up holding 4 consecutive channels of one pixel per accumulator
//     quad: the epilogue adds the bias, rounds to fp16, parks the tile in LDS as [pixel][channel]
//     and writes it out (adding the residual, applying the activation) as 16-byte row segments;
//   - workgroup ids are re-ordered so that tiles sharing an input slice run on the same XCD
//     (consecutive hardware ids are dealt round-robin over the 8 XCDs, each with its own L2).
#include <atomic>
#include <type_traits>

#include "kernels.hpp"

namespace strait {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

enum { MODE_1X1 = 0, MODE_GATHER8 = 1, MODE_SCALAR = 2 };

// erf by the rational approximation 7.1.26 of Abramowitz & Stegun (|error| <= 1.5e-7, far below
// the 2^-11 resolution of the fp16 result): 1 - (a1 t + ... + a5 t^5) exp(-x^2), t = 1/(1 + p|x|).
__device__ __forceinline__ float fast_erf(float x) {
    const float ax = fabsf(x);
    const float t = __builtin_amdgcn_rcpf(1.f + 0.3275911f * ax);
    const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
    const float r = 1.f - poly * __expf(-ax * ax);
    return copysignf(r, x);
}
__device__ __forceinline__ float gelu_f(float v) { return 0.5f * v * (1.f + fast_erf(v * 0.70710678118654752440f)); }

__device__ __forceinline__ float apply_act(float v, int act) {
    if (act == ACT_RELU) return fmaxf(v, 0.f);
    if (act == ACT_RELU6) return fminf(fmaxf(v, 0.f), 6.f);
    if (act == ACT_GELU) return gelu_f(v);
    return v;
}

template <int BM, int BN, int MODE, bool STAGED>
__global__ void __launch_bounds__(256) conv_igemm_kernel(const ConvParams p) {
    constexpr int BK = 32, LDK = BK + 8;
    constexpr int TM = BM / 2, TN = BN / 2;          // wave tile
    constexpr int TMB = TM / 32, TNB = TN / 32;      // 32x32 MFMA blocks per wave tile
    constexpr int XC = BM * 4 / 256, WC = BN * 4 / 256;   // 16-byte chunks per thread per slice
    constexpr int LDC = BN + 8;
    static_assert(XC >= 1 && WC >= 1, "tile too small for 256 threads");
    static_assert(2 * (BM + BN) * LDK >= BM * LDC, "epilogue tile must fit in the pipeline buffers");

    __shared__ __attribute__((aligned(16))) half_t smem[2 * (BM + BN) * LDK];
    half_t* Xs = smem;                       // [2][BM][LDK]
    half_t* Ws = smem + 2 * BM * LDK;        // [2][BN][LDK]

    if (p.hp) __builtin_amdgcn_s_setprio(3);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave & 1) * TM, wn0 = (wave >> 1) * TN;
    const int l32 = lane & 31, lh = lane >> 5;

    // XCD-aware tile order: hardware workgroup id b runs on XCD b % 8.
    const int tiles_n = (p.Cout + BN - 1) / BN;
    int logical;
    {
        const int nb = gridDim.x, b = blockIdx.x;
        const int per = nb >> 3, rem = nb & 7, xcd = b & 7, idx = b >> 3;
        logical = (xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per) + idx;
    }
    const int m0 = (logical / tiles_n) * BM;
    const int n0 = (logical % tiles_n) * BN;

    // ---- per-thread gather state ------------------------------------------------------
    const int ch = tid & 3;                  // which 8-element chunk of the 32-wide slice
    long long xbase[XC];
    int ih0[XC], iw0[XC];
    bool mval[XC];
#pragma unroll
    for (int i = 0; i < XC; ++i) {
        const int row = (tid >> 2) + i * 64;
        const int m = m0 + row;
        mval[i] = m < p.M;
        const int mm = mval[i] ? m : 0;
        if (MODE == MODE_1X1 && p.stride_h == 1) {
            xbase[i] = (long long)mm * p.sW;     // dense [M][C] matrix (sW == row pitch)
            ih0[i] = iw0[i] = 0;
        } else {
            const int n = mm / p.PQ, rem = mm - n * p.PQ;
            const int pp = rem / p.Q, qq = rem - pp * p.Q;
            ih0[i] = pp * p.stride_h - p.pad_h;
            iw0[i] = qq * p.stride_w - p.pad_w;
            xbase[i] = (long long)n * p.sN + (long long)ih0[i] * p.sH + (long long)iw0[i] * p.sW;
        }
    }
    int k0 = ch * 8;                         // this thread's k index within the reduction
    int r = 0, s = 0, c0 = k0;               // MODE_GATHER8: (r, s, c0) of k0
    if (MODE == MODE_GATHER8) {
        while (c0 >= p.C) { c0 -= p.C; if (++s == p.S) { s = 0; ++r; } }
    }
    bool wval[WC];
    const half_t* wptr[WC];
#pragma unroll
    for (int i = 0; i < WC; ++i) {
        const int row = (tid >> 2) + i * 64;
        wval[i] = (n0 + row) < p.Cout;
        wptr[i] = p.w + (long long)(wval[i] ? n0 + row : 0) * p.ldw + ch * 8;
    }

    const int nk = (p.Kg + BK - 1) / BK;
    uint4 xr[XC], wr[WC];

    auto fetch = [&](int kt) {
        const bool kval = k0 < p.Kg;
#pragma unroll
        for (int i = 0; i < WC; ++i) {
            // weight rows are zero padded up to ldw (a multiple of 8), so a chunk that starts
            // below ldw is entirely readable
            wr[i] = (wval[i] && (kt * BK + ch * 8) < p.ldw) ? *(const uint4*)(wptr[i] + kt * BK) : make_uint4(0, 0, 0, 0);
        }
        if (MODE == MODE_1X1) {
#pragma unroll
            for (int i = 0; i < XC; ++i)
                xr[i] = (mval[i] && kval) ? *(const uint4*)(p.x + xbase[i] + k0) : make_uint4(0, 0, 0, 0);
        } else if (MODE == MODE_GATHER8) {
            const int koff = r * p.sH + s * p.sW + c0;
#pragma unroll
            for (int i = 0; i < XC; ++i) {
                const bool ok = mval[i] && kval && (unsigned)(ih0[i] + r) < (unsigned)p.H &&
                                (unsigned)(iw0[i] + s) < (unsigned)p.W;
                xr[i] = ok ? *(const uint4*)(p.x + xbase[i] + koff) : make_uint4(0, 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int i = 0; i < XC; ++i) {
                half8 v;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int k = k0 + j;
                    const int rs = k / p.C, c = k - rs * p.C;
                    const int rr = rs / p.S, ss = rs - rr * p.S;
                    const bool ok = mval[i] && k < p.Kg && (unsigned)(ih0[i] + rr) < (unsigned)p.H &&
                                    (unsigned)(iw0[i] + ss) < (unsigned)p.W;
                    v[j] = ok ? p.x[xbase[i] + (long long)rr * p.sH + (long long)ss * p.sW + c] : (half_t)0;
                }
                xr[i] = *(uint4*)&v;
            }
        }
        // advance to the next slice
        k0 += BK;
        if (MODE == MODE_GATHER8) {
            c0 += BK;
            while (c0 >= p.C) { c0 -= p.C; if (++s == p.S) { s = 0; ++r; } }
        }
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int i = 0; i < XC; ++i)
            *(uint4*)(Xs + (buf * BM + (tid >> 2) + i * 64) * LDK + ch * 8) = xr[i];
#pragma unroll
        for (int i = 0; i < WC; ++i)
            *(uint4*)(Ws + (buf * BN + (tid >> 2) + i * 64) * LDK + ch * 8) = wr[i];
    };

    floatx16 acc[TNB][TMB];
#pragma unroll
    for (int a = 0; a < TNB; ++a)
#pragma unroll
        for (int b = 0; b < TMB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    fetch(0);
    stash(0);
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) fetch(kt + 1);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            half8 wf[TNB], xf[TMB];
#pragma unroll
            for (int a = 0; a < TNB; ++a)
                wf[a] = *(const half8*)(Ws + (buf * BN + wn0 + a * 32 + l32) * LDK + ks * 16 + lh * 8);
#pragma unroll
            for (int b = 0; b < TMB; ++b)
                xf[b] = *(const half8*)(Xs + (buf * BM + wm0 + b * 32 + l32) * LDK + ks * 16 + lh * 8);
#pragma unroll
            for (int a = 0; a < TNB; ++a)
#pragma unroll
                for (int b = 0; b < TMB; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wf[a], xf[b], acc[a][b], 0, 0, 0);
        }
        if (kt + 1 < nk) stash(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue ---------------------------------------------------------------------
    // lane holds, for accumulator (a, b) and quad g: pixel wm0 + b*32 + l32,
    // channels wn0 + a*32 + 8g + 4*lh + {0,1,2,3}
    if (STAGED) {
        half_t* Cs = smem;                   // [BM][LDC]; all waves are past the last barrier
        const bool fuse_act = (p.res == nullptr);
#pragma unroll
        for (int a = 0; a < TNB; ++a)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int cl = wn0 + a * 32 + 8 * g + 4 * lh;
                float bv[4];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    bv[j] = (p.bias && (n0 + cl + j) < p.Cout) ? p.bias[n0 + cl + j] : 0.f;
#pragma unroll
                for (int b = 0; b < TMB; ++b) {
                    half4 h;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        float v = acc[a][b][4 * g + j] + bv[j];
                        if (fuse_act) v = apply_act(v, p.act);
                        h[j] = (half_t)v;
                    }
                    *(half4*)(Cs + (wm0 + b * 32 + l32) * LDC + cl) = h;
                }
            }
        __syncthreads();
        constexpr int CPR = BN / 8;          // 16-byte chunks per tile row
#pragma unroll
        for (int i = 0; i < BM * CPR / 256; ++i) {
            const int id = tid + i * 256;
            const int row = id / CPR, c8 = id - row * CPR;
            const int m = m0 + row, n = n0 + c8 * 8;
            if (m < p.M && n < p.Cout) {
                half8 v = *(const half8*)(Cs + row * LDC + c8 * 8);
                if (!fuse_act) {
                    const half8 rv = *(const half8*)(p.res + (long long)m * p.ldy + n);
#pragma unroll
                    for (int j = 0; j < 8; ++j) v[j] = (half_t)apply_act((float)v[j] + (float)rv[j], p.act);
                }
                *(half8*)((half_t*)p.y + (long long)m * p.ldy + n) = v;
            }
        }
    } else {
#pragma unroll
        for (int a = 0; a < TNB; ++a)
#pragma unroll
            for (int b = 0; b < TMB; ++b) {
                const int m = m0 + wm0 + b * 32 + l32;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int n = n0 + wn0 + a * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
                    if (m < p.M && n < p.Cout) {
                        float val = acc[a][b][v] + (p.bias ? p.bias[n] : 0.f);
                        if (p.res) val += (float)p.res[(long long)m * p.ldy + n];
                        val = apply_act(val, p.act);
                        if (p.out_f32) ((float*)p.y)[(long long)m * p.ldy + n] = val;
                        else ((half_t*)p.y)[(long long)m * p.ldy + n] = (half_t)val;
                    }
                }
            }
    }
}


// ------------------------------------------------------------------------------------------
// Deep-pipelined variant for the regular cases: dense 1x1 / GEMM, and filters whose channel count
// is a multiple of the 32-wide slice (so a slice never straddles two filter taps).
//
// The kernel above keeps one slice in flight per workgroup and spends most of its issue slots on
// per-lane gather arithmetic.  Here
//   - slices travel global -> LDS directly (buffer_load_dwordx4 ... lds: each lane names a 16-byte
//     chunk, the wave's 64 chunks land in 1 KB of consecutive LDS) through a ring of STAGES
//     buffers, STAGES-1 slices in flight, one barrier per slice;
//   - the address of a chunk is split into a per-lane part fixed for the whole kernel (pixel or
//     channel row, chunk within the slice) held in a VGPR, and a part that is the same for the
//     whole workgroup (filter tap, channel base of the slice) kept in a scalar register and
//     advanced by scalar instructions: a weight load costs no vector instruction at all, an input
//     load one bit test and one select;
//   - whether tap (r,s) of an output pixel falls inside the image is precomputed per lane as a bit
//     mask over the taps; a tap outside, a row beyond M or a channel beyond Cout gets the offset
//     0x80000000, which the buffer's range check turns into zeros in LDS (no stale data, no branch);
//   - the hardware fixes the LDS position of lane i's chunk, so the bank-conflict-avoiding layout
//     is obtained from the other side: rows are 64 bytes (4 chunks) and lane i fetches logical
//     chunk (i & 3) ^ ((i >> 4) & 3) of its row, i.e. LDS holds chunk c of row r at position
//     c ^ ((r >> 2) & 3); any 16 consecutive rows read at one logical chunk then touch 16
//     distinct 16-byte bank groups;
//   - the loads are issued from inline assembly so that the waits are ours: "all but the newest
//     STAGES-2 slices have landed" before the barrier, rather than a wait for everything.
typedef int intx4 __attribute__((ext_vector_type(4)));

constexpr unsigned OOB_OFFSET = 0x80000000u;       // beyond any buffer this kernel accepts

__device__ __forceinline__ intx4 make_rsrc(const void* base, unsigned bytes) {
    const unsigned long long a = (unsigned long long)base;
    intx4 r;
    r[0] = (int)(unsigned)a;
    r[1] = (int)((unsigned)(a >> 32) & 0xffffu);   // stride 0: raw buffer
    r[2] = (int)bytes;                              // num_records in bytes
    r[3] = 0x00020000;                              // 32-bit data format, offsets in bytes
    return r;
}

// One wave-wide transfer of 64 x 16 bytes: lane i's chunk at rsrc.base + voff + soff goes to
// LDS byte address lds_base + 16 i; lanes whose voff is out of range deposit zeros.
__device__ __forceinline__ void dma16(intx4 rsrc, unsigned voff, unsigned soff, unsigned lds_base) {
    const unsigned m0v = __builtin_amdgcn_readfirstlane(lds_base);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds" ::"s"(m0v), "v"(voff), "s"(rsrc), "s"(soff) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_loads_then_barrier() {
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

// Waves per SIMD that the LDS footprint of a tile configuration allows (the register allocator is asked
// for that many: left to itself it splits accumulators into AGPRs and loses waves for nothing).
template <int BM, int BN, int BK, int WGM, int WGN, int STAGES>
constexpr int dma_tile_waves_per_simd() {
    constexpr int ring = STAGES * (BM + BN) * BK * 2, ctile = BM * (BN + 8) * 2;
    constexpr int lds = (ring > ctile ? ring : ctile) + 1024;
    constexpr int blocks = 160 * 1024 / lds;
    constexpr int w = blocks * WGM * WGN / 4;
    return w < 1 ? 1 : (w > 8 ? 8 : w);
}

// KG > 1: the workgroup holds KG groups of WGM x WGN wavefronts, all on the same output tile; group g reduces the g-th
// part of the slices in a ring of its own, the groups step through their parts together (the barriers are the
// workgroup's), and at the end groups 1.. hand their partial sums to group 0 through LDS, which adds them in group
// order and finishes the tile.  A split reduction without a second launch, for the small batches where one more
// launch costs as much as the convolution.
template <int BM, int BN, int BK, int WGM, int WGN, int MODE, int STAGES, bool GELU, bool HOIST, bool DUAL = false, int KG = 1>
__global__ void __launch_bounds__(64 * WGM * WGN * KG, (KG > 1 ? WGM * WGN * KG / 4 : dma_tile_waves_per_simd<BM, BN, BK, WGM, WGN, STAGES>())) conv_igemm_dma_kernel(const ConvParams p) {
    static_assert(!DUAL || (MODE == MODE_1X1 && !HOIST && !GELU), "a second source belongs to a plain pointwise convolution");
    static_assert(KG == 1 || (!GELU && !DUAL && KG * STAGES * (BM + BN) * BK * 2 + 1024 <= 160 * 1024 && WGM * WGN * KG <= 16), "groups: LDS or workgroup limit");
    constexpr int CPRW = BK / 8;                       // 16-byte chunks per LDS row
    constexpr int RPI = 64 / CPRW;                     // rows covered by one wave-wide transfer
    constexpr int SWD = 16 / CPRW;                     // rows that share a bank window
    constexpr int NW = WGM * WGN, NT = 64 * NW;        // the waves form a WGM x WGN grid over the tile
    constexpr int TM = BM / WGM, TN = BN / WGN;
    constexpr int TMB = TM / 32, TNB = TN / 32;
    constexpr int XI = BM / (NW * RPI), WI = BN / (NW * RPI); // transfers per wave per slice
    static_assert((BK == 32 || BK == 64) && TM % 32 == 0 && TN % 32 == 0 && XI >= 1 && WI >= 1, "unsupported tile");
    constexpr int STAGE = (BM + BN) * BK;              // halfs per stage
    constexpr int LDC = BN + 8;
    static_assert(MODE == MODE_1X1 || MODE == MODE_GATHER8, "vector modes only");
    static_assert(STAGES >= 2 && STAGES * STAGE * 2 <= 160 * 1024 && BM * LDC * 2 <= 160 * 1024, "LDS limit");

    extern __shared__ __attribute__((aligned(1024))) half_t smem_all[];    // max(KG * STAGES * STAGE, BM * LDC) halfs
    const int group = KG > 1 ? __builtin_amdgcn_readfirstlane((int)threadIdx.x / NT) : 0;
    half_t* const smem = smem_all + group * (STAGES * STAGE);          // this group's ring
    const unsigned lds0 = (unsigned)(uintptr_t)smem;

    if (p.hp) __builtin_amdgcn_s_setprio(3);

    const int tid = (int)threadIdx.x - group * NT;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (wave % WGM) * TM, wn0 = (wave / WGM) * TN;
    const int l32 = lane & 31, lh = lane >> 5;

    const int tiles_n = (p.Cout + BN - 1) / BN;
    int logical;
    {
        const int nb = gridDim.x, b = blockIdx.x;
        const int per = nb >> 3, rem = nb & 7, xcd = b & 7, idx = b >> 3;
        logical = (xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per) + idx;
    }
    // split-K: the grid holds ksplit copies of the tile grid; copy z reduces slices [k_begin, k_end)
    int zsplit = 0, tile = logical;
    if (KG > 1) zsplit = group;
    else if (p.ksplit > 1) {
        const int ntiles = gridDim.x / p.ksplit;
        zsplit = logical / ntiles;
        tile = logical - zsplit * ntiles;
    }
    int tm;                                             // tiles_n is a power of two for every served layer
    if (p.tiles_n_shift >= 0) tm = tile >> p.tiles_n_shift; else tm = tile / tiles_n;
    const int m0 = tm * BM;
    const int n0 = (tile - tm * tiles_n) * BN;

    // The input buffer starts `lead` elements before x so that the per-lane offset of an output
    // pixel (its window's top-left tap, which may lie in the padding) is never negative.
    const long long lead = (long long)p.pad_h * p.sH + (long long)p.pad_w * p.sW;
    const intx4 xrsrc = make_rsrc(p.x - lead, (unsigned)((p.x_elems + lead) * 2));
    const intx4 wrsrc = make_rsrc(p.w, (unsigned)((long long)p.Cout * p.ldw * 2));

    // ---- per-lane constants: row (lane >> 2) of each 16-row group, logical chunk cl ---------------
    const int rsub = lane / CPRW;
    const int cl = (lane % CPRW) ^ (((wave * RPI + rsub) / SWD) & (CPRW - 1));
    unsigned xoff[XI], tapmask[XI];
#pragma unroll
    for (int j = 0; j < XI; ++j) {
        const int m = m0 + (j * NW + wave) * RPI + rsub;
        xoff[j] = OOB_OFFSET;
        tapmask[j] = 0xffffffffu;
        if (m < p.M) {
            if (MODE == MODE_1X1 && p.stride_h == 1) {
                xoff[j] = (unsigned)(((long long)m * p.sW + cl * 8) * 2);
            } else {
                const int n = m / p.PQ, rem = m - n * p.PQ;
                const int pp = rem / p.Q, qq = rem - pp * p.Q;
                const int ih0 = pp * p.stride_h - p.pad_h, iw0 = qq * p.stride_w - p.pad_w;
                xoff[j] = (unsigned)(((long long)n * p.sN + (long long)(pp * p.stride_h) * p.sH +
                                      (long long)(qq * p.stride_w) * p.sW + cl * 8) * 2);
                if (MODE == MODE_GATHER8) {
                    unsigned mask = 0;
                    for (int rr = 0; rr < p.R; ++rr)
                        for (int ss = 0; ss < p.S; ++ss)
                            if ((unsigned)(ih0 + rr) < (unsigned)p.H && (unsigned)(iw0 + ss) < (unsigned)p.W)
                                mask |= 1u << (rr * p.S + ss);
                    tapmask[j] = mask;
                }
            }
        }
    }
    // DUAL: the slices from p.C on come from the second tensor, addressed by output pixel with its own strides
    const intx4 xrsrc2 = DUAL ? make_rsrc(p.x2, (unsigned)(p.x2_elems * 2)) : xrsrc;
    unsigned xoff2[DUAL ? XI : 1];
    if (DUAL) {
#pragma unroll
        for (int j = 0; j < XI; ++j) {
            const int m = m0 + (j * NW + wave) * RPI + rsub;
            xoff2[j] = OOB_OFFSET;
            if (m < p.M) {
                const int n = m / p.PQ, rem = m - n * p.PQ;
                const int pp = rem / p.Q, qq = rem - pp * p.Q;
                xoff2[j] = (unsigned)(((long long)n * p.sN2 + (long long)(pp * p.stride2) * p.sH2 +
                                       (long long)(qq * p.stride2) * p.sW2 + cl * 8) * 2);
            }
        }
    }
    unsigned woff[WI];
#pragma unroll
    for (int j = 0; j < WI; ++j) {
        const int n = n0 + (j * NW + wave) * RPI + rsub;
        woff[j] = n < p.Cout ? (unsigned)(((long long)n * p.ldw + cl * 8) * 2) : OOB_OFFSET;
    }

    // ---- workgroup-uniform position of the slice being issued ---------------------------------
    const int nk_all = (p.Kg + BK - 1) / BK;
    const int kparts = KG > 1 ? KG : p.ksplit;
    const int kchunk = (nk_all + kparts - 1) / kparts;
    const int k_begin = zsplit * kchunk;
    const int k_end = k_begin + kchunk < nk_all ? k_begin + kchunk : nk_all;
    // (the groups of one workgroup share its barriers: all of them take kchunk steps, slices past a group's part arrive as zeros)
    const int nk = KG > 1 ? kchunk : (k_end > k_begin ? k_end - k_begin : 0);
    const bool ragged_k = (p.Kg & (BK - 1)) != 0;      // only possible for 1x1 / GEMM
    int ki = k_begin;                                  // slice index
    int tap = 0, ts = 0, cb = 0;                       // filter tap, its column, channel base
    unsigned tap_off = 0;                              // byte offset of the tap: (r*sH + s*sW) * 2
    if (MODE == MODE_GATHER8 && k_begin > 0) {
        const int per_tap = p.C / BK;
        tap = k_begin / per_tap;
        cb = (k_begin - tap * per_tap) * BK;
        const int r0 = tap / p.S;
        ts = tap - r0 * p.S;
        tap_off = (unsigned)(r0 * p.sH + ts * p.sW) * 2u;
    }
    const unsigned row_step = (unsigned)(p.sH - p.S * p.sW) * 2u;   // from the end of a filter row to the next

    auto issue = [&](int stage) {
        const unsigned sx = lds0 + (unsigned)(stage * STAGE) * 2u;
        const unsigned sw = sx + (unsigned)(BM * BK) * 2u;
        const bool live = ki < k_end;                  // slices past the end deposit zeros
        const bool second = DUAL && ki * BK >= p.C;   // workgroup-uniform
        const unsigned soff_x = MODE == MODE_1X1 ? (unsigned)(second ? ki * BK - p.C : ki * BK) * 2u : tap_off + (unsigned)cb * 2u;
#pragma unroll
        for (int j = 0; j < XI; ++j) {
            unsigned v = xoff[j];
            if (DUAL && second) v = xoff2[j];
            if (MODE == MODE_GATHER8) v = ((tapmask[j] >> tap) & 1u) ? v : OOB_OFFSET;
            if (MODE == MODE_1X1 && ragged_k) v = (ki * BK + cl * 8 < p.Kg) ? v : OOB_OFFSET;
            if (!live) v = OOB_OFFSET;
            dma16(second ? xrsrc2 : xrsrc, v, live ? soff_x : 0u, sx + (unsigned)((j * NW + wave) * 1024));
        }
#pragma unroll
        for (int j = 0; j < WI; ++j)
            dma16(wrsrc, live ? woff[j] : OOB_OFFSET, live ? (unsigned)ki * (BK * 2) : 0u, sw + (unsigned)((j * NW + wave) * 1024));
        ++ki;
        if (MODE == MODE_GATHER8) {
            cb += BK;
            if (cb >= p.C) {
                cb = 0;
                ++tap;
                tap_off += (unsigned)p.sW * 2u;
                if (++ts == p.S) { ts = 0; tap_off += row_step; }
            }
        }
    };

    floatx16 acc[TNB][TMB];
#pragma unroll
    for (int a = 0; a < TNB; ++a)
#pragma unroll
        for (int b = 0; b < TMB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    // The tile's bias row goes to LDS with the very first transfer (channels past Cout, or no bias at all,
    // arrive as zeros), so that the epilogue does not start with a round trip to L2.
    constexpr unsigned BIAS_LDS = (KG * STAGES * STAGE > BM * LDC ? KG * STAGES * STAGE : BM * LDC) * 2;   // byte offset
    static_assert(BN <= 256, "bias row: one transfer carries 256 floats");
    if (wave == 0) {                                   // (every group fetches it, so that the wavefronts' transfer counts agree)
        const intx4 brsrc = make_rsrc(p.bias, p.bias ? (unsigned)p.Cout * 4u : 0u);
        const int c = n0 + lane * 4;
        dma16(brsrc, (p.bias && lane * 4 < BN && c + 3 < p.Cout) ? (unsigned)c * 4u : OOB_OFFSET, 0u, (unsigned)(uintptr_t)smem_all + BIAS_LDS);
    }

#pragma unroll
    for (int i = 0; i < STAGES - 1; ++i) issue(i);

    // MFMA operand fragments are double-buffered in registers: the LDS reads of 16-wide step ks+1
    // are in flight while the MFMAs of step ks issue.
    const int swz = (l32 / SWD) & (CPRW - 1);
    constexpr int KS = BK / 16;
    int rd = 0, wr = STAGES - 1;
    for (int kt = 0; kt < nk; ++kt) {
        wait_loads_then_barrier<(STAGES - 2) * (XI + WI)>();   // slice kt has landed everywhere; buffer wr is free
        const half_t* Xs = smem + rd * STAGE;
        const half_t* Ws = Xs + BM * BK;
        half8 wf[2][TNB], xf[2][TMB];
        auto load_frags = [&](int buf, int ks) {
            const int pos = ((ks * 2 + lh) ^ swz) * 8;
#pragma unroll
            for (int a = 0; a < TNB; ++a) wf[buf][a] = *(const half8*)(Ws + (wn0 + a * 32 + l32) * BK + pos);
#pragma unroll
            for (int b = 0; b < TMB; ++b) xf[buf][b] = *(const half8*)(Xs + (wm0 + b * 32 + l32) * BK + pos);
        };
        load_frags(0, 0);
        issue(wr);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            // scheduling fences keep the reads of the next step ahead of this step's MFMAs; without
            // them the compiler sinks the reads below the MFMAs and folds the two buffers into one
            if (ks + 1 < KS) load_frags((ks + 1) & 1, ks + 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int a = 0; a < TNB; ++a)
#pragma unroll
                for (int b = 0; b < TMB; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wf[ks & 1][a], xf[ks & 1][b], acc[a][b], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        rd = rd + 1 == STAGES ? 0 : rd + 1;
        wr = wr + 1 == STAGES ? 0 : wr + 1;
    }
    wait_loads_then_barrier<0>();                      // trailing transfers have landed; LDS is free

    // ---- groups: partial sums of groups 1.. to group 0 through LDS, added in group order ----------------------
    if (KG > 1) {
        float* xch = (float*)smem_all;                 // [KG - 1][NW][TNB * TMB * 16][64 lanes]
        if (group > 0) {
            float* dst = xch + ((group - 1) * NW + wave) * (TNB * TMB * 16 * 64) + lane;
#pragma unroll
            for (int a = 0; a < TNB; ++a)
#pragma unroll
                for (int b = 0; b < TMB; ++b)
#pragma unroll
                    for (int v = 0; v < 16; ++v) dst[((a * TMB + b) * 16 + v) * 64] = acc[a][b][v];
        }
        __syncthreads();
        if (group == 0) {
            for (int g = 1; g < KG; ++g) {
                const float* src = xch + ((g - 1) * NW + wave) * (TNB * TMB * 16 * 64) + lane;
#pragma unroll
                for (int a = 0; a < TNB; ++a)
#pragma unroll
                    for (int b = 0; b < TMB; ++b)
#pragma unroll
                        for (int v = 0; v < 16; ++v) acc[a][b][v] += src[((a * TMB + b) * 16 + v) * 64];
            }
        }
        __syncthreads();                               // before the epilogue parks the output tile in the same memory
    }
    const bool finisher = KG == 1 || group == 0;       // the other groups only keep the epilogue's barrier company

    // ---- split-K: fp32 partial sums to this copy's slab; a second kernel reduces and finishes ------
    if (p.ksplit > 1) {
        float* slab = p.ws + (long long)zsplit * p.M * p.Cout;
#pragma unroll
        for (int a = 0; a < TNB; ++a)
#pragma unroll
            for (int b = 0; b < TMB; ++b) {
                const int m = m0 + wm0 + b * 32 + l32;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int n = n0 + wn0 + a * 32 + 8 * g + 4 * lh;
                    if (m < p.M && n < p.Cout) {
                        float4 v = make_float4(acc[a][b][4 * g], acc[a][b][4 * g + 1], acc[a][b][4 * g + 2], acc[a][b][4 * g + 3]);
                        *(float4*)(slab + (long long)m * p.Cout + n) = v;
                    }
                }
            }
        return;
    }

    // ---- epilogue (same as the first kernel's staged path) --------------------------------------
    // ReLU / ReLU6 / none are one clamp with workgroup-uniform bounds; GELU is a separate instantiation
    // The epilogue's arithmetic after the bias is done on packed fp16 pairs: adding two fp16 numbers, or
    // clamping one against 0, 6 or an infinity, gives the same fp16 result whether it is done in fp16 or
    // in fp32 and then rounded, and it takes a quarter of the instructions (short-reduction layers spend
    // most of their instructions here).  Bias and residual are fetched where they are used: holding
    // them across the reduction would cost a wave per SIMD in registers.  Layers that add a residual
    // (HOIST) request it right after the reduction, before the staging barrier: that takes its latency
    // off the path between the last MFMA and the stores.
    constexpr int CPR = BN / 8, NCH = BM * CPR / NT;
    half_t* Cs = smem_all;
    const bool fuse_act = (p.res == nullptr);
    const half_t lo = (p.act == ACT_RELU || p.act == ACT_RELU6) ? (half_t)0.f : (half_t)-INFINITY;
    const half_t hi = p.act == ACT_RELU6 ? (half_t)6.f : (half_t)INFINITY;
    const half_t lo1 = fuse_act ? lo : (half_t)-INFINITY, hi1 = fuse_act ? hi : (half_t)INFINITY;
    const half4 lo4 = {lo1, lo1, lo1, lo1}, hi4 = {hi1, hi1, hi1, hi1};
    const half8 lo8 = {lo, lo, lo, lo, lo, lo, lo, lo}, hi8 = {hi, hi, hi, hi, hi, hi, hi, hi};
    auto residual_chunk = [&](int i) {
        const int id = tid + i * NT;
        const int row = id / CPR, c8 = id - row * CPR;
        const int m = m0 + row, n = n0 + c8 * 8;
        half8 r;
#pragma unroll
        for (int j = 0; j < 8; ++j) r[j] = (half_t)0.f;
        if (m < p.M && n < p.Cout) r = *(const half8*)(p.res + (long long)m * p.ldy + n);
        return r;
    };
    const float* bias_s = (const float*)((const char*)smem_all + BIAS_LDS);
    auto bias4 = [&](int a, int g, float (&bv)[4]) {
        const float4 b4 = *(const float4*)(bias_s + wn0 + a * 32 + 8 * g + 4 * lh);
        bv[0] = b4.x; bv[1] = b4.y; bv[2] = b4.z; bv[3] = b4.w;
    };
    half8 rv[HOIST ? NCH : 1];
    if (HOIST && !fuse_act && finisher) {
#pragma unroll
        for (int i = 0; i < NCH; ++i) rv[i] = residual_chunk(i);
    }
    if (finisher)
#pragma unroll
    for (int a = 0; a < TNB; ++a)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int cn = wn0 + a * 32 + 8 * g + 4 * lh;
            float bv[4];
            bias4(a, g, bv);
#pragma unroll
            for (int b = 0; b < TMB; ++b) {
                half4 h;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    float v = acc[a][b][4 * g + j] + bv[j];
                    if (GELU) v = gelu_f(v);
                    h[j] = (half_t)v;
                }
                h = __builtin_elementwise_min(__builtin_elementwise_max(h, lo4), hi4);
                *(half4*)(Cs + (wm0 + b * 32 + l32) * LDC + cn) = h;
            }
        }
    __syncthreads();
    if (!finisher) return;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int id = tid + i * NT;
        const int row = id / CPR, c8 = id - row * CPR;
        const int m = m0 + row, n = n0 + c8 * 8;
        if (m < p.M && n < p.Cout) {
            half8 v = *(const half8*)(Cs + row * LDC + c8 * 8);
            if (!fuse_act) {
                const half8 r = HOIST ? rv[i] : residual_chunk(i);
                v = __builtin_elementwise_min(__builtin_elementwise_max(v + r, lo8), hi8);
            }
            *(half8*)((half_t*)p.y + (long long)m * p.ldy + n) = v;
        }
    }
}

// Second pass of a split-K launch: y = act(sum_z slab_z + bias (+ res)), 8 channels per thread,
// slabs summed in a fixed order so that results do not depend on scheduling.
__global__ void __launch_bounds__(256) splitk_finish_kernel(const ConvParams p) {
    if (p.hp) __builtin_amdgcn_s_setprio(3);
    const int c8n = p.Cout >> 3;
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= (long long)p.M * c8n) return;
    const int m = (int)(i / c8n), n = (int)(i - (long long)m * c8n) * 8;
    float v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = p.bias ? p.bias[n + j] : 0.f;
    const long long slab = (long long)p.M * p.Cout;
    const float* src = p.ws + (long long)m * p.Cout + n;
    // The slabs are fetched several at a time and added in slab order: one load per trip of a loop whose length the
    // compiler does not know costs a trip to L2 per slab (a 32-way split: 11 us for this kernel against 4).
    auto add_slabs = [&](int z0, auto nconst) {
        constexpr int NB = decltype(nconst)::value;
        float4 lo[NB], hi[NB];
#pragma unroll
        for (int u = 0; u < NB; ++u) { lo[u] = *(const float4*)(src + (z0 + u) * slab); hi[u] = *(const float4*)(src + (z0 + u) * slab + 4); }
#pragma unroll
        for (int u = 0; u < NB; ++u) { v[0] += lo[u].x; v[1] += lo[u].y; v[2] += lo[u].z; v[3] += lo[u].w; v[4] += hi[u].x; v[5] += hi[u].y; v[6] += hi[u].z; v[7] += hi[u].w; }
    };
    int z = 0;
    for (; z + 8 <= p.ksplit; z += 8) add_slabs(z, std::integral_constant<int, 8>());
    if (z + 4 <= p.ksplit) { add_slabs(z, std::integral_constant<int, 4>()); z += 4; }
    if (z + 2 <= p.ksplit) { add_slabs(z, std::integral_constant<int, 2>()); z += 2; }
    if (z < p.ksplit) add_slabs(z, std::integral_constant<int, 1>());
    if (p.res) {
        const half8 r = *(const half8*)(p.res + (long long)m * p.ldy + n);
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] += (float)r[j];
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = apply_act(v[j], p.act);
    if (p.out_f32) {
        float* dst = (float*)p.y + (long long)m * p.ldy + n;
        *(float4*)dst = make_float4(v[0], v[1], v[2], v[3]);
        *(float4*)(dst + 4) = make_float4(v[4], v[5], v[6], v[7]);
    } else {
        half8 o;
#pragma unroll
        for (int j = 0; j < 8; ++j) o[j] = (half_t)v[j];
        *(half8*)((half_t*)p.y + (long long)m * p.ldy + n) = o;
    }
}

// ------------------------------------------------------------------------------------------
// 3x3, stride 1, padding 1, from an input patch held in LDS.
//
// The kernel above fetches every input pixel nine times, once per filter tap; on the wide early layers that
// traffic between L2 and LDS, not the MFMAs, sets the pace.  Here pixels are numbered in a bordered space: every
// image row is preceded by one border slot and every image by one border row, v = (n (H+1) + y) (W+1) + x for
// output (n, y, x), and the slot with number u holds input pixel (u's row - 1, u's column - 1) or, in the border,
// zero.  A row's right border is the next row's left border and an image's bottom border row the next image's top
// one, so one slot per row and one row per image suffice.  Tap (r, s) of output v then reads slot
// v + r (W+1) + s: one offset per tap for the whole tile.  A workgroup owns BM consecutive v (the one in W+1 with
// x = W and the one row in H+1 with y = H are computed and never stored) and BN output channels.  Per
// 32-channel slice of the input it holds the BM + 2 (W+1) + 2 slots its taps touch (64 bytes each; border slots
// arrive as zeros from out-of-range transfers) and feeds all nine taps' MFMAs from them; only the weights, one
// 32-channel slice of one tap at a time, stream through a three-stage ring.  The patch of the next slice arrives
// in a second buffer during the first seven tap steps of the current one.  Per tap step every wave issues a
// fixed number of transfers, so the in-order load counter tells when a given stage has landed.  LDS rows of 64
// bytes are swizzled as in the kernel above (16-byte chunk c of row i sits at c ^ ((i >> 2) & 3)), which keeps
// the operand reads conflict free for any run of consecutive rows, i.e. for every tap offset.
__device__ __forceinline__ void divmod_f(int v, int d, float rcp, int& q, int& r) {   // exact for 0 <= v < 2^24
    q = (int)((float)v * rcp);
    r = v - q * d;
    if (r < 0) { --q; r += d; }
    if (r >= d) { ++q; r -= d; }
}
constexpr int patch_share(int npw, int as, int t) { return npw - t * as < 0 ? 0 : (npw - t * as > as ? as : npw - t * as); }

constexpr int patch_wait(int npw, int as, int wi, int pre, int t) {     // transfers a wave may have in flight when tap step t starts
    int n = patch_share(npw, as, (t + 9 - pre) % 9);
    for (int k = 1; k < pre; ++k) n += wi + patch_share(npw, as, (t + 9 - k) % 9);
    return n;
}

template <int BM, int BN, int WGM, int WGN, int NPW, int NBS>
__global__ void __launch_bounds__(64 * WGM * WGN, WGM * WGN / 2) conv3x3_patch_kernel(const ConvParams p) {
    constexpr int NW = WGM * WGN, NT = 64 * NW;
    static_assert((NW == 4 || NW == 8) && BM % (32 * WGM) == 0 && BN % (32 * WGN) == 0 && BN % (16 * NW) == 0, "unsupported tile");
    constexpr int TM = BM / WGM, TN = BN / WGN, TMB = TM / 32, TNB = TN / 32;
    constexpr int WI = BN / (NW * 16);                 // weight transfers per wave per tap step
    constexpr int PRE = NBS - 1;                       // weight stages in flight ahead of the one in use
    constexpr int AS = (NPW + 8 - PRE) / (9 - PRE);    // patch transfers per wave per tap step (steps 0..8-PRE)
    static_assert(NBS >= 3 && NBS <= 8, "ring depth");
    constexpr int PATCH = NPW * NW * 1024;             // bytes of one patch buffer: NPW * 64 pixels
    constexpr int WSTAGE = BN * 64;                    // bytes of one weight stage
    constexpr int RING = 2 * PATCH + NBS * WSTAGE;
    constexpr int LDC = BN + 8;
    constexpr int CT = BM * LDC * 2;
    constexpr unsigned BIAS_LDS = RING > CT ? RING : CT;
    static_assert(BIAS_LDS + 1024 <= 160 * 1024, "LDS limit");

    extern __shared__ __attribute__((aligned(1024))) half_t smem[];
    const unsigned lds0 = (unsigned)(uintptr_t)smem;
    if (p.hp) __builtin_amdgcn_s_setprio(3);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (wave % WGM) * TM, wn0 = (wave / WGM) * TN;
    const int l32 = lane & 31, lh = lane >> 5;

    const int tiles_n = p.Cout / BN;
    int tile;
    {
        const int nb = gridDim.x, b = blockIdx.x;
        const int per = nb >> 3, rem = nb & 7, xcd = b & 7, idx = b >> 3;
        tile = (xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per) + idx;
    }
    const int tm = tile / tiles_n;
    const int m0 = tm * BM, n0 = (tile - tm * tiles_n) * BN;

    // rows wider than 64 pixels are cut into strips, each numbered as an image of its own with a border slot on
    // either side that holds the neighbouring strip's pixel (zero only at the true edges), so those are not shared
    const int SW = p.strip_w, NS = __builtin_amdgcn_readfirstlane(p.W / SW);
    const int Wp = SW + (NS == 1 ? 1 : 2), HpWp = (p.H + 1) * Wp, NI = (p.M / p.PQ) * NS;   // borders shared between neighbours
    const float rcp_w = 1.f / (float)Wp, rcp_i = 1.f / (float)HpWp, rcp_s = 1.f / (float)NS;
    const intx4 xrsrc = make_rsrc(p.x, (unsigned)(p.x_elems * 2));
    const intx4 wrsrc = make_rsrc(p.w, (unsigned)((long long)p.Cout * p.ldw * 2));

    // ---- per-lane source offsets: patch pixel (16 per transfer, 4 chunks each), weight row ----------
    unsigned aoff[NPW];
#pragma unroll
    for (int j = 0; j < NPW; ++j) {
        const int pp = (j * NW + wave) * 16 + (lane >> 2);
        int img, rem, yp, xp, n, st;
        divmod_f(m0 + pp, HpWp, rcp_i, img, rem);
        divmod_f(rem, Wp, rcp_w, yp, xp);
        divmod_f(img, NS, rcp_s, n, st);
        const int xr = st * SW + xp - 1;
        const int lc = (lane & 3) ^ ((pp >> 2) & 3);
        const bool inside = img < NI && yp >= 1 && yp <= p.H && xr >= 0 && xr < p.W;
        aoff[j] = inside ? (unsigned)(((long long)n * p.sN + (long long)(yp - 1) * p.sH + (long long)xr * p.sW + lc * 8) * 2) : OOB_OFFSET;
    }
    unsigned woff[WI];
#pragma unroll
    for (int j = 0; j < WI; ++j) {
        const int row = (j * NW + wave) * 16 + (lane >> 2);
        const int lc = (lane & 3) ^ ((row >> 2) & 3);
        woff[j] = n0 + row < p.Cout ? (unsigned)(((long long)(n0 + row) * p.ldw + lc * 8) * 2) : OOB_OFFSET;
    }
    const int ncs = p.C >> 5;
    auto issue_w = [&](int stage, int tap, int cs) {
        const bool live = cs < ncs;
        const unsigned soff = live ? (unsigned)(tap * p.C + cs * 32) * 2u : 0u;
#pragma unroll
        for (int j = 0; j < WI; ++j)
            dma16(wrsrc, live ? woff[j] : OOB_OFFSET, soff, lds0 + (unsigned)(2 * PATCH + stage * WSTAGE + (j * NW + wave) * 1024));
    };
    auto issue_a = [&](int buf, int j, int cs) {
        const bool live = cs < ncs;
        dma16(xrsrc, live ? aoff[j] : OOB_OFFSET, live ? (unsigned)cs * 64u : 0u, lds0 + (unsigned)(buf * PATCH + (j * NW + wave) * 1024));
    };

    floatx16 acc[TNB][TMB];
#pragma unroll
    for (int a = 0; a < TNB; ++a)
#pragma unroll
        for (int b = 0; b < TMB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    static_assert(BN <= 256, "bias row: one transfer carries 256 floats");
    if (wave == 0) {
        const intx4 brsrc = make_rsrc(p.bias, p.bias ? (unsigned)p.Cout * 4u : 0u);
        const int c = n0 + lane * 4;
        dma16(brsrc, (p.bias && lane * 4 < BN && c + 3 < p.Cout) ? (unsigned)c * 4u : OOB_OFFSET, 0u, lds0 + BIAS_LDS);
    }
#pragma unroll
    for (int j = 0; j < NPW; ++j) issue_a(0, j, 0);
#pragma unroll
    for (int t = 0; t < PRE; ++t) issue_w(t, t, 0);    // PRE < 9: all in the first slice
    int rd = 0, wr = PRE;                              // ring stage in use, stage being filled

    const unsigned wrow = (unsigned)((lh ^ ((l32 >> 2) & 3)) << 4);   // chunk lh of weight row l32 (+ multiples of 32 rows)
    for (int cs = 0; cs < ncs; ++cs) {
        const char* Pa = (const char*)smem + (cs & 1) * PATCH;
        const int nbuf = (cs + 1) & 1;
        int wp_l = Wp;                                 // opaque per iteration: keeps the nine taps' operand addresses from being
        asm volatile("" : "+s"(wp_l));                 // hoisted out of the loop, where they would cost eighteen registers
#define STRAIT_TAP_STEP(T)                                                                                              \
        {                                                                                                               \
            wait_loads_then_barrier<patch_wait(NPW, AS, WI, PRE, T)>();                                                  \
            const char* Ws = (const char*)smem + 2 * PATCH + rd * WSTAGE;                                               \
            const int tapoff = (T / 3) * wp_l + (T % 3);                                                                 \
            unsigned a0[TMB];                                                                                           \
            _Pragma("unroll") for (int b = 0; b < TMB; ++b) {                                                           \
                const unsigned pp = (unsigned)(wm0 + b * 32 + l32 + tapoff);                                            \
                a0[b] = pp * 64u + (((lh ^ (pp >> 2)) & 3u) << 4);                                                      \
            }                                                                                                           \
            half8 wf[2][TNB], xf[2][TMB];                                                                               \
            _Pragma("unroll") for (int a = 0; a < TNB; ++a) wf[0][a] = *(const half8*)(Ws + (wn0 + a * 32 + l32) * 64 + wrow); \
            _Pragma("unroll") for (int b = 0; b < TMB; ++b) xf[0][b] = *(const half8*)(Pa + a0[b]);                     \
            issue_w(wr, (T + PRE) % 9, cs + (T + PRE) / 9);                                                             \
            rd = rd + 1 == NBS ? 0 : rd + 1;                                                                            \
            wr = wr + 1 == NBS ? 0 : wr + 1;                                                                            \
            _Pragma("unroll") for (int j = T * AS; j < (T + 1) * AS && j < NPW; ++j) issue_a(nbuf, j, cs + 1);          \
            _Pragma("unroll") for (int a = 0; a < TNB; ++a) wf[1][a] = *(const half8*)(Ws + (((wn0 + a * 32 + l32) * 64 + wrow) ^ 32u)); \
            _Pragma("unroll") for (int b = 0; b < TMB; ++b) xf[1][b] = *(const half8*)(Pa + (a0[b] ^ 32u));             \
            __builtin_amdgcn_sched_barrier(0);                                                                          \
            _Pragma("unroll") for (int ks = 0; ks < 2; ++ks)                                                            \
                _Pragma("unroll") for (int a = 0; a < TNB; ++a)                                                         \
                    _Pragma("unroll") for (int b = 0; b < TMB; ++b)                                                     \
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wf[ks][a], xf[ks][b], acc[a][b], 0, 0, 0);   \
            __builtin_amdgcn_sched_barrier(0);                                                                          \
        }
        STRAIT_TAP_STEP(0) STRAIT_TAP_STEP(1) STRAIT_TAP_STEP(2) STRAIT_TAP_STEP(3) STRAIT_TAP_STEP(4)
        STRAIT_TAP_STEP(5) STRAIT_TAP_STEP(6) STRAIT_TAP_STEP(7) STRAIT_TAP_STEP(8)
#undef STRAIT_TAP_STEP
    }
    wait_loads_then_barrier<0>();                      // trailing (empty) transfers have landed; LDS is free

    // ---- epilogue: bias, clamp, tile parked in LDS as [pixel][channel], 16-byte row segments out ----
    half_t* Cs = smem;
    const half_t lo = (p.act == ACT_RELU || p.act == ACT_RELU6) ? (half_t)0.f : (half_t)-INFINITY;
    const half_t hi = p.act == ACT_RELU6 ? (half_t)6.f : (half_t)INFINITY;
    const half4 lo4 = {lo, lo, lo, lo}, hi4 = {hi, hi, hi, hi};
    const float* bias_s = (const float*)((const char*)smem + BIAS_LDS);
#pragma unroll
    for (int a = 0; a < TNB; ++a)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int cn = wn0 + a * 32 + 8 * g + 4 * lh;
            const float4 b4 = *(const float4*)(bias_s + cn);
            const float bv[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
            for (int b = 0; b < TMB; ++b) {
                half4 h;
#pragma unroll
                for (int j = 0; j < 4; ++j) h[j] = (half_t)(acc[a][b][4 * g + j] + bv[j]);
                h = __builtin_elementwise_min(__builtin_elementwise_max(h, lo4), hi4);
                *(half4*)(Cs + (wm0 + b * 32 + l32) * LDC + cn) = h;
            }
        }
    __syncthreads();
    constexpr int CPR = BN / 8, NCH = BM * CPR / NT;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int id = tid + i * NT;
        const int row = id / CPR, c8 = id - row * CPR;
        int img, rem, yy, xx, n, st;
        divmod_f(m0 + row, HpWp, rcp_i, img, rem);
        divmod_f(rem, Wp, rcp_w, yy, xx);
        divmod_f(img, NS, rcp_s, n, st);
        if (img < NI && yy < p.H && xx < SW) {
            const half8 v = *(const half8*)(Cs + row * LDC + c8 * 8);
            *(half8*)((half_t*)p.y + ((long long)(n * p.H + yy) * p.W + st * SW + xx) * p.ldy + n0 + c8 * 8) = v;
        }
    }
}

// The same computation for layers whose tiles are short (one to four input slices: the eighteen tap steps of a
// 64-channel layer take about as long as setting a tile up and putting it away).  Half as many workgroups as the
// compute units hold at a time are launched, and each walks over every gridDim.x-th tile: the next tile's first patch
// and first weights arrive during the last slice of the current one, in the buffers that slice no longer reads, and the
// finished tile leaves straight from the accumulators (8 bytes per lane and store), so that no LDS is tied up and no
// barrier separates two tiles.  All output channels in one tile (Cout == BN): weight offsets and the bias row stay put.
// Stores count in the same counter as the transfers.  The waits of the tap steps are not adjusted for them: a wait
// that allows the n newest requests in flight then also waits for stores issued before those, which costs the first
// steps of a tile a little time (counting them in was worth 1 us in 50) and never lets a transfer be read early.
template <int BM, int BN, int WGM, int WGN, int NPW, int NBS>
__global__ void __launch_bounds__(64 * WGM * WGN, WGM * WGN / 2) conv3x3_patch_walk_kernel(const ConvParams p, const int tiles) {
    constexpr int NW = WGM * WGN;
    static_assert((NW == 4 || NW == 8) && BM % (32 * WGM) == 0 && BN % (32 * WGN) == 0 && BN % (16 * NW) == 0, "unsupported tile");
    constexpr int TM = BM / WGM, TN = BN / WGN, TMB = TM / 32, TNB = TN / 32;
    constexpr int WI = BN / (NW * 16);
    constexpr int PRE = NBS - 1;
    constexpr int AS = (NPW + 8 - PRE) / (9 - PRE);
    static_assert(NBS >= 3 && NBS <= 8, "ring depth");
    constexpr int PATCH = NPW * NW * 1024;
    constexpr int WSTAGE = BN * 64;
    constexpr int RING = 2 * PATCH + NBS * WSTAGE;
    static_assert(RING + 1024 <= 160 * 1024 && BN <= 256, "LDS limit; one transfer carries the bias row");

    extern __shared__ __attribute__((aligned(1024))) half_t smem[];
    const unsigned lds0 = (unsigned)(uintptr_t)smem;
    if (p.hp) __builtin_amdgcn_s_setprio(3);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (wave % WGM) * TM, wn0 = (wave / WGM) * TN;
    const int l32 = lane & 31, lh = lane >> 5;

    const int SW = p.strip_w, NS = __builtin_amdgcn_readfirstlane(p.W / SW);
    const int Wp = SW + (NS == 1 ? 1 : 2), HpWp = (p.H + 1) * Wp, NI = (p.M / p.PQ) * NS;
    const float rcp_w = 1.f / (float)Wp, rcp_i = 1.f / (float)HpWp, rcp_s = 1.f / (float)NS;
    const intx4 xrsrc = make_rsrc(p.x, (unsigned)(p.x_elems * 2));
    const intx4 wrsrc = make_rsrc(p.w, (unsigned)((long long)p.Cout * p.ldw * 2));

    // virtual workgroup v -> tile: the hardware deals consecutive workgroups to the eight XCDs in turn, and gridDim.x is a
    // multiple of eight, so v mod 8 is this workgroup's XCD for every v it takes; each XCD gets a contiguous range of tiles
    auto tile_m0 = [&](int v) __attribute__((always_inline)) -> int {
        const int per = tiles >> 3, rem = tiles & 7, xcd = v & 7, idx = v >> 3;
        return ((xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per) + idx) * BM;
    };
    auto patch_offsets = [&](int m0, bool live, unsigned (&ao)[NPW]) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < NPW; ++j) {
            const int pp = (j * NW + wave) * 16 + (lane >> 2);
            int img, rem, yp, xp, n, st;
            divmod_f(m0 + pp, HpWp, rcp_i, img, rem);
            divmod_f(rem, Wp, rcp_w, yp, xp);
            divmod_f(img, NS, rcp_s, n, st);
            const int xr = st * SW + xp - 1;
            const int lc = (lane & 3) ^ ((pp >> 2) & 3);
            const bool inside = live && img < NI && yp >= 1 && yp <= p.H && xr >= 0 && xr < p.W;
            ao[j] = inside ? (unsigned)(((long long)n * p.sN + (long long)(yp - 1) * p.sH + (long long)xr * p.sW + lc * 8) * 2) : OOB_OFFSET;
        }
    };
    unsigned woff[WI];
#pragma unroll
    for (int j = 0; j < WI; ++j) {
        const int row = (j * NW + wave) * 16 + (lane >> 2);
        const int lc = (lane & 3) ^ ((row >> 2) & 3);
        woff[j] = row < p.Cout ? (unsigned)(((long long)row * p.ldw + lc * 8) * 2) : OOB_OFFSET;
    }
    const int ncs = p.C >> 5;
    auto issue_w = [&](int stage, int tap, int cs, bool live) __attribute__((always_inline)) {
        const unsigned soff = live ? (unsigned)(tap * p.C + cs * 32) * 2u : 0u;
#pragma unroll
        for (int j = 0; j < WI; ++j)
            dma16(wrsrc, live ? woff[j] : OOB_OFFSET, soff, lds0 + (unsigned)(2 * PATCH + stage * WSTAGE + (j * NW + wave) * 1024));
    };

    floatx16 acc[TNB][TMB];
#pragma unroll
    for (int a = 0; a < TNB; ++a)
#pragma unroll
        for (int b = 0; b < TMB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    if (wave == 0) {                                   // the oldest transfer: every later wait covers it
        const intx4 brsrc = make_rsrc(p.bias, p.bias ? (unsigned)p.Cout * 4u : 0u);
        const int c = lane * 4;
        dma16(brsrc, (p.bias && c < BN && c + 3 < p.Cout) ? (unsigned)c * 4u : OOB_OFFSET, 0u, lds0 + RING);
    }
    const int G = (int)gridDim.x;
    int vb = (int)blockIdx.x;
    int m0 = tile_m0(vb);
    unsigned aoff[NPW], anext[NPW];
    patch_offsets(m0, true, aoff);
#pragma unroll
    for (int j = 0; j < NPW; ++j) dma16(xrsrc, aoff[j], 0u, lds0 + (unsigned)((j * NW + wave) * 1024));
#pragma unroll
    for (int t = 0; t < PRE; ++t) issue_w(t, t, 0, true);
    int rd = 0, wr = PRE, par = 0;

    const half_t lo = (p.act == ACT_RELU || p.act == ACT_RELU6) ? (half_t)0.f : (half_t)-INFINITY;
    const half_t hi = p.act == ACT_RELU6 ? (half_t)6.f : (half_t)INFINITY;
    const half4 lo4 = {lo, lo, lo, lo}, hi4 = {hi, hi, hi, hi};
    const float* bias_s = (const float*)((const char*)smem + RING);
    const unsigned wrow = (unsigned)((lh ^ ((l32 >> 2) & 3)) << 4);

    for (;;) {
        const int vnext = vb + G;
        const bool has_next = vnext < tiles;
        const int m0n = has_next ? tile_m0(vnext) : 0;
        patch_offsets(m0n, has_next, anext);
        for (int cs = 0; cs < ncs; ++cs) {
            const bool wrap = cs + 1 == ncs;           // the slice after this one is the next tile's first
            const int csn = wrap ? 0 : cs + 1;
            const bool nlive = !wrap || has_next;
            unsigned asrc[NPW];
#pragma unroll
            for (int j = 0; j < NPW; ++j) asrc[j] = wrap ? anext[j] : aoff[j];
            const char* Pa = (const char*)smem + par * PATCH;
            const unsigned nbuf = lds0 + (unsigned)((par ^ 1) * PATCH);
            int wp_l = Wp;
            asm volatile("" : "+s"(wp_l));
#define STRAIT_WALK_STEP(T)                                                                                             \
            {                                                                                                           \
                wait_loads_then_barrier<patch_wait(NPW, AS, WI, PRE, T)>();                                              \
                const char* Ws = (const char*)smem + 2 * PATCH + rd * WSTAGE;                                           \
                const int tapoff = (T / 3) * wp_l + (T % 3);                                                             \
                unsigned a0[TMB];                                                                                       \
                _Pragma("unroll") for (int b = 0; b < TMB; ++b) {                                                       \
                    const unsigned pp = (unsigned)(wm0 + b * 32 + l32 + tapoff);                                        \
                    a0[b] = pp * 64u + (((lh ^ (pp >> 2)) & 3u) << 4);                                                  \
                }                                                                                                       \
                half8 wf[2][TNB], xf[2][TMB];                                                                           \
                _Pragma("unroll") for (int a = 0; a < TNB; ++a) wf[0][a] = *(const half8*)(Ws + (wn0 + a * 32 + l32) * 64 + wrow); \
                _Pragma("unroll") for (int b = 0; b < TMB; ++b) xf[0][b] = *(const half8*)(Pa + a0[b]);                 \
                if (T + PRE < 9) issue_w(wr, T + PRE, cs, true); else issue_w(wr, T + PRE - 9, csn, nlive);             \
                rd = rd + 1 == NBS ? 0 : rd + 1;                                                                        \
                wr = wr + 1 == NBS ? 0 : wr + 1;                                                                        \
                _Pragma("unroll") for (int j = T * AS; j < (T + 1) * AS && j < NPW; ++j)                                \
                    dma16(xrsrc, asrc[j], (unsigned)csn * 64u, nbuf + (unsigned)((j * NW + wave) * 1024));             \
                _Pragma("unroll") for (int a = 0; a < TNB; ++a) wf[1][a] = *(const half8*)(Ws + (((wn0 + a * 32 + l32) * 64 + wrow) ^ 32u)); \
                _Pragma("unroll") for (int b = 0; b < TMB; ++b) xf[1][b] = *(const half8*)(Pa + (a0[b] ^ 32u));         \
                __builtin_amdgcn_sched_barrier(0);                                                                      \
                _Pragma("unroll") for (int ks = 0; ks < 2; ++ks)                                                        \
                    _Pragma("unroll") for (int a = 0; a < TNB; ++a)                                                     \
                        _Pragma("unroll") for (int b = 0; b < TMB; ++b)                                                 \
                            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wf[ks][a], xf[ks][b], acc[a][b], 0, 0, 0); \
                __builtin_amdgcn_sched_barrier(0);                                                                      \
            }
            STRAIT_WALK_STEP(0) STRAIT_WALK_STEP(1) STRAIT_WALK_STEP(2) STRAIT_WALK_STEP(3) STRAIT_WALK_STEP(4)
            STRAIT_WALK_STEP(5) STRAIT_WALK_STEP(6) STRAIT_WALK_STEP(7) STRAIT_WALK_STEP(8)
#undef STRAIT_WALK_STEP
            par ^= 1;
        }
        // ---- the tile leaves from the registers: lane (l32, lh) holds channels 8 g + 4 lh + (0..3) of pixel l32 per 32 x 32 block
        long long ybase[TMB];                          // this lane's pixel in y, in elements; -1: a border slot, nothing to store
#pragma unroll
        for (int b = 0; b < TMB; ++b) {
            int img, rem, yy, xx, n, st;
            divmod_f(m0 + wm0 + b * 32 + l32, HpWp, rcp_i, img, rem);
            divmod_f(rem, Wp, rcp_w, yy, xx);
            divmod_f(img, NS, rcp_s, n, st);
            ybase[b] = (img < NI && yy < p.H && xx < SW) ? ((long long)(n * p.H + yy) * p.W + st * SW + xx) * p.ldy : -1;
        }
#pragma unroll
        for (int a = 0; a < TNB; ++a)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int cn = wn0 + a * 32 + 8 * g + 4 * lh;
                const float4 b4 = *(const float4*)(bias_s + cn);
                const float bv[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
                for (int b = 0; b < TMB; ++b) {
                    half4 h;
#pragma unroll
                    for (int j = 0; j < 4; ++j) { h[j] = (half_t)(acc[a][b][4 * g + j] + bv[j]); acc[a][b][4 * g + j] = 0.f; }
                    h = __builtin_elementwise_min(__builtin_elementwise_max(h, lo4), hi4);
                    if (ybase[b] >= 0) *(half4*)((half_t*)p.y + ybase[b] + cn) = h;
                }
            }
        if (!has_next) break;
        vb = vnext;
        m0 = m0n;
#pragma unroll
        for (int j = 0; j < NPW; ++j) aoff[j] = anext[j];
    }
    wait_loads_then_barrier<0>();                      // trailing (empty) transfers have landed
}

template <int BM, int BN, int WGM, int WGN, int NPW, int NBS>
static int launch_patch_walk(const ConvParams& p, long long mv, hipStream_t stream) {
    constexpr int NW = WGM * WGN;
    const long long tiles = (mv + BM - 1) / BM;
    if (p.Cout != BN || tiles < 512 || tiles > 0x7fffffffLL) { set_error("conv: bad grid (%lld tiles)", tiles); return -5; }
    constexpr unsigned lds = 2 * NPW * NW * 1024 + NBS * BN * 64 + 1024;
    static_assert(2 * (lds + 1024) <= 160 * 1024, "two workgroups per compute unit");
    auto kernel = conv3x3_patch_walk_kernel<BM, BN, WGM, WGN, NPW, NBS>;
    static std::atomic<bool> configured{false};
    if (!configured.load(std::memory_order_acquire) && lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) { set_error("conv: cannot reserve %u bytes of LDS: %s", lds, hipGetErrorString(e)); return -2; }
    }
    configured.store(true, std::memory_order_release);
    hipLaunchKernelGGL(kernel, dim3(512), dim3(64 * NW), lds, stream, p, (int)tiles);   // two workgroups on each of 256 compute units
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_error("conv launch: %s", hipGetErrorString(e)); return -2; }
    return 0;
}

template <int BM, int BN, int WGM, int WGN, int NPW, int NBS>
static int launch_patch_tile(const ConvParams& p, long long mv, hipStream_t stream) {
    constexpr int NW = WGM * WGN;
    const long long tiles = ((mv + BM - 1) / BM) * (p.Cout / BN);
    if (tiles <= 0 || tiles > 0x7fffffffLL) { set_error("conv: bad grid (%lld tiles)", tiles); return -5; }
    constexpr unsigned ring = 2 * NPW * NW * 1024 + NBS * BN * 64, ctile = BM * (BN + 8) * 2;
    constexpr unsigned lds = (ring > ctile ? ring : ctile) + 1024;
    auto kernel = conv3x3_patch_kernel<BM, BN, WGM, WGN, NPW, NBS>;
    static std::atomic<bool> configured{false};
    if (!configured.load(std::memory_order_acquire) && lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) { set_error("conv: cannot reserve %u bytes of LDS: %s", lds, hipGetErrorString(e)); return -2; }
    }
    configured.store(true, std::memory_order_release);
    hipLaunchKernelGGL(kernel, dim3((unsigned)tiles), dim3(64 * NW), lds, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_error("conv launch: %s", hipGetErrorString(e)); return -2; }
    return 0;
}

// Whether the patch kernel takes a layer, and with which tile; -1 = not this kernel's.
static int launch_conv3x3_patch(const ConvParams& params, hipStream_t stream) {
    ConvParams p = params;
    int sw = p.W;
    while (sw > 64 && sw % 2 == 0) sw /= 2;
    if (sw > 128) return -1;
    p.strip_w = sw;
    const int wp = sw + (p.W == sw ? 1 : 2);
    const long long mv = (long long)(p.M / p.PQ) * (p.W / sw) * (p.H + 1) * wp;
    // with fewer tiles than half the compute units the generic kernel, which may split its reduction, is the faster one
    // (ResNet-50 batch 8, 28 x 28 x 128, 53 tiles: 12.2 against 9.2 us; batch 32, 210 tiles: 12.7 against 17.1 us)
    if ((p.Cout % 128 == 0 ? (mv + 127) / 128 * (p.Cout / 128) : (mv + 255) / 256 * (p.Cout / 64)) < 128) return -1;
    if (mv >= (1LL << 24) - 4096) return -1;           // the kernel's index arithmetic is exact below 2^24
    auto per_wave = [&](int bm, int nw) { return ((bm + 2 * wp + 2 + 15) / 16 + nw - 1) / nw; };
    if (p.Cout % 128 == 0) {
        if (((mv + 255) / 256) * (p.Cout / 128) >= 768) {          // a round and a half of workgroups at least: 8 waves on 256 x 128
            const int npw = per_wave(256, 8);
            if (npw <= 3) return launch_patch_tile<256, 128, 4, 2, 3, 3>(p, mv, stream);
            if (npw <= 4) return launch_patch_tile<256, 128, 4, 2, 4, 3>(p, mv, stream);
        }
        const int npw = per_wave(128, 4);
        if (npw <= 4) return launch_patch_tile<128, 128, 2, 2, 4, 3>(p, mv, stream);
        if (npw <= 6) return launch_patch_tile<128, 128, 2, 2, 6, 3>(p, mv, stream);
        return -1;
    }
    if (p.Cout % 64 == 0) {
        const int npw = per_wave(256, 4);
        // 64 channels in and out and tiles enough for two per workgroup: workgroups that walk over tiles
        const bool walk = p.Cout == 64 && p.C <= 128 && (mv + 255) / 256 >= 1024;
        if (npw <= 6) return walk ? launch_patch_walk<256, 64, 4, 1, 6, 3>(p, mv, stream) : launch_patch_tile<256, 64, 4, 1, 6, 3>(p, mv, stream);
        if (npw <= 8) return walk ? launch_patch_walk<256, 64, 4, 1, 8, 3>(p, mv, stream) : launch_patch_tile<256, 64, 4, 1, 8, 3>(p, mv, stream);
        return -1;
    }
    return -1;
}

template <int BM, int BN, int BK, int WGM, int WGN, int STAGES>
static int launch_dma_tile(const ConvParams& p, int mode, hipStream_t stream) {
    const long long tiles = (long long)((p.M + BM - 1) / BM) * ((p.Cout + BN - 1) / BN) * p.ksplit;
    if (tiles <= 0 || tiles > 0x7fffffffLL) { set_error("conv: bad grid (%lld tiles)", tiles); return -5; }
    constexpr unsigned ring = STAGES * (BM + BN) * BK * 2, ctile = BM * (BN + 8) * 2;
    constexpr unsigned lds = (ring > ctile ? ring : ctile) + 1024;    // the epilogue parks the output tile in the ring's LDS; + the tile's bias row
    dim3 grid((unsigned)tiles), block(64 * WGM * WGN);
    ConvParams q = p;
    {
        const int tn = (p.Cout + BN - 1) / BN;
        q.tiles_n_shift = -1;
        for (int sft = 0; sft < 31; ++sft) if ((1 << sft) == tn) q.tiles_n_shift = sft;
    }
    auto go = [&](auto kernel) -> int {
        static std::atomic<bool> configured{false};     // one flag per instantiation; setting the attribute twice is harmless
        if (!configured.load(std::memory_order_acquire) && lds > 48 * 1024) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) { set_error("conv: cannot reserve %u bytes of LDS: %s", lds, hipGetErrorString(e)); return -2; }
        }
        configured.store(true, std::memory_order_release);
        hipLaunchKernelGGL(kernel, grid, block, lds, stream, q);
        return 0;
    };
    int rc;
    if (mode == MODE_1X1 && p.act == ACT_GELU) rc = go(conv_igemm_dma_kernel<BM, BN, BK, WGM, WGN, MODE_1X1, STAGES, true, false>);
    else if (mode == MODE_1X1 && p.x2) rc = go(conv_igemm_dma_kernel<BM, BN, BK, WGM, WGN, MODE_1X1, STAGES, false, false, true>);
    else if (mode == MODE_1X1 && p.res && p.ksplit == 1) rc = go(conv_igemm_dma_kernel<BM, BN, BK, WGM, WGN, MODE_1X1, STAGES, false, true>);
    else if (mode == MODE_1X1) rc = go(conv_igemm_dma_kernel<BM, BN, BK, WGM, WGN, MODE_1X1, STAGES, false, false>);
    else rc = go(conv_igemm_dma_kernel<BM, BN, BK, WGM, WGN, MODE_GATHER8, STAGES, false, false>);
    if (rc) return rc;
    if (p.ksplit > 1) {
        const long long n8 = (long long)p.M * (p.Cout / 8);
        hipLaunchKernelGGL(splitk_finish_kernel, dim3((unsigned)((n8 + 255) / 256)), dim3(256), 0, stream, q);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_error("conv launch: %s", hipGetErrorString(e)); return -2; }
    return 0;
}


// The same tile with the reduction split over KG groups of wavefronts inside the workgroup (no second launch).
template <int BM, int BN, int BK, int WGM, int WGN, int STAGES, int KG>
static int launch_dma_tile_groups(const ConvParams& p, int mode, hipStream_t stream) {
    const long long tiles = (long long)((p.M + BM - 1) / BM) * ((p.Cout + BN - 1) / BN);
    if (tiles <= 0 || tiles > 0x7fffffffLL) { set_error("conv: bad grid (%lld tiles)", tiles); return -5; }
    constexpr unsigned ring = KG * STAGES * (BM + BN) * BK * 2, ctile = BM * (BN + 8) * 2;
    constexpr unsigned lds = (ring > ctile ? ring : ctile) + 1024;
    static_assert(lds <= 160 * 1024, "LDS limit");
    dim3 grid((unsigned)tiles), block(64 * WGM * WGN * KG);
    ConvParams q = p;
    q.ksplit = 1;
    {
        const int tn = (p.Cout + BN - 1) / BN;
        q.tiles_n_shift = -1;
        for (int sft = 0; sft < 31; ++sft) if ((1 << sft) == tn) q.tiles_n_shift = sft;
    }
    auto go = [&](auto kernel) -> int {
        static std::atomic<bool> configured{false};
        if (!configured.load(std::memory_order_acquire)) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) { set_error("conv: cannot reserve %u bytes of LDS: %s", lds, hipGetErrorString(e)); return -2; }
        }
        configured.store(true, std::memory_order_release);
        hipLaunchKernelGGL(kernel, grid, block, lds, stream, q);
        return 0;
    };
    int rc;
    if (mode == MODE_1X1 && p.res) rc = go(conv_igemm_dma_kernel<BM, BN, BK, WGM, WGN, MODE_1X1, STAGES, false, true, false, KG>);
    else if (mode == MODE_1X1) rc = go(conv_igemm_dma_kernel<BM, BN, BK, WGM, WGN, MODE_1X1, STAGES, false, false, false, KG>);
    else rc = go(conv_igemm_dma_kernel<BM, BN, BK, WGM, WGN, MODE_GATHER8, STAGES, false, false, false, KG>);
    if (rc) return rc;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_error("conv launch: %s", hipGetErrorString(e)); return -2; }
    return 0;
}

template <int BM, int BN>
static int launch_tile(const ConvParams& p, int mode, bool staged, hipStream_t stream) {
    const long long tiles = (long long)((p.M + BM - 1) / BM) * ((p.Cout + BN - 1) / BN);
    if (tiles <= 0 || tiles > 0x7fffffffLL) { set_error("conv: bad grid (%lld tiles)", tiles); return -5; }
    dim3 grid((unsigned)tiles), block(256);
#define STRAIT_LAUNCH(MODE, ST) hipLaunchKernelGGL((conv_igemm_kernel<BM, BN, MODE, ST>), grid, block, 0, stream, p)
    if (mode == MODE_1X1) { if (staged) STRAIT_LAUNCH(MODE_1X1, true); else STRAIT_LAUNCH(MODE_1X1, false); }
    else if (mode == MODE_GATHER8) { if (staged) STRAIT_LAUNCH(MODE_GATHER8, true); else STRAIT_LAUNCH(MODE_GATHER8, false); }
    else { if (staged) STRAIT_LAUNCH(MODE_SCALAR, true); else STRAIT_LAUNCH(MODE_SCALAR, false); }
#undef STRAIT_LAUNCH
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_error("conv launch: %s", hipGetErrorString(e)); return -2; }
    return 0;
}

int launch_conv(const ConvParams& params, hipStream_t stream) {
    ConvParams p = params;
    if (!p.x || !p.w || !p.y || p.M <= 0 || p.Cout <= 0 || p.Kg <= 0 || p.C <= 0 || p.R <= 0 || p.S <= 0 ||
        p.Q <= 0 || p.PQ <= 0 || p.stride_h <= 0 || p.stride_w <= 0) {
        set_error("conv: invalid parameters"); return -1;
    }
    if (p.x2) {
        // a second source: both parts whole 64-wide slices, the first part a dense pointwise input, no residual
        if (p.R != 1 || p.S != 1 || p.stride_h != 1 || p.stride_w != 1 || p.pad_h || p.pad_w || p.res || p.out_f32 || p.act == ACT_GELU ||
            p.C % 64 != 0 || p.K2 <= 0 || p.K2 % 64 != 0 || p.Kg != p.C + p.K2 || p.sW != p.C || p.stride2 <= 0 ||
            p.sW2 % 8 != 0 || p.sH2 % 8 != 0 || p.sN2 % 8 != 0 || p.Cout % 8 != 0 || p.ldy % 8 != 0 ||
            (reinterpret_cast<uintptr_t>(p.x2) & 15)) {
            set_error("conv: unsupported use of a second source"); return -5;
        }
        // the furthest element any output pixel reads from it
        p.x2_elems = (long long)(p.M / p.PQ - 1) * p.sN2 + (long long)((p.PQ / p.Q - 1) * p.stride2) * p.sH2 +
                     (long long)((p.Q - 1) * p.stride2) * p.sW2 + p.K2;
        if (p.x2_elems * 2 > 0x7fffffffLL) { set_error("conv: second source too large"); return -5; }
    } else if (p.Kg != p.R * p.S * p.C) { set_error("conv: Kg != R*S*C"); return -5; }
    if (p.ldw % 8 != 0 || p.ldw < p.Kg) { set_error("conv: weight pitch %d must be a multiple of 8 and >= %d", p.ldw, p.Kg); return -5; }
    if (p.ldy < p.Cout) { set_error("conv: ldy < Cout"); return -5; }
    if ((reinterpret_cast<uintptr_t>(p.x) | reinterpret_cast<uintptr_t>(p.w) | reinterpret_cast<uintptr_t>(p.y) |
         reinterpret_cast<uintptr_t>(p.res)) & 15) { set_error("conv: pointers must be 16-byte aligned"); return -1; }
    const bool vec_ok = (p.C % 8 == 0) && (p.sW % 8 == 0) && (p.sH % 8 == 0) && (p.sN % 8 == 0);
    int mode;
    if (vec_ok && p.R == 1 && p.S == 1 && p.pad_h == 0 && p.pad_w == 0) mode = MODE_1X1;
    else if (vec_ok) mode = MODE_GATHER8;
    else mode = MODE_SCALAR;
    const bool staged = !p.out_f32 && (p.Cout % 8 == 0) && (p.ldy % 8 == 0);
    // pick the largest tile that still gives the 256 CUs about two workgroups each
    auto tiles = [&](int bm, int bn) { return (long long)((p.M + bm - 1) / bm) * ((p.Cout + bn - 1) / bn); };
    const bool dense = mode == MODE_1X1 && p.stride_h == 1;
    p.x_elems = dense ? (long long)p.M * p.sW : (long long)(p.M / p.PQ) * p.sN;
    const long long lead = (long long)p.pad_h * p.sH + (long long)p.pad_w * p.sW;
    const bool small = (p.x_elems + lead) * 2 <= 0x7fffffffLL && (long long)p.Cout * p.ldw * 2 <= 0x7fffffffLL;
    p.ksplit = 1;
    // (GELU after a residual add is left to the first kernel: this one applies GELU before the staging)
    const bool regular = (mode == MODE_1X1 && !(p.act == ACT_GELU && p.res)) || (mode == MODE_GATHER8 && p.C % 32 == 0 && p.R * p.S <= 32 && p.act != ACT_GELU);
    // Few output tiles and a long reduction (small batches, late layers): one workgroup per tile
    // would leave most CUs idle behind a serial chain of slices.  Split the reduction: over two groups of
    // wavefronts inside the workgroup where a shallow split will do, else over ksplit workgroups per tile,
    // each writing an fp32 slab, with a second launch that reduces them.
    if (regular && small && p.Cout % 8 == 0 && p.ldy % 8 == 0) {
        const long long t = tiles(64, 64);
        const int nk = (p.Kg + 31) / 32;
        // about one workgroup per CU and a bit hides the chain of slices; a layer that streams megabytes of
        // weights for a handful of rows (the fully connected layers of a plain CNN) is bound by the bytes in
        // flight and takes four times as many
        const long long target = (long long)p.Cout * p.Kg * 2 >= (8LL << 20) ? 1280 : 320;
        long long ks = (target + t - 1) / t;
        if (ks > nk / 4) ks = nk / 4;
        if (ks > 32) ks = 32;
        // Up to an eight-way split, and up to one tile per CU: two groups of wavefronts in one workgroup, half of the
        // slices each and no second launch (ResNet-50 batch 8: 1024 -> 256 at 14 x 14 10.7 -> 6.3 us, its 3x3 14.1 -> 12.0 us;
        // batch 16, 196 tiles, the same 3x3 13.7 -> 11.9 us; four groups with shallower rings are no faster, and from 400
        // tiles on the groups cost more than they save).  Deeper splits are layers that stream megabytes of weights
        // for a few rows and need the workgroups (512-channel 3x3 at 7 x 7, batch 1: 12.8 us split 32 ways, 18.7 us in
        // two groups; the same layer at batch 8, split six ways: 14.3 against 19.5 us, so reductions of more than 96
        // slices keep the slabs wherever those are an option).
        if (t <= 256 && nk >= 8 && ks <= 8 && (t > 128 || (ks > 1 && nk <= 96)) && staged && !p.x2 && p.act != ACT_GELU) {
            if (mode == MODE_1X1 && p.Kg % 64 == 0) return launch_dma_tile_groups<64, 64, 64, 2, 2, 3, 2>(p, mode, stream);
            return launch_dma_tile_groups<64, 64, 32, 2, 2, 4, 2>(p, mode, stream);
        }
        if (t <= 128 && nk >= 8 && p.ws && (reinterpret_cast<uintptr_t>(p.ws) & 15) == 0) {
            while (ks > 1 && ks * (long long)p.M * p.Cout * 4 > (long long)p.ws_bytes) --ks;
            if (ks > 1) {
                p.ksplit = (int)ks;
                // dense products with four or more 32-wide slices per workgroup take them 64 wide: half the barriers and
                // round trips of the chain (1024 -> 256 at 14 x 14, batch 1: 10.2 -> 7.9 us); gathered 3x3 slices do not gain
                if (mode == MODE_1X1 && p.Kg % 64 == 0 && nk / ks >= 4) return launch_dma_tile<64, 64, 64, 2, 2, 3>(p, mode, stream);
                return launch_dma_tile<64, 64, 32, 2, 2, 3>(p, mode, stream);
            }
        }
    }
    // wide 3x3 stride-1 layers: the patch kernel fetches each input pixel once per slice instead of once per tap
    if (staged && regular && small && mode == MODE_GATHER8 && p.R == 3 && p.S == 3 && p.stride_h == 1 && p.stride_w == 1 &&
        p.pad_h == 1 && p.pad_w == 1 && !p.res && p.act != ACT_GELU && p.W >= 14 && p.Q == p.W && p.PQ == p.H * p.W && p.ldy % 8 == 0) {
        const int rc = launch_conv3x3_patch(p, stream);
        if (rc != -1) return rc;
    }
    if (staged && regular && small) {
        // Tile choice, from sweeps over the served networks' layer shapes on MI355X:
        //  - deep reductions (K >= 512) with at least 128 output channels are limited by how fast
        //    operands reach the CU: the 128x128 tile halves the bytes per flop and 64-wide slices
        //    halve the barriers; a third stage (one workgroup per CU) pays only when there is at most one tile per CU anyway;
        //  - shallow reductions stream activations: the 128x64 tile with few stages keeps the LDS
        //    footprint small, i.e. more workgroups in flight per CU to cover memory latency.
        const bool bk64 = mode == MODE_1X1 ? p.Kg % 64 == 0 : p.C % 64 == 0;
        const long long t128 = tiles(128, 128), t64 = tiles(128, 64);
        if (p.Kg >= 512 && p.Cout >= 256 && tiles(256, 128) >= 512)      // plenty of tiles: 8 waves on 256x128
            return launch_dma_tile<256, 128, 32, 2, 4, 3>(p, mode, stream);
        if (p.Kg >= 256 && p.Kg < 512 && p.Cout >= 1024 && tiles(128, 256) >= 192)   // wide outputs, medium reduction
            return launch_dma_tile<128, 256, 32, 2, 4, 2>(p, mode, stream);
        if (p.Kg >= 256 && p.Kg < 512 && p.Cout >= 512 && tiles(256, 128) >= 512)    // the same with half the width (a block-closing
            return launch_dma_tile<256, 128, 32, 2, 4, 3>(p, mode, stream);           // convolution with its projection: 81 -> 66 us at batch 128)
        if (p.Kg >= 512 && p.Cout >= 128 && t128 >= 192) {
            if (bk64) return t128 <= 256 ? launch_dma_tile<128, 128, 64, 2, 2, 3>(p, mode, stream)
                                         : launch_dma_tile<128, 128, 64, 2, 2, 2>(p, mode, stream);
            return launch_dma_tile<128, 128, 32, 2, 2, 3>(p, mode, stream);
        }
        if (t64 >= 256) return p.Kg >= 288 ? launch_dma_tile<128, 64, 32, 2, 2, 3>(p, mode, stream)
                                           : launch_dma_tile<128, 64, 32, 2, 2, 2>(p, mode, stream);
        // few, small tiles: nothing competes for LDS, and four slices in flight per workgroup instead of two shorten the
        // latency chain of the reduction (ResNet-50 b32 0.96 -> 0.87 ms, b8 0.55 -> 0.53 ms; six are no better)
        if (bk64) return launch_dma_tile<64, 64, 64, 2, 2, 3>(p, mode, stream);      // the same bytes in flight in half the steps
        return launch_dma_tile<64, 64, 32, 2, 2, 4>(p, mode, stream);
    }
    if (p.x2) { set_error("conv: a second source needs the LDS-direct kernels (sizes out of their range)"); return -5; }
    if (p.Cout > 64 && tiles(128, 128) >= 512) return launch_tile<128, 128>(p, mode, staged, stream);
    if (tiles(128, 64) >= 512) return launch_tile<128, 64>(p, mode, staged, stream);
    return launch_tile<64, 64>(p, mode, staged, stream);
}

}  // namespace strait
