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
#include "kernels.hpp"

namespace strait {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

enum { MODE_1X1 = 0, MODE_GATHER8 = 1, MODE_SCALAR = 2 };

__device__ __forceinline__ float apply_act(float v, int act) {
    if (act == ACT_RELU) return fmaxf(v, 0.f);
    if (act == ACT_RELU6) return fminf(fmaxf(v, 0.f), 6.f);
    if (act == ACT_GELU) return 0.5f * v * (1.f + erff(v * 0.70710678118654752440f));
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

int launch_conv(const ConvParams& p, hipStream_t stream) {
    if (!p.x || !p.w || !p.y || p.M <= 0 || p.Cout <= 0 || p.Kg <= 0 || p.C <= 0 || p.R <= 0 || p.S <= 0 ||
        p.Q <= 0 || p.PQ <= 0 || p.stride_h <= 0 || p.stride_w <= 0) {
        set_error("conv: invalid parameters"); return -1;
    }
    if (p.Kg != p.R * p.S * p.C) { set_error("conv: Kg != R*S*C"); return -5; }
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
    if (p.Cout > 64 && tiles(128, 128) >= 512) return launch_tile<128, 128>(p, mode, staged, stream);
    if (tiles(128, 64) >= 512) return launch_tile<128, 64>(p, mode, staged, stream);
    return launch_tile<64, 64>(p, mode, staged, stream);
}

}  // namespace strait
