// Bandwidth-bound kernels of the served models for gfx950: input packing, depthwise 3x3
// convolution, pooling, softmax + top-1, LayerNorm, argmax.  (Paper Section 3.2 step (2): the
// kernel sequence of a batch; these are its non-GEMM members.)
//
// None of these is a contraction worth MFMA: each reads its operands once from HBM/L2 and
// writes its result once, so the design rule is 16-byte accesses that are contiguous across
// the lanes of a wavefront (the channel axis of NHWC), fp32 arithmetic in registers, and
// enough workgroups (>> 256) to cover the chip.
#include <algorithm>

#include "kernels.hpp"

namespace strait {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));

#define STRAIT_CHECK_LAUNCH(what)                                                   \
    do {                                                                            \
        hipError_t e_ = hipGetLastError();                                          \
        if (e_ != hipSuccess) { set_error(what ": %s", hipGetErrorString(e_)); return -2; } \
    } while (0)

__device__ __forceinline__ float act_f(float v, int act) {
    if (act == ACT_RELU) return fmaxf(v, 0.f);
    if (act == ACT_RELU6) return fminf(fmaxf(v, 0.f), 6.f);
    return v;
}

// ------------------------------------------------------------------------------------------
// fill
__global__ void fill_zero_kernel(uint4* p, size_t n16) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t step = (size_t)gridDim.x * blockDim.x;
    for (; i < n16; i += step) p[i] = make_uint4(0, 0, 0, 0);
}
int launch_fill_zero(void* p, size_t bytes, hipStream_t stream) {
    if (bytes == 0) return 0;
    if ((reinterpret_cast<uintptr_t>(p) & 15) || (bytes & 15)) { set_error("fill: 16-byte alignment required"); return -1; }
    const size_t n16 = bytes / 16;
    unsigned blocks = (unsigned)((n16 + 255) / 256 > 4096 ? 4096 : (n16 + 255) / 256);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, stream, (uint4*)p, n16);
    STRAIT_CHECK_LAUNCH("fill");
    return 0;
}

// ------------------------------------------------------------------------------------------
// Small transfers between pinned host memory that the GPU can address and device memory, done by a kernel:
// results on their way out, and inputs of up to a few megabytes on their way in.  (A hipMemcpyAsync of such a
// size, in either direction, now and then blocks the submitting thread for milliseconds when other streams are
// busy; a kernel launch does not.)  Both pointers 16-byte aligned, bytes a multiple of 4.  Four independent
// 16-byte loads per thread and round keep enough requests in flight to fill the host link on the way in.
__global__ void __launch_bounds__(256) copy_mapped_kernel(const uint32_t* __restrict__ src, uint32_t* __restrict__ dst, size_t n4, int hp) {
    if (hp) __builtin_amdgcn_s_setprio(3);
    const size_t n16 = n4 >> 2;
    const size_t step = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 3 * step < n16; i += 4 * step) {
        const uint4 a = ((const uint4*)src)[i], b = ((const uint4*)src)[i + step], c = ((const uint4*)src)[i + 2 * step], d = ((const uint4*)src)[i + 3 * step];
        ((uint4*)dst)[i] = a; ((uint4*)dst)[i + step] = b; ((uint4*)dst)[i + 2 * step] = c; ((uint4*)dst)[i + 3 * step] = d;
    }
    for (; i < n16; i += step) ((uint4*)dst)[i] = ((const uint4*)src)[i];
    const size_t tail = n16 << 2;
    if (blockIdx.x == 0 && tail + threadIdx.x < n4) dst[tail + threadIdx.x] = src[tail + threadIdx.x];
}
int launch_copy_mapped(const void* src, void* dst, size_t bytes, int hp, hipStream_t stream) {
    if (bytes == 0) return 0;
    if (!src || !dst || (reinterpret_cast<uintptr_t>(src) & 15) || (reinterpret_cast<uintptr_t>(dst) & 15) || (bytes & 3)) {
        set_error("mapped copy: 16-byte aligned buffers and a multiple of 4 bytes required"); return -1;
    }
    const size_t n4 = bytes / 4, n16 = n4 / 4;
    const unsigned blocks = (unsigned)std::min<size_t>(256, std::max<size_t>(1, (n16 + 255) / 256));
    hipLaunchKernelGGL(copy_mapped_kernel, dim3(blocks), dim3(256), 0, stream, (const uint32_t*)src, (uint32_t*)dst, n4, hp);
    STRAIT_CHECK_LAUNCH("mapped copy");
    return 0;
}

// ------------------------------------------------------------------------------------------
// pack: [N][H][W][C] (C <= Cpad, Cpad in {4, 8}) -> zero-bordered [N][Hp][Wp][Cpad].
// One thread per output pixel.
template <int CPAD>
__global__ void __launch_bounds__(256) pack_input_kernel(const half_t* __restrict__ x, int N, int H, int W, int C,
                                                          half_t* __restrict__ y, int Hp, int Wp, int pt, int pl, int hp) {
    if (hp) __builtin_amdgcn_s_setprio(3);
    const long long total = (long long)N * Hp * Wp;
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int wp = (int)(i % Wp);
    const long long t = i / Wp;
    const int hpix = (int)(t % Hp);
    const int n = (int)(t / Hp);
    const int h = hpix - pt, w = wp - pl;
    _Float16 v[CPAD];
#pragma unroll
    for (int c = 0; c < CPAD; ++c) v[c] = (half_t)0;
    if ((unsigned)h < (unsigned)H && (unsigned)w < (unsigned)W) {
        const half_t* src = x + (((long long)n * H + h) * W + w) * C;
#pragma unroll
        for (int c = 0; c < CPAD; ++c)
            if (c < C) v[c] = src[c];
    }
    half_t* dst = y + i * CPAD;
    if (CPAD == 4) *(half4*)dst = *(half4*)v; else *(half8*)dst = *(half8*)v;
}

int launch_pack_input(const half_t* x, int N, int H, int W, int C, half_t* y, int Hp, int Wp, int Cpad,
                      int pad_top, int pad_left, int hp, hipStream_t stream) {
    if (!x || !y || N <= 0 || H <= 0 || W <= 0 || C <= 0 || C > Cpad || (Cpad != 4 && Cpad != 8) ||
        Hp < H + pad_top || Wp < W + pad_left) { set_error("pack: invalid shape"); return -5; }
    const long long total = (long long)N * Hp * Wp;
    const long long blocks = (total + 255) / 256;
    if (blocks > 0x7fffffffLL) { set_error("pack: grid too large"); return -5; }
    if (Cpad == 4)
        hipLaunchKernelGGL(pack_input_kernel<4>, dim3((unsigned)blocks), dim3(256), 0, stream, x, N, H, W, C, y, Hp, Wp, pad_top, pad_left, hp);
    else
        hipLaunchKernelGGL(pack_input_kernel<8>, dim3((unsigned)blocks), dim3(256), 0, stream, x, N, H, W, C, y, Hp, Wp, pad_top, pad_left, hp);
    STRAIT_CHECK_LAUNCH("pack");
    return 0;
}

// Hardware workgroup id b runs on XCD b mod 8, each XCD with an L2 of its own.  This gives every XCD a contiguous
// range of logical block numbers instead, so that blocks which share input rows (vertically adjacent row tiles of a
// stencil) fetch them through one L2 rather than through several.
__device__ __forceinline__ unsigned xcd_contiguous_block() {
    const unsigned nb = gridDim.x, b = blockIdx.x;
    const unsigned per = nb >> 3, rem = nb & 7, xcd = b & 7, idx = b >> 3;
    return (xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per) + idx;
}

// ------------------------------------------------------------------------------------------
// depthwise 3x3, pad 1, stride 1 or 2, fused bias + activation.
// A thread owns 8 channels (16 bytes) of TW consecutive output pixels of one output row.  For each
// of the three input rows it loads the (TW-1)*stride+3 input vectors the strip touches once and
// feeds all TW outputs from registers, so a strip of 4 costs 18 (stride 1) or 27 (stride 2) loads
// instead of 36, and the index arithmetic is paid once per strip.  Lanes of a wavefront cover
// consecutive channel groups, i.e. contiguous memory.  fp16 operands, fp32 accumulation.
template <int STRIDE, int TW>
__global__ void __launch_bounds__(256) dwconv3x3_kernel(const half_t* __restrict__ x, int N, int H, int W, int C,
                                                         const half_t* __restrict__ w, const float* __restrict__ bias,
                                                         int act, half_t* __restrict__ y, int P, int Q, int hp) {
    if (hp) __builtin_amdgcn_s_setprio(3);
    constexpr int NV = (TW - 1) * STRIDE + 3;
    const unsigned C8 = (unsigned)C >> 3;
    const unsigned QT = (unsigned)(Q + TW - 1) / TW;
    const unsigned long long total = (unsigned long long)N * P * QT * C8;
    const unsigned long long i = (unsigned long long)xcd_contiguous_block() * 256 + threadIdx.x;
    if (i >= total) return;
    const unsigned c8 = (unsigned)(i % C8);
    unsigned t = (unsigned)(i / C8);
    const unsigned qt = t % QT; t /= QT;
    const unsigned pp = t % (unsigned)P;
    const unsigned n = t / (unsigned)P;
    const int c = (int)c8 * 8;

    half8 wv[9];
#pragma unroll
    for (int k = 0; k < 9; ++k) wv[k] = *(const half8*)(w + (long long)k * C + c);
    float acc[TW][8];
    {
        float bv[8];
        if (bias) {
            const float4 b0 = *(const float4*)(bias + c), b1 = *(const float4*)(bias + c + 4);
            bv[0] = b0.x; bv[1] = b0.y; bv[2] = b0.z; bv[3] = b0.w; bv[4] = b1.x; bv[5] = b1.y; bv[6] = b1.z; bv[7] = b1.w;
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) bv[j] = 0.f;
        }
#pragma unroll
        for (int tq = 0; tq < TW; ++tq)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[tq][j] = bv[j];
    }
    const int q0 = (int)qt * TW;
    const int iw0 = q0 * STRIDE - 1;
    const half_t* xin = x + (long long)n * H * W * C + c;
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        const int ih = (int)pp * STRIDE - 1 + r;
        if ((unsigned)ih >= (unsigned)H) continue;
        const half_t* row = xin + (long long)ih * W * C;
        half8 xv[NV];
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            const int iw = iw0 + k;
            if ((unsigned)iw < (unsigned)W) xv[k] = *(const half8*)(row + (long long)iw * C);
            else {
#pragma unroll
                for (int j = 0; j < 8; ++j) xv[k][j] = (half_t)0;
            }
        }
#pragma unroll
        for (int tq = 0; tq < TW; ++tq)
#pragma unroll
            for (int s = 0; s < 3; ++s)
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[tq][j] += (float)xv[tq * STRIDE + s][j] * (float)wv[r * 3 + s][j];
    }
    half_t* yout = y + (((long long)n * P + pp) * Q + q0) * C + c;
#pragma unroll
    for (int tq = 0; tq < TW; ++tq) {
        if (q0 + tq < Q) {
            half8 o;
#pragma unroll
            for (int j = 0; j < 8; ++j) o[j] = (half_t)act_f(acc[tq][j], act);
            *(half8*)(yout + (long long)tq * C) = o;
        }
    }
}


// Stride 1, a column of TH outputs per thread.  Consecutive threads own consecutive 16-byte chunks along an image
// row (pixel-major, then channel group), so every load and store instruction of a wavefront covers one contiguous
// kilobyte whatever the channel count; a thread fetches the left, centre and right vector of each of the TH + 2
// input rows its column touches (the neighbours' copies of the same vectors hit in L1).  The strips of the kernel
// above leave, with few channels, gaps of TW pixels between the lanes of one instruction.  Every output
// accumulates its nine taps in the same order as there, so results are identical.
template <int TH>
__global__ void __launch_bounds__(256) dwconv3x3_s1_cols_kernel(const half_t* __restrict__ x, int N, int H, int W, int C,
                                                                 const half_t* __restrict__ w, const float* __restrict__ bias,
                                                                 int act, half_t* __restrict__ y, int hp) {
    if (hp) __builtin_amdgcn_s_setprio(3);
    const unsigned C8 = (unsigned)C >> 3;
    const unsigned PT = (unsigned)(H + TH - 1) / TH;
    const unsigned long long total = (unsigned long long)N * PT * W * C8;
    const unsigned long long i = (unsigned long long)xcd_contiguous_block() * 256 + threadIdx.x;
    if (i >= total) return;
    const unsigned c8 = (unsigned)(i % C8);
    unsigned t = (unsigned)(i / C8);
    const unsigned q = t % (unsigned)W; t /= (unsigned)W;
    const unsigned pt = t % PT;
    const unsigned n = t / PT;
    const int c = (int)c8 * 8;
    half8 wv[9];
#pragma unroll
    for (int k = 0; k < 9; ++k) wv[k] = *(const half8*)(w + (long long)k * C + c);
    float acc[TH][8];
    {
        float bv[8];
        if (bias) {
            const float4 b0 = *(const float4*)(bias + c), b1 = *(const float4*)(bias + c + 4);
            bv[0] = b0.x; bv[1] = b0.y; bv[2] = b0.z; bv[3] = b0.w; bv[4] = b1.x; bv[5] = b1.y; bv[6] = b1.z; bv[7] = b1.w;
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) bv[j] = 0.f;
        }
#pragma unroll
        for (int o = 0; o < TH; ++o)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[o][j] = bv[j];
    }
    const int p0 = (int)pt * TH;
    const half_t* xin = x + ((long long)n * H * W + q) * C + c;
    const bool has_l = q > 0, has_r = q + 1 < (unsigned)W;
#pragma unroll
    for (int r = 0; r < TH + 2; ++r) {
        const int ih = p0 - 1 + r;
        if ((unsigned)ih >= (unsigned)H) continue;
        const half_t* row = xin + (long long)ih * W * C;
        half8 xv[3];
#pragma unroll
        for (int j = 0; j < 8; ++j) { xv[0][j] = (half_t)0; xv[2][j] = (half_t)0; }
        if (has_l) xv[0] = *(const half8*)(row - C);
        xv[1] = *(const half8*)row;
        if (has_r) xv[2] = *(const half8*)(row + C);
#pragma unroll
        for (int o = 0; o < TH; ++o) {
            const int fr = r - o;                       // filter row this input row is for output row p0 + o
            if (fr < 0 || fr > 2) continue;
#pragma unroll
            for (int sx = 0; sx < 3; ++sx)
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[o][j] += (float)xv[sx][j] * (float)wv[fr * 3 + sx][j];
        }
    }
#pragma unroll
    for (int o = 0; o < TH; ++o) {
        if (p0 + o >= H) continue;
        half8 ov;
#pragma unroll
        for (int j = 0; j < 8; ++j) ov[j] = (half_t)act_f(acc[o][j], act);
        *(half8*)(y + (((long long)n * H + p0 + o) * W + q) * C + c) = ov;
    }
}

int launch_dwconv3x3(const half_t* x, int N, int H, int W, int C, const half_t* w_rsc, const float* bias,
                     int stride, int act, half_t* y, int hp, hipStream_t stream) {
    if (!x || !w_rsc || !y || N <= 0 || H <= 0 || W <= 0 || C <= 0 || C % 8 != 0 || (stride != 1 && stride != 2)) {
        set_error("dwconv3x3: needs C %% 8 == 0 and stride 1 or 2"); return -5;
    }
    if ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(w_rsc) | reinterpret_cast<uintptr_t>(y) |
         reinterpret_cast<uintptr_t>(bias)) & 15) { set_error("dwconv3x3: pointers must be 16-byte aligned"); return -1; }
    const int P = (H + 2 - 3) / stride + 1, Q = (W + 2 - 3) / stride + 1;
    constexpr int TW = 4;
    const long long total = (long long)N * P * ((Q + TW - 1) / TW) * (C / 8);
    const long long blocks = (total + 255) / 256;
    if (blocks > 0x7fffffffLL || (long long)N * P * ((Q + TW - 1) / TW) > 0xffffffffLL) { set_error("dwconv3x3: grid too large"); return -5; }
    constexpr int TH = 4;
    const long long total_cols = (long long)N * ((H + TH - 1) / TH) * W * (C / 8);
    if (stride == 1 && total_cols >= 16384 && (total_cols + 255) / 256 <= 0x7fffffffLL && (long long)N * ((H + TH - 1) / TH) * W <= 0xffffffffLL) {
        hipLaunchKernelGGL((dwconv3x3_s1_cols_kernel<TH>), dim3((unsigned)((total_cols + 255) / 256)), dim3(256), 0, stream, x, N, H, W, C, w_rsc, bias, act, y, hp);
    } else if (stride == 1)
        hipLaunchKernelGGL((dwconv3x3_kernel<1, TW>), dim3((unsigned)blocks), dim3(256), 0, stream, x, N, H, W, C, w_rsc, bias, act, y, P, Q, hp);
    else
        hipLaunchKernelGGL((dwconv3x3_kernel<2, TW>), dim3((unsigned)blocks), dim3(256), 0, stream, x, N, H, W, C, w_rsc, bias, act, y, P, Q, hp);
    STRAIT_CHECK_LAUNCH("dwconv3x3");
    return 0;
}

// ------------------------------------------------------------------------------------------
// max pooling 3x3 / stride 2 / pad 1.  Thread = 8 channels of one output pixel.
__global__ void __launch_bounds__(256) maxpool3x3s2_kernel(const half_t* __restrict__ x, int N, int H, int W, int C,
                                                            half_t* __restrict__ y, int P, int Q, int hp) {
    if (hp) __builtin_amdgcn_s_setprio(3);
    const int C8 = C >> 3;
    const long long total = (long long)N * P * Q * C8;
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int c8 = (int)(i % C8);
    long long t = i / C8;
    const int q = (int)(t % Q); t /= Q;
    const int pp = (int)(t % P);
    const int n = (int)(t / P);
    half8 m;
#pragma unroll
    for (int j = 0; j < 8; ++j) m[j] = (half_t)(-65504.f);
    bool any = false;
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        const int ih = pp * 2 - 1 + r;
        if ((unsigned)ih >= (unsigned)H) continue;
#pragma unroll
        for (int s = 0; s < 3; ++s) {
            const int iw = q * 2 - 1 + s;
            if ((unsigned)iw >= (unsigned)W) continue;
            const half8 v = *(const half8*)(x + (((long long)n * H + ih) * W + iw) * C + c8 * 8);
#pragma unroll
            for (int j = 0; j < 8; ++j) m[j] = (!any || v[j] > m[j]) ? v[j] : m[j];
            any = true;
        }
    }
    *(half8*)(y + (((long long)n * P + pp) * Q + q) * C + c8 * 8) = m;
}

int launch_maxpool3x3s2(const half_t* x, int N, int H, int W, int C, half_t* y, int hp, hipStream_t stream) {
    if (!x || !y || N <= 0 || H <= 0 || W <= 0 || C <= 0 || C % 8 != 0) { set_error("maxpool: needs C %% 8 == 0"); return -5; }
    const int P = (H + 2 - 3) / 2 + 1, Q = (W + 2 - 3) / 2 + 1;
    const long long blocks = ((long long)N * P * Q * (C / 8) + 255) / 256;
    if (blocks > 0x7fffffffLL) { set_error("maxpool: grid too large"); return -5; }
    hipLaunchKernelGGL(maxpool3x3s2_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, x, N, H, W, C, y, P, Q, hp);
    STRAIT_CHECK_LAUNCH("maxpool");
    return 0;
}

// ------------------------------------------------------------------------------------------
// max pooling 2x2 / stride 2, no padding (H, W even).  Thread = 8 channels of one output pixel.
__global__ void __launch_bounds__(256) maxpool2x2s2_kernel(const half_t* __restrict__ x, int N, int H, int W, int C,
                                                            half_t* __restrict__ y, int hp) {
    if (hp) __builtin_amdgcn_s_setprio(3);
    const int C8 = C >> 3, P = H >> 1, Q = W >> 1;
    const long long total = (long long)N * P * Q * C8;
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int c8 = (int)(i % C8);
    long long t = i / C8;
    const int q = (int)(t % Q); t /= Q;
    const int pp = (int)(t % P);
    const int n = (int)(t / P);
    const half_t* src = x + (((long long)n * H + 2 * pp) * W + 2 * q) * C + c8 * 8;
    const half8 a = *(const half8*)src, b = *(const half8*)(src + C);
    const half8 c = *(const half8*)(src + (long long)W * C), d = *(const half8*)(src + (long long)W * C + C);
    const half8 m = __builtin_elementwise_max(__builtin_elementwise_max(a, b), __builtin_elementwise_max(c, d));
    *(half8*)(y + (((long long)n * P + pp) * Q + q) * C + c8 * 8) = m;
}

int launch_maxpool2x2s2(const half_t* x, int N, int H, int W, int C, half_t* y, int hp, hipStream_t stream) {
    if (!x || !y || N <= 0 || H <= 0 || W <= 0 || C <= 0 || C % 8 != 0 || H % 2 != 0 || W % 2 != 0) {
        set_error("maxpool 2x2: needs C %% 8 == 0 and even H, W"); return -5;
    }
    const long long blocks = ((long long)N * (H / 2) * (W / 2) * (C / 8) + 255) / 256;
    if (blocks > 0x7fffffffLL) { set_error("maxpool 2x2: grid too large"); return -5; }
    hipLaunchKernelGGL(maxpool2x2s2_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, x, N, H, W, C, y, hp);
    STRAIT_CHECK_LAUNCH("maxpool 2x2");
    return 0;
}

// ------------------------------------------------------------------------------------------
// Token assembly of a Vision Transformer: z[n][0] = cls + pos[0], z[n][1 + t] = patch[n][t] + pos[1 + t],
// sums in fp32 rounded once.  patch [N][T][D], cls [D], pos [T + 1][D] fp32, z [N][T + 1][D].
__global__ void __launch_bounds__(256) vit_tokens_kernel(const half_t* __restrict__ patch, const float* __restrict__ cls,
                                                          const float* __restrict__ pos, int N, int T, int D,
                                                          half_t* __restrict__ z, int hp) {
    if (hp) __builtin_amdgcn_s_setprio(3);
    const int D8 = D >> 3;
    const long long total = (long long)N * (T + 1) * D8;
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int d8 = (int)(i % D8);
    long long t = i / D8;
    const int tok = (int)(t % (T + 1));
    const int n = (int)(t / (T + 1));
    float v[8];
    if (tok == 0) {
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = cls[d8 * 8 + j];
    } else {
        const half8 h = *(const half8*)(patch + ((long long)n * T + tok - 1) * D + d8 * 8);
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = (float)h[j];
    }
    half8 o;
#pragma unroll
    for (int j = 0; j < 8; ++j) o[j] = (half_t)(v[j] + pos[(long long)tok * D + d8 * 8 + j]);
    *(half8*)(z + ((long long)n * (T + 1) + tok) * D + d8 * 8) = o;
}

int launch_vit_tokens(const half_t* patch, const float* cls, const float* pos, int N, int T, int D, half_t* z, int hp,
                      hipStream_t stream) {
    if (!patch || !cls || !pos || !z || N <= 0 || T <= 0 || D <= 0 || D % 8 != 0) { set_error("tokens: needs D %% 8 == 0"); return -5; }
    const long long blocks = ((long long)N * (T + 1) * (D / 8) + 255) / 256;
    if (blocks > 0x7fffffffLL) { set_error("tokens: grid too large"); return -5; }
    hipLaunchKernelGGL(vit_tokens_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, patch, cls, pos, N, T, D, z, hp);
    STRAIT_CHECK_LAUNCH("tokens");
    return 0;
}

// ------------------------------------------------------------------------------------------
// global average pooling: [N][HW][C] -> [N][C], fp32 sum / HW, rounded once to fp16.
// A workgroup covers 32 channel groups (256 channels) of one image; its 8 wavefront-halves each
// sum every 8th position and the partial sums meet in LDS, so the loads of one image are spread
// over 8 independent chains instead of one serial walk over HW.
__global__ void __launch_bounds__(256) gap_kernel(const half_t* __restrict__ x, int N, int HW, int C,
                                                   half_t* __restrict__ y, int hp) {
    __shared__ float part[8][32][8];
    if (hp) __builtin_amdgcn_s_setprio(3);
    const int C8 = C >> 3;
    const int g = threadIdx.x & 31, part_id = threadIdx.x >> 5;
    const int c8 = blockIdx.x * 32 + g, n = blockIdx.y;
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (c8 < C8) {
        const half_t* src = x + (long long)n * HW * C + c8 * 8;
        for (int k = part_id; k < HW; k += 8) {
            const half8 v = *(const half8*)(src + (long long)k * C);
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] += (float)v[j];
        }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) part[part_id][g][j] = acc[j];
    __syncthreads();
    if (part_id == 0 && c8 < C8) {
        const float inv = 1.f / (float)HW;
        half8 o;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            float s = 0.f;
#pragma unroll
            for (int q = 0; q < 8; ++q) s += part[q][g][j];
            o[j] = (half_t)(s * inv);
        }
        *(half8*)(y + (long long)n * C + c8 * 8) = o;
    }
}

int launch_global_avgpool(const half_t* x, int N, int HW, int C, half_t* y, int hp, hipStream_t stream) {
    if (!x || !y || N <= 0 || HW <= 0 || C <= 0 || C % 8 != 0 || N > 65535) { set_error("avgpool: needs C %% 8 == 0 and N <= 65535"); return -5; }
    hipLaunchKernelGGL(gap_kernel, dim3((unsigned)((C / 8 + 31) / 32), (unsigned)N), dim3(256), 0, stream, x, N, HW, C, y, hp);
    STRAIT_CHECK_LAUNCH("avgpool");
    return 0;
}

// ------------------------------------------------------------------------------------------
// wavefront reductions (64 lanes) through cross-lane shuffles
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// softmax + top-1: one wavefront per row of fp32 logits; rows of up to 64 * PER elements are read
// once and kept in registers (PER = 16 covers the 1000-class heads), longer rows are re-read.
template <int PER>
__global__ void __launch_bounds__(256) softmax_top1_kernel(const float* __restrict__ logits, int rows, int n,
                                                            float* __restrict__ probs, int32_t* __restrict__ top1, int hp) {
    if (hp) __builtin_amdgcn_s_setprio(3);
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const float* src = logits + (long long)row * n;
    float v[PER > 0 ? PER : 1];
    float mx = -INFINITY;
    int mi = 0x7fffffff;
    if (PER > 0) {
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            const int i = lane + k * 64;
            v[k] = i < n ? src[i] : -INFINITY;
            if (v[k] > mx) { mx = v[k]; mi = i; }           // ascending i: keeps the lowest index on ties
        }
    } else {
        for (int i = lane; i < n; i += 64) {
            const float t = src[i];
            if (t > mx) { mx = t; mi = i; }
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(mx, o, 64);
        const int oi = __shfl_xor(mi, o, 64);
        if (ov > mx || (ov == mx && oi < mi)) { mx = ov; mi = oi; }
    }
    float sum = 0.f;
    if (PER > 0) {
#pragma unroll
        for (int k = 0; k < PER; ++k) { v[k] = __expf(v[k] - mx); sum += v[k]; }    // exp(-inf) = 0 past the row end
    } else {
        for (int i = lane; i < n; i += 64) sum += __expf(src[i] - mx);
    }
    sum = wave_sum(sum);
    const float inv = 1.f / sum;
    float* dst = probs + (long long)row * n;
    if (PER > 0) {
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            const int i = lane + k * 64;
            if (i < n) dst[i] = v[k] * inv;
        }
    } else {
        for (int i = lane; i < n; i += 64) dst[i] = __expf(src[i] - mx) * inv;
    }
    if (lane == 0) top1[row] = mi;
}

int launch_softmax_top1(const float* logits, int rows, int n, float* probs, int32_t* top1, int hp, hipStream_t stream) {
    if (!logits || !probs || !top1 || rows <= 0 || n <= 0) { set_error("softmax: invalid shape"); return -5; }
    const dim3 grid((rows + 3) / 4), block(256);
    if (n <= 128) hipLaunchKernelGGL(softmax_top1_kernel<2>, grid, block, 0, stream, logits, rows, n, probs, top1, hp);
    else if (n <= 1024) hipLaunchKernelGGL(softmax_top1_kernel<16>, grid, block, 0, stream, logits, rows, n, probs, top1, hp);
    else hipLaunchKernelGGL(softmax_top1_kernel<0>, grid, block, 0, stream, logits, rows, n, probs, top1, hp);
    STRAIT_CHECK_LAUNCH("softmax");
    return 0;
}

// argmax over n fp16 features of selected rows: one wavefront per row.
__global__ void __launch_bounds__(256) argmax_f16_kernel(const half_t* __restrict__ x, int rows, int n, long long row_stride,
                                                          int32_t* __restrict__ top1, int hp) {
    if (hp) __builtin_amdgcn_s_setprio(3);
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const half_t* src = x + (long long)row * row_stride;
    float mx = -INFINITY;
    int mi = 0x7fffffff;
    for (int i = lane; i < n; i += 64) {
        const float v = (float)src[i];
        if (v > mx) { mx = v; mi = i; }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(mx, o, 64);
        const int oi = __shfl_xor(mi, o, 64);
        if (ov > mx || (ov == mx && oi < mi)) { mx = ov; mi = oi; }
    }
    if (lane == 0) top1[row] = mi;
}

int launch_argmax_f16(const half_t* x, int rows, int n, long long row_stride, int32_t* top1, int hp, hipStream_t stream) {
    if (!x || !top1 || rows <= 0 || n <= 0 || row_stride < n) { set_error("argmax: invalid shape"); return -5; }
    hipLaunchKernelGGL(argmax_f16_kernel, dim3((rows + 3) / 4), dim3(256), 0, stream, x, rows, n, row_stride, top1, hp);
    STRAIT_CHECK_LAUNCH("argmax");
    return 0;
}

// ------------------------------------------------------------------------------------------
// LayerNorm: one wavefront per row, the row held in registers (n <= 8192 -> at most 16 chunks
// of 8 per lane), two-pass mean / variance in fp32.  Rows whose 8-element chunks do not fill 64 lanes evenly but do
// fill 32 (768 features = 96 chunks) go to half a wavefront each: LPR lanes per row.
template <int MAXC, int LPR>
__global__ void __launch_bounds__(256) layernorm_kernel(const half_t* __restrict__ x, const float* __restrict__ gamma,
                                                         const float* __restrict__ beta, int rows, int n, float eps,
                                                         half_t* __restrict__ y, int hp, long long x_row_stride) {
    if (hp) __builtin_amdgcn_s_setprio(3);
    const int lane = threadIdx.x & (LPR - 1);
    const int row = blockIdx.x * (256 / LPR) + threadIdx.x / LPR;
    if (row >= rows) return;                    // whole groups of LPR lanes leave together: the shuffles below stay inside a group
    auto group_sum = [](float t) {
#pragma unroll
        for (int o = LPR / 2; o > 0; o >>= 1) t += __shfl_xor(t, o, 64);
        return t;
    };
    const int nch = n >> 3;
    const half_t* src = x + (long long)row * x_row_stride;
    float v[MAXC][8];
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
        const int idx = lane + c * LPR;
        if (idx < nch) {
            const half8 h = *(const half8*)(src + idx * 8);
#pragma unroll
            for (int j = 0; j < 8; ++j) { v[c][j] = (float)h[j]; s += v[c][j]; }
        }
    }
    const float mean = group_sum(s) / (float)n;
    float q = 0.f;
#pragma unroll
    for (int c = 0; c < MAXC; ++c)
        if (lane + c * LPR < nch) {
#pragma unroll
            for (int j = 0; j < 8; ++j) { const float d = v[c][j] - mean; q += d * d; }
        }
    const float rstd = 1.f / sqrtf(group_sum(q) / (float)n + eps);
    half_t* dst = y + (long long)row * n;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
        const int idx = lane + c * LPR;
        if (idx < nch) {
            half8 o;
#pragma unroll
            for (int j = 0; j < 8; ++j)
                o[j] = (half_t)((v[c][j] - mean) * rstd * gamma[idx * 8 + j] + beta[idx * 8 + j]);
            *(half8*)(dst + idx * 8) = o;
        }
    }
}

int launch_layernorm(const half_t* x, const float* gamma, const float* beta, int rows, int n, float eps,
                     half_t* y, int hp, hipStream_t stream, long long x_row_stride) {
    if (x_row_stride == 0) x_row_stride = n;
    if (!x || !gamma || !beta || !y || rows <= 0 || n <= 0 || n % 8 != 0 || n > 8192 || x_row_stride < n || x_row_stride % 8 != 0) {
        set_error("layernorm: needs n %% 8 == 0, n <= 8192 and a row stride that is a multiple of 8, at least n"); return -5;
    }
    const dim3 grid((rows + 3) / 4), block(256);
    const int nch = n / 8;
    if (nch <= 128 && nch % 32 == 0 && nch % 64 != 0)
        hipLaunchKernelGGL((layernorm_kernel<4, 32>), dim3((rows + 7) / 8), block, 0, stream, x, gamma, beta, rows, n, eps, y, hp, x_row_stride);
    else if (nch <= 128)
        hipLaunchKernelGGL((layernorm_kernel<2, 64>), grid, block, 0, stream, x, gamma, beta, rows, n, eps, y, hp, x_row_stride);
    else if (nch <= 512)
        hipLaunchKernelGGL((layernorm_kernel<8, 64>), grid, block, 0, stream, x, gamma, beta, rows, n, eps, y, hp, x_row_stride);
    else
        hipLaunchKernelGGL((layernorm_kernel<16, 64>), grid, block, 0, stream, x, gamma, beta, rows, n, eps, y, hp, x_row_stride);
    STRAIT_CHECK_LAUNCH("layernorm");
    return 0;
}

}  // namespace strait
