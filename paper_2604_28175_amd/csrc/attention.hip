// Fused masked multi-head attention for gfx950: scores, key-padding mask, softmax and the
// product with V in one kernel; the S x S score matrix never leaves registers.
// (Paper Section 3.2 step (2): one member of the encoder workload's kernel sequence.)
//
//   out[b, i, h*64 + :] = softmax_j( q_i . k_j / sqrt(64) ,  j < valid_len[b] ) @ V
//
// One workgroup per (sequence, head); wavefront w owns query rows 32w .. 32w+31.  Sequences of up to 128 keys
// run 4 wavefronts and keep 4 key blocks of scores in registers, up to 256 keys 8 wavefronts and 8 blocks (a
// Vision Transformer's 197 tokens), so K and V are staged once per head whatever the length; S need not be a
// multiple of anything: query rows at or beyond S are neither read nor written, key rows at or beyond
// valid_len never leave zero-filled LDS.
//   - K is staged in LDS as [key][d] and V transposed as [d][key], rows at or beyond
//     valid_len zero-filled, so masked keys can never inject non-finite values;
//   - scores^T = K Q^T with v_mfma_f32_32x32x16_f16 (K rows are the "A" operand), which leaves
//     each lane holding 16 keys x up to 4 key blocks of ONE query: the row maximum and sum need
//     a single exchange with lane ^ 32;
//   - the probabilities, rounded to fp16, are already laid out as the "B" operand of
//     out^T = V^T P^T provided V^T's reduction index is enumerated in the same (permuted) key
//     order, which the two 8-byte LDS reads per operand do;
//   - 32-key blocks and 16-key steps that lie entirely beyond valid_len are skipped.
#include <atomic>

#include "kernels.hpp"

namespace strait {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int ATT_D = 64;
constexpr int ATT_LDK = ATT_D + 8;       // K tile row pitch (halfs)

template <int NKB>                       // key blocks of 32 held in registers = wavefronts: sequences of up to 32 * NKB keys
__global__ void __launch_bounds__(64 * NKB) attention_kernel(const half_t* __restrict__ qkv, const int32_t* __restrict__ valid_len,
                                                         int S, int heads, half_t* __restrict__ out, int hp) {
    constexpr int ATT_SMAX = 32 * NKB;
    constexpr int ATT_LDV = ATT_SMAX + 8;    // V^T tile row pitch (halfs)
    extern __shared__ __attribute__((aligned(16))) half_t att_lds[];
    half_t* Ks = att_lds;                    // [ATT_SMAX][ATT_LDK]
    half_t* Vt = att_lds + ATT_SMAX * ATT_LDK;   // [ATT_D][ATT_LDV]
    if (hp) __builtin_amdgcn_s_setprio(3);

    const int b = blockIdx.x / heads, h = blockIdx.x % heads;
    const int hidden = heads * ATT_D;
    const long long row_pitch = 3LL * hidden;
    const half_t* base = qkv + (long long)b * S * row_pitch + h * ATT_D;
    int L = valid_len[b];
    L = L < 0 ? 0 : (L > S ? S : L);

    const int tid = threadIdx.x;
    const int nkb = (L + 31) >> 5;          // key blocks that hold at least one valid key
    // ---- stage K and V^T: every row of the key blocks in use, zeros at and beyond valid_len ----
    // a thread moves 8 features of two neighbouring keys: the transposed V tile is then written two keys (one dword)
    // at a time
    typedef _Float16 half2v __attribute__((ext_vector_type(2)));
    for (int id = tid; id < nkb * 16 * 8; id += 64 * NKB) {
        const int key = (id >> 3) * 2, c8 = id & 7;
        half8 k0, k1, v0, v1;
#pragma unroll
        for (int j = 0; j < 8; ++j) { k0[j] = k1[j] = v0[j] = v1[j] = (half_t)0; }
        if (key < L) {
            k0 = *(const half8*)(base + key * row_pitch + hidden + c8 * 8);
            v0 = *(const half8*)(base + key * row_pitch + 2 * hidden + c8 * 8);
        }
        if (key + 1 < L) {
            k1 = *(const half8*)(base + (key + 1) * row_pitch + hidden + c8 * 8);
            v1 = *(const half8*)(base + (key + 1) * row_pitch + 2 * hidden + c8 * 8);
        }
        *(half8*)(Ks + key * ATT_LDK + c8 * 8) = k0;
        *(half8*)(Ks + (key + 1) * ATT_LDK + c8 * 8) = k1;
#pragma unroll
        for (int j = 0; j < 8; ++j) *(half2v*)(Vt + (c8 * 8 + j) * ATT_LDV + key) = half2v{v0[j], v1[j]};
    }
    __syncthreads();

    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, lh = lane >> 5;
    const int q0 = wave * 32;
    if (q0 >= S) return;
    const bool row_ok = q0 + l32 < S;       // a ragged last block: rows at or beyond S are not written
    half_t* orow = out + ((long long)b * S + q0 + l32) * hidden + h * ATT_D;
    if (q0 >= L) {                          // whole query block is padding: defined output, no work
        half4 z = {(half_t)0, (half_t)0, (half_t)0, (half_t)0};
        if (row_ok) {
#pragma unroll
            for (int i = 0; i < 8; ++i) *(half4*)(orow + 8 * i + 4 * lh) = z;
        }
        return;
    }

    half8 qf[4];
    const half_t* qrow = base + (long long)(row_ok ? q0 + l32 : S - 1) * row_pitch;   // ... and read a row that exists
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) qf[ks] = *(const half8*)(qrow + ks * 16 + lh * 8);

    floatx16 sc[NKB];
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {
#pragma unroll
        for (int v = 0; v < 16; ++v) sc[kb][v] = 0.f;
        if (kb < nkb) {
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const half8 kf = *(const half8*)(Ks + (kb * 32 + l32) * ATT_LDK + ks * 16 + lh * 8);
                sc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf, qf[ks], sc[kb], 0, 0, 0);
            }
        }
    }
    // lane holds scores of query q0+l32 against keys kb*32 + 8g + 4*lh + j  (v = 4g + j)
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int key = kb * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
            if (key < L) mx = fmaxf(mx, sc[kb][v]);
        }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float scale = 0.125f;             // 1/sqrt(64)
    float sum = 0.f;
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int key = kb * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
            const float pv = key < L ? __expf((sc[kb][v] - mx) * scale) : 0.f;
            sc[kb][v] = pv;
            sum += pv;
        }
    sum += __shfl_xor(sum, 32, 64);
    const float inv = 1.f / sum;

    floatx16 oacc[2];
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[db][v] = 0.f;
    const int nsteps = (L + 15) >> 4;       // 16-key steps with at least one valid key
#pragma unroll
    for (int st = 0; st < 2 * NKB; ++st) {
        if (st < nsteps) {
            half8 pf;
#pragma unroll
            for (int j = 0; j < 8; ++j) pf[j] = (half_t)sc[st >> 1][(st & 1) * 8 + j];
#pragma unroll
            for (int db = 0; db < 2; ++db) {
                const half_t* vrow = Vt + (db * 32 + l32) * ATT_LDV + st * 16 + 4 * lh;
                const half4 lo = *(const half4*)vrow;
                const half4 hi = *(const half4*)(vrow + 8);
                half8 vf;
#pragma unroll
                for (int j = 0; j < 4; ++j) { vf[j] = lo[j]; vf[4 + j] = hi[j]; }
                oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, pf, oacc[db], 0, 0, 0);
            }
        }
    }
    // lane holds out[q0+l32][db*32 + 8g + 4*lh + j]
    if (!row_ok) return;
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            half4 o;
#pragma unroll
            for (int j = 0; j < 4; ++j) o[j] = (half_t)(oacc[db][4 * g + j] * inv);
            *(half4*)(orow + db * 32 + 8 * g + 4 * lh) = o;
        }
}

int launch_attention(const half_t* qkv, const int32_t* valid_len, int B, int S, int heads, half_t* out, int hp,
                     hipStream_t stream) {
    if (!qkv || !valid_len || !out || B <= 0 || heads <= 0) { set_error("attention: invalid arguments"); return -1; }
    if (S <= 0 || S > 256) { set_error("attention: sequence length %d must be in 1..256", S); return -5; }
    if ((long long)B * heads > 0x7fffffffLL) { set_error("attention: grid too large"); return -5; }
    const dim3 grid((unsigned)(B * heads));
    auto lds_bytes = [](int nkb) { return (size_t)(32 * nkb * ATT_LDK + ATT_D * (32 * nkb + 8)) * sizeof(half_t); };
    if (S <= 128) {
        hipLaunchKernelGGL(attention_kernel<4>, grid, dim3(256), lds_bytes(4), stream, qkv, valid_len, S, heads, out, hp);
    } else {
        static std::atomic<bool> configured{false};      // more than 64 KB of LDS has to be asked for once
        if (!configured.load(std::memory_order_acquire)) {
            hipError_t ea = hipFuncSetAttribute(reinterpret_cast<const void*>(&attention_kernel<8>),
                                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes(8));
            if (ea != hipSuccess) { set_error("attention: hipFuncSetAttribute: %s", hipGetErrorString(ea)); return -2; }
            configured.store(true, std::memory_order_release);
        }
        hipLaunchKernelGGL(attention_kernel<8>, grid, dim3(512), lds_bytes(8), stream, qkv, valid_len, S, heads, out, hp);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_error("attention launch: %s", hipGetErrorString(e)); return -2; }
    return 0;
}

}  // namespace strait
