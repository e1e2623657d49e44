// strait_k_gemm_noalloc: the GEMM entry point for callers that may not allocate device memory
// (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).
//
// strait_k_gemm gives small products a split-K workspace (fp32 partial sums, one slab per slice of the
// reduction, summed by a second kernel) that it allocates and frees around the launch.  Here the same
// kernels get the same amount of workspace from a static device array instead.  The array exists once
// per GPU for the life of the process; every call on a GPU shares it, so calls that overlap on one GPU
// race on it (calls on one stream, or otherwise ordered, are fine).  Nothing in it has to start at
// zero: the first kernel writes every element of every slab the second one reads.
#include <mutex>

#include "../../include/strait.h"
#include "kernels.hpp"

namespace {

constexpr size_t SCRATCH_BYTES = 16u << 20;           // the workspace strait_k_gemm allocates per call
constexpr long long MAX_OUTPUTS = 128LL * 4096;       // the largest M * N for which strait_k_gemm uses one
constexpr int MAX_DEVICES = 64;

static __device__ __align__(256) __attribute__((used)) unsigned char scratch[SCRATCH_BYTES];

std::mutex g_mu;
void* g_scratch_ptr[MAX_DEVICES] = {nullptr};         // device address of `scratch` on each GPU

// The array's device address on the current GPU (each GPU holds its own copy at its own address); looked
// up once per device.  The array's name itself is only a host-side handle and is never passed to a kernel.
int scratch_on_current_device(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { strait::set_error("gemm_noalloc: hipGetDevice: %s", hipGetErrorString(e)); return STRAIT_E_HIP; }
    if (dev < 0 || dev >= MAX_DEVICES) { strait::set_error("gemm_noalloc: device %d out of range", dev); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            strait::set_error("gemm_noalloc: hipGetSymbolAddress: %s", hipGetErrorString(e));
            return STRAIT_E_HIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return STRAIT_OK;
}

}  // namespace

extern "C" strait_status strait_k_gemm_noalloc(void* stream, const void* x, const void* w, const float* bias, int32_t M,
                                               int32_t N, int32_t K, int32_t act, const void* res, void* y,
                                               int32_t out_f32, int32_t hp) {
    using namespace strait;
    if (M <= 0 || N <= 0 || K <= 0 || K % 8 != 0) { set_error("gemm_noalloc: needs positive sizes and K %% 8 == 0"); return STRAIT_E_SHAPE; }
    if ((long long)M * N > MAX_OUTPUTS) {
        set_error("gemm_noalloc: M * N = %lld exceeds the %lld outputs the static workspace is sized for "
                  "(larger products use no workspace: strait_k_gemm allocates nothing for them)", (long long)M * N, MAX_OUTPUTS);
        return STRAIT_E_SHAPE;
    }
    void* ws = nullptr;
    const int rc = scratch_on_current_device(&ws);
    if (rc) return rc;
    ConvParams p{};
    p.x = (const half_t*)x; p.w = (const half_t*)w; p.bias = bias; p.res = (const half_t*)res; p.y = y;
    p.M = M; p.PQ = 1; p.Q = 1; p.H = 1; p.W = 1; p.C = K; p.R = 1; p.S = 1;
    p.stride_h = p.stride_w = 1; p.pad_h = p.pad_w = 0;
    p.sN = K; p.sH = K; p.sW = K; p.Kg = K; p.ldw = K; p.Cout = N; p.ldy = N; p.act = act; p.out_f32 = out_f32; p.hp = hp;
    p.ws = (float*)ws; p.ws_bytes = SCRATCH_BYTES;
    return launch_conv(p, (hipStream_t)stream);
}
