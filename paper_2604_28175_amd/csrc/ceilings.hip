// Measured ceilings of one MI355X for the quantities the kernels of this library are bound by.  A stand-alone program
// (built next to the library as paper_2604_28175_amd/ceilings); it is not part of the served path.
//
//   1. v_mfma_f32_32x32x16_f16 from registers: constant operands, and operands that differ from instruction to
//      instruction (pseudo-random bits): the switching activity of real data lowers the clock the chip sustains.
//   2. the same MFMA fed from LDS with the convolution kernel's operand layout (64 x 64 outputs per wavefront, 16-byte
//      fragment reads, one barrier per 64-wide slice), no global memory traffic.
//   3. streaming kernels: fill, read-only reduction, copy (16 bytes per lane, grid-stride), at a size that fits the
//      256 MB memory-side cache and at sizes that do not.
//   4. pinned host-to-device hipMemcpyAsync.
//   5. the cadence of dependent launches on one stream: an empty kernel, and a kernel whose single workgroup makes one
//      round trip to memory (load, then a dependent store), which is what the shortest possible layer costs.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

#define CK(x)                                                                                     \
    do {                                                                                          \
        hipError_t e_ = (x);                                                                      \
        if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 1; } \
    } while (0)

template <bool RANDOM>
__global__ void __launch_bounds__(256) mfma_regs(float* out, int iters) {
    half8 a[4], b[4];
    unsigned s = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 8; ++j) {
            s = s * 1664525u + 1013904223u;
            a[i][j] = RANDOM ? (_Float16)(((int)(s >> 20) - 2048) * (1.f / 1024.f)) : (_Float16)1.f;
            s = s * 1664525u + 1013904223u;
            b[i][j] = RANDOM ? (_Float16)(((int)(s >> 20) - 2048) * (1.f / 1024.f)) : (_Float16)0.5f;
        }
    floatx16 acc[4];
    for (int i = 0; i < 4; ++i)
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    for (int it = 0; it < iters; it += 4) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[(i + u) & 3], acc[i], 0, 0, 0);
    }
    float r = 0;
    for (int i = 0; i < 4; ++i)
        for (int v = 0; v < 16; ++v) r += acc[i][v];
    out[blockIdx.x * 256 + threadIdx.x] = r;
}

// 128 x 128 x 64 slice in LDS (A: 128 rows of 64 halfs, B likewise, 16-byte chunks XOR-swizzled by row); four wavefronts,
// 64 x 64 outputs each; per 16-wide step a wavefront reads 2 + 2 fragments and issues 4 MFMAs.
__global__ void __launch_bounds__(256) mfma_lds(float* out, int iters) {
    __shared__ __attribute__((aligned(16))) _Float16 smem[2 * 128 * 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, lh = lane >> 5;
    unsigned s = tid * 2654435761u + 99u;
    for (int i = tid; i < 2 * 128 * 64; i += 256) {
        s = s * 1664525u + 1013904223u;
        smem[i] = (_Float16)(((int)(s >> 20) - 2048) * (1.f / 1024.f));
    }
    __syncthreads();
    const _Float16* A = smem + (wave & 1) * 64 * 64;
    const _Float16* B = smem + 128 * 64 + (wave >> 1) * 64 * 64;
    floatx16 acc[2][2];
    for (int a = 0; a < 2; ++a)
        for (int b = 0; b < 2; ++b)
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            half8 af[2], bf[2];
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                const int row = a * 32 + l32;
                af[a] = *(const half8*)(A + row * 64 + (((ks * 2 + lh) ^ ((row >> 1) & 7)) * 8));
                bf[a] = *(const half8*)(B + row * 64 + (((ks * 2 + lh) ^ ((row >> 1) & 7)) * 8));
            }
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[a], bf[b], acc[a][b], 0, 0, 0);
        }
        __syncthreads();
    }
    float r = 0;
    for (int a = 0; a < 2; ++a)
        for (int b = 0; b < 2; ++b)
            for (int v = 0; v < 16; ++v) r += acc[a][b][v];
    out[blockIdx.x * 256 + tid] = r;
}

__global__ void __launch_bounds__(256) stream_fill(uint4* dst, size_t n16) {
    const uint4 v = make_uint4(1, 2, 3, 4);
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = v;
}
__global__ void __launch_bounds__(256) stream_copy(const uint4* src, uint4* dst, size_t n16) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}
__global__ void __launch_bounds__(256) stream_read(const uint4* src, unsigned* out, size_t n16) {
    unsigned acc = 0;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) {
        const uint4 v = src[i];
        acc += v.x ^ v.y ^ v.z ^ v.w;
    }
    if (acc == 0x12345678u) out[0] = acc;             // practically never: keeps the loads alive
}

__global__ void empty_kernel() {}
__global__ void __launch_bounds__(256) round_trip_kernel(const float* src, float* dst) { dst[threadIdx.x] = src[threadIdx.x] + 1.f; }

int main() {
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    float* out;
    CK(hipMalloc(&out, 2048 * 256 * 4));
    float ms = 0;
    printf("MI355X ceilings (this box, this run)\n\n");

    printf("1. v_mfma_f32_32x32x16_f16 from registers, 4 accumulators per wavefront, 20000 x 4 MFMAs per wavefront\n");
    for (int blocks : {512, 1024, 2048}) {
        for (int random = 0; random < 2; ++random) {
            for (int rep = 0; rep < 2; ++rep) {
                CK(hipEventRecord(e0));
                if (random) hipLaunchKernelGGL(mfma_regs<true>, dim3(blocks), dim3(256), 0, 0, out, 20000);
                else hipLaunchKernelGGL(mfma_regs<false>, dim3(blocks), dim3(256), 0, 0, out, 20000);
                CK(hipEventRecord(e1));
                CK(hipEventSynchronize(e1));
                CK(hipEventElapsedTime(&ms, e0, e1));
            }
            printf("   %4d workgroups (%d wavefronts per SIMD), %s operands: %7.1f TFLOP/s\n", blocks, blocks / 256,
                   random ? "random  " : "constant", (double)blocks * 4 * 20000 * 4 * 32768.0 / (ms * 1e-3) / 1e12);
        }
    }
    printf("\n2. the same MFMA fed from LDS (128 x 128 x 64 slice, 64 x 64 outputs per wavefront, barrier per slice, random data)\n");
    for (int blocks : {256, 512, 1024}) {
        for (int rep = 0; rep < 2; ++rep) {
            CK(hipEventRecord(e0));
            hipLaunchKernelGGL(mfma_lds, dim3(blocks), dim3(256), 0, 0, out, 4000);
            CK(hipEventRecord(e1));
            CK(hipEventSynchronize(e1));
            CK(hipEventElapsedTime(&ms, e0, e1));
        }
        printf("   %4d workgroups (%d per compute unit): %7.1f TFLOP/s\n", blocks, blocks / 256,
               (double)blocks * 4 * 4000 * 16 * 32768.0 / (ms * 1e-3) / 1e12);
    }

    printf("\n3. streaming kernels, 16 bytes per lane, 4096 workgroups of 256 threads, grid-stride\n");
    const size_t cap = (size_t)2048 << 20;
    uint4 *a, *b;
    unsigned* flag;
    CK(hipMalloc(&a, cap));
    CK(hipMalloc(&b, cap));
    CK(hipMalloc(&flag, 4));
    CK(hipMemset(a, 1, cap));
    CK(hipMemset(b, 2, cap));
    for (size_t mb : {(size_t)64, (size_t)512, (size_t)2048}) {
        const size_t n16 = (mb << 20) / 16;
        float t[3] = {0, 0, 0};
        for (int k = 0; k < 3; ++k) {
            for (int rep = 0; rep < 6; ++rep) {
                if (rep == 1) CK(hipEventRecord(e0));
                if (k == 0) hipLaunchKernelGGL(stream_fill, dim3(4096), dim3(256), 0, 0, b, n16);
                else if (k == 1) hipLaunchKernelGGL(stream_read, dim3(4096), dim3(256), 0, 0, a, flag, n16);
                else hipLaunchKernelGGL(stream_copy, dim3(4096), dim3(256), 0, 0, a, b, n16);
            }
            CK(hipEventRecord(e1));
            CK(hipEventSynchronize(e1));
            CK(hipEventElapsedTime(&t[k], e0, e1));
            t[k] /= 5;
        }
        const double by = (double)(mb << 20);
        printf("   %5zu MiB: fill %5.2f TB/s   read %5.2f TB/s   copy %5.2f TB/s (read + written bytes)\n", mb, by / (t[0] * 1e-3) / 1e12,
               by / (t[1] * 1e-3) / 1e12, 2 * by / (t[2] * 1e-3) / 1e12);
    }

    printf("\n4. pinned host memory -> device, hipMemcpyAsync on a stream\n");
    void* host;
    CK(hipHostMalloc(&host, (size_t)256 << 20, hipHostMallocDefault));
    for (size_t i = 0; i < ((size_t)256 << 20); i += 4096) ((char*)host)[i] = 1;
    hipStream_t st;
    CK(hipStreamCreate(&st));
    for (size_t mb : {(size_t)2, (size_t)19, (size_t)38, (size_t)256}) {
        for (int rep = 0; rep < 4; ++rep) {
            if (rep == 1) CK(hipEventRecord(e0, st));
            CK(hipMemcpyAsync(a, host, mb << 20, hipMemcpyHostToDevice, st));
        }
        CK(hipEventRecord(e1, st));
        CK(hipEventSynchronize(e1));
        CK(hipEventElapsedTime(&ms, e0, e1));
        printf("   %4zu MiB: %5.1f GB/s (%.3f ms per copy)\n", mb, (double)(mb << 20) * 3 / (ms * 1e-3) / 1e9, ms / 3);
    }

    printf("\n5. dependent launches on one stream (1000 in a row, events around them)\n");
    for (int kind = 0; kind < 3; ++kind) {
        for (int rep = 0; rep < 2; ++rep) {
            CK(hipEventRecord(e0, st));
            for (int i = 0; i < 1000; ++i) {
                if (kind == 0) hipLaunchKernelGGL(empty_kernel, dim3(1), dim3(64), 0, st);
                else if (kind == 1) hipLaunchKernelGGL(round_trip_kernel, dim3(1), dim3(256), 0, st, (const float*)a + (i & 1) * 256, (float*)a + ((i + 1) & 1) * 256);
                else hipLaunchKernelGGL(round_trip_kernel, dim3(256), dim3(256), 0, st, (const float*)a + (i & 1) * 256, (float*)a + ((i + 1) & 1) * 256);
            }
            CK(hipEventRecord(e1, st));
            CK(hipEventSynchronize(e1));
            CK(hipEventElapsedTime(&ms, e0, e1));
        }
        printf("   %-58s %5.2f us per launch\n", kind == 0 ? "empty kernel, one wavefront:" : kind == 1 ? "load + dependent store, one workgroup:" : "load + dependent store, 256 workgroups (same addresses):", ms);
    }
    return 0;
}
