/*
 * CPU oracle, convolution and pooling loops.  TEST INFRASTRUCTURE ONLY: this file is the
 * checker for the GPU library and is never part of the served path.
 *
 * Each routine is the textbook definition written as nested loops, NHWC activations:
 *
 *   conv2d   y[n,p,q,k] = b[k] + sum_{r,s,c} x[n, p*stride+r-pad, q*stride+s-pad, c] * w[r,s,c,k]
 *            (zero outside the image; output size floor((H+2*pad-R)/stride)+1)
 *   dwconv   y[n,p,q,c] = b[c] + sum_{r,s}   x[n, p*stride+r-pad, q*stride+s-pad, c] * w[r,s,c]
 *   maxpool  y[n,p,q,c] = max over the in-bounds taps of the window (padding never wins)
 *
 * These are the operators of the kernel sequence a served batch executes (Section 2,
 * "executing a batch is equivalent to executing a sequence of kernels"; Section 3.2 step (2)).
 * Activations and accumulators are `real` (double in the oracle proper; a float build exists
 * only to measure the oracle's own rounding).  Weights are passed as float because every
 * stored weight is an fp16 value.  OpenMP splits independent output rows only.
 */
#include <stddef.h>
#include <stdint.h>
#include <math.h>

#ifndef REAL
#define REAL double
#endif
#ifndef SUFFIX
#define SUFFIX f64
#endif
#define CAT_(a, b) a##_##b
#define CAT(a, b) CAT_(a, b)
#define FN(name) CAT(name, SUFFIX)

typedef REAL real;

#ifdef ORACLE_COMMON
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
#endif

void FN(oracle_conv2d)(const real* x, int N, int H, int W, int C,
                       const float* w /* [R][S][C][K] */, const real* b /* [K] or NULL */,
                       int K, int R, int S, int stride, int pad, real* y)
{
    const int P = (H + 2 * pad - R) / stride + 1;
    const int Q = (W + 2 * pad - S) / stride + 1;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int n = 0; n < N; ++n)
        for (int p = 0; p < P; ++p) {
            for (int q = 0; q < Q; ++q) {
                real* acc = y + (((size_t)n * P + p) * Q + q) * K;
                for (int k = 0; k < K; ++k) acc[k] = b ? b[k] : (real)0;
                for (int r = 0; r < R; ++r) {
                    const int ih = p * stride + r - pad;
                    if (ih < 0 || ih >= H) continue;
                    for (int s = 0; s < S; ++s) {
                        const int iw = q * stride + s - pad;
                        if (iw < 0 || iw >= W) continue;
                        const real* xp = x + (((size_t)n * H + ih) * W + iw) * C;
                        const float* wp = w + ((size_t)r * S + s) * C * K;
                        for (int c = 0; c < C; ++c) {
                            const real xv = xp[c];
                            const float* wk = wp + (size_t)c * K;
                            for (int k = 0; k < K; ++k) acc[k] += xv * (real)wk[k];
                        }
                    }
                }
            }
        }
}

void FN(oracle_dwconv2d)(const real* x, int N, int H, int W, int C,
                         const float* w /* [R][S][C] */, const real* b /* [C] or NULL */,
                         int R, int S, int stride, int pad, real* y)
{
    const int P = (H + 2 * pad - R) / stride + 1;
    const int Q = (W + 2 * pad - S) / stride + 1;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int n = 0; n < N; ++n)
        for (int p = 0; p < P; ++p) {
            for (int q = 0; q < Q; ++q) {
                real* acc = y + (((size_t)n * P + p) * Q + q) * C;
                for (int c = 0; c < C; ++c) acc[c] = b ? b[c] : (real)0;
                for (int r = 0; r < R; ++r) {
                    const int ih = p * stride + r - pad;
                    if (ih < 0 || ih >= H) continue;
                    for (int s = 0; s < S; ++s) {
                        const int iw = q * stride + s - pad;
                        if (iw < 0 || iw >= W) continue;
                        const real* xp = x + (((size_t)n * H + ih) * W + iw) * C;
                        const float* wp = w + ((size_t)r * S + s) * C;
                        for (int c = 0; c < C; ++c) acc[c] += xp[c] * (real)wp[c];
                    }
                }
            }
        }
}

void FN(oracle_maxpool2d)(const real* x, int N, int H, int W, int C,
                          int k, int stride, int pad, real* y)
{
    const int P = (H + 2 * pad - k) / stride + 1;
    const int Q = (W + 2 * pad - k) / stride + 1;
#pragma omp parallel for collapse(2)
    for (int n = 0; n < N; ++n)
        for (int p = 0; p < P; ++p)
            for (int q = 0; q < Q; ++q) {
                real* out = y + (((size_t)n * P + p) * Q + q) * C;
                for (int c = 0; c < C; ++c) out[c] = -INFINITY;
                for (int r = 0; r < k; ++r) {
                    const int ih = p * stride + r - pad;
                    if (ih < 0 || ih >= H) continue;
                    for (int s = 0; s < k; ++s) {
                        const int iw = q * stride + s - pad;
                        if (iw < 0 || iw >= W) continue;
                        const real* xp = x + (((size_t)n * H + ih) * W + iw) * C;
                        for (int c = 0; c < C; ++c)
                            if (xp[c] > out[c]) out[c] = xp[c];
                    }
                }
            }
}
