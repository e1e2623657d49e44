// Internal launcher interface between the runtime and the gfx950 kernels.
// Every launcher validates the operand shapes its kernel and grid assume and returns a
// negative status (see strait.h) instead of launching when they do not hold.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace strait {

typedef _Float16 half_t;

enum Act { ACT_NONE = 0, ACT_RELU = 1, ACT_RELU6 = 2, ACT_GELU = 3 };

// One implicit-GEMM convolution (or plain GEMM) launch.
//   y[m, k] = act(bias[k] + sum_{r,s,c} x[addr(m) + r*sH + s*sW + c] * w[k*ldw + (r*S + s)*C + c] (+ res[m*ldy + k]))
// with m = (n, p, q), addr(m) = n*sN + (p*stride - pad)*sH + (q*stride_w - pad_w)*sW, taps outside
// [0,H) x [0,W) contributing zero.  A plain NHWC convolution has sW = C, sH = W*C, sN = H*W*C;
// the decoupled strides also describe a channel-padded, spatially pre-padded stem input whose
// taps along a row are contiguous ("virtual" 1-wide kernel with C = taps*Cpad).
struct ConvParams {
    const half_t* x;
    const half_t* w;
    const float* bias;       // [Cout] or nullptr
    const half_t* res;       // [M][ldy] or nullptr
    void* y;                 // fp16 (or fp32 when out_f32) [M][ldy]
    int M;                   // N * P * Q
    int PQ, Q;
    int H, W, C, R, S;
    int stride_h, stride_w, pad_h, pad_w;
    long long sN;
    int sH, sW;
    int Kg;                  // R * S * C
    int ldw;                 // weight row pitch in elements (multiple of 8, zero padded past Kg)
    int Cout, ldy;
    int act;
    int out_f32;
    int hp;                  // raise wave priority (high-priority batch)
    long long x_elems;       // extent of x in elements; filled in by launch_conv
    float* ws;               // optional split-K workspace (16-byte aligned) and its size in bytes
    size_t ws_bytes;
    int ksplit;              // filled in by launch_conv
    int tiles_n_shift;       // log2 of the number of tiles along Cout, or -1; filled in by the launcher
    int strip_w;             // 3x3 patch kernel: width of the strips a row is cut into; filled in by the launcher
    // Optional second source of a 1x1 convolution with stride 1 (a block-closing convolution that absorbs the block's 1x1
    // projection shortcut): reduction elements [C, C + K2) are x2[n*sN2 + p*stride2*sH2 + q*stride2*sW2 + (k - C)], and
    // w is [Cout][C + K2].  Kg = C + K2; no res.
    const half_t* x2;
    int K2, stride2, sH2, sW2;
    long long sN2;
    long long x2_elems;      // extent of x2 in elements; filled in by launch_conv
};

int launch_conv(const ConvParams& p, hipStream_t stream);

// Two chained pointwise convolutions in one launch (pointwise_pair.hip):
//   y[m, 0:N1] = act1(x[m, 0:K1] w3^T + b3 (+ res[m, 0:N1]));   z[m, 0:N2] = act2(y[m, 0:N1] w1^T + b1)
// x [M][K1], w3 [N1][K1], res and y [M][N1], w1 [N2][N1], z [M][N2], all dense fp16; biases fp32 or nullptr.
// z must not share memory with x or res (other workgroups may still be reading them).
// With x2 (a second input [M][K2], for a block whose shortcut is a 1x1 projection of x2) the first product is
// [x | x2] w3^T with w3 [N1][K1 + K2], and there is no res.
struct PairParams {
    const half_t* x; const half_t* w3; const float* b3; const half_t* res; half_t* y;
    const half_t* w1; const float* b1; half_t* z;
    int M, K1, N1, N2, act1, act2, hp;
    const half_t* x2; int K2;
};
bool pointwise_pair_supported(int K1, int N1, int N2);
bool pointwise_pair_proj_supported(int K1, int K2, int N1, int N2);
int launch_pointwise_pair(const PairParams& p, hipStream_t stream);

int launch_pack_input(const half_t* x, int N, int H, int W, int C, half_t* y, int Hp, int Wp, int Cpad,
                      int pad_top, int pad_left, int hp, hipStream_t stream);
// 7x7 stride-2 pad-3 convolution of a 3-channel image to 64 channels + bias + ReLU + 3x3 stride-2 pad-1 max pooling.
// wf: [64][176] fp16, row k = 22 fragments of 8: fragment 3r + j holds halfs 8j..8j+7 of filter row r's 24-half window
// {0, w[k][r][s=0][c=0..2], ..., w[k][r][6][0..2], 0, 0}; the 22nd fragment is zero.  W even.
// w1 [64][64] fp16, b1 [64] fp32 or nullptr, t1 like y: optionally also t1 = relu(y w1^T + b1), the 1x1 convolution behind it
int launch_stem_pool(const half_t* x, const half_t* wf, const float* bias, int N, int H, int W, half_t* y, int hp,
                     hipStream_t stream, const half_t* w1 = nullptr, const float* b1 = nullptr, half_t* t1 = nullptr);
// 3x3 stride-2 pad-1 convolution of a 3-channel image to Kout <= 32 channels + bias + activation (stem3x3.hip).
// wf: [32][48] fp16, row k = 3 filter rows x 16 halfs {0, w[k][r][s=0][c=0..2], w[k][r][1][..], w[k][r][2][..], 0 x 6}; rows
// from Kout on zero.  W even, Kout a multiple of 8.
int launch_stem3x3s2(const half_t* x, const half_t* wf, const float* bias, int N, int H, int W, int Kout, int act, half_t* y, int hp,
                     hipStream_t stream);
// The same stem (32 output channels) with a stride-1 depthwise 3x3 behind it (wd_rsc [3][3][32], + bd, act2) in one launch;
// y [N,P,Q,32].  Bit-identical to launch_stem3x3s2 followed by launch_dwconv3x3.
int launch_stem3x3s2_dw(const half_t* x, const half_t* wf, const float* bias, int act1, const half_t* wd_rsc, const float* bd, int act2,
                        int N, int H, int W, half_t* y, int hp, hipStream_t stream);
// 1x1 convolution Cin -> Chid (+ b1, act1) and the depthwise 3x3 of stride 1 or 2, padding 1, behind it (+ bd, act2) in one
// launch (expand_dw.hip): x [N,H,W,Cin] -> y [N,P,Q,Chid]; w1 [Chid][ldw1], wd_rsc [3][3][Chid].  Bit-identical to the two
// launches.  expand_dw_supported: whether the kernel takes these channel counts and this stride.
bool expand_dw_supported(int Cin, int Chid, int stride);
int launch_expand_dw(const half_t* x, int N, int H, int W, int Cin, const half_t* w1, int ldw1, const float* b1, int Chid, int act1,
                     const half_t* wd_rsc, const float* bd, int stride, int act2, half_t* y, int hp, hipStream_t stream);
int launch_dwconv3x3(const half_t* x, int N, int H, int W, int C, const half_t* w_rsc, const float* bias,
                     int stride, int act, half_t* y, int hp, hipStream_t stream);
int launch_maxpool3x3s2(const half_t* x, int N, int H, int W, int C, half_t* y, int hp, hipStream_t stream);
int launch_maxpool2x2s2(const half_t* x, int N, int H, int W, int C, half_t* y, int hp, hipStream_t stream);
int launch_vit_tokens(const half_t* patch, const float* cls, const float* pos, int N, int T, int D, half_t* z, int hp,
                      hipStream_t stream);
int launch_global_avgpool(const half_t* x, int N, int HW, int C, half_t* y, int hp, hipStream_t stream);
int launch_softmax_top1(const float* logits, int rows, int n, float* probs, int32_t* top1, int hp,
                        hipStream_t stream);
// x_row_stride: elements between consecutive input rows (0 = n); the output rows are contiguous.
int launch_layernorm(const half_t* x, const float* gamma, const float* beta, int rows, int n, float eps,
                     half_t* y, int hp, hipStream_t stream, long long x_row_stride = 0);
int launch_attention(const half_t* qkv, const int32_t* valid_len, int B, int S, int heads, half_t* out, int hp,
                     hipStream_t stream);
int launch_argmax_f16(const half_t* x, int rows, int n, long long row_stride, int32_t* top1, int hp,
                      hipStream_t stream);
// Weight preparation on the device (load time): BatchNorm fold + OIHW -> kernel layout.
int launch_fill_zero(void* p, size_t bytes, hipStream_t stream);
// Copies `bytes` (multiple of 4) from device memory to host memory the GPU can address, with a kernel.
int launch_copy_mapped(const void* src, void* dst, size_t bytes, int hp, hipStream_t stream);

void set_error(const char* fmt, ...);

}  // namespace strait
