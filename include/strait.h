/*
 * strait.h -- C ABI of the MI355X (gfx950) hot path under a dual-priority inference server.
 *
 * The served unit is a *batch of one model*.  Following the paper's description of what
 * happens to a batch on a discrete GPU (Section 3.2, "Interference Prediction", steps (1)-(3)):
 *   (1) the input is written to pinned host memory and copied host-to-device,
 *   (2) a sequence of dependent kernels runs,
 *   (3) the result is copied back to pinned host memory,
 * and every model carries one of two priority levels that selects the stream its batches are
 * issued on (Section 3.1, "Priority Level").  Several batches may be in flight on one GPU at
 * once ("spatial sharing", Section 1/2).  On completion the measured transfer and kernel
 * latencies of the batch are reported (Section 3.2 "Online calibration"; Section 3.3, last
 * paragraph; Section 5.1 "Evaluation Metrics").  Model instances own their pinned staging
 * buffers and execution resources (Section 4, "Implementation").
 *
 * Conventions
 *   - every function returns a strait_status (0 = OK, negative = error); nothing throws or
 *     aborts across this boundary.  strait_last_error() gives a per-thread message.
 *   - "host" pointers are ordinary host memory; "device" pointers are HIP device memory of the
 *     context's GPU; streams are hipStream_t passed as void*.
 *   - the library never creates, destroys or changes the streams handed to it.
 *   - all activations are fp16 (IEEE binary16), NHWC; accumulation is fp32.
 *   - one GPU per context; no collectives.
 */
#ifndef STRAIT_H
#define STRAIT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t strait_status;
enum {
    STRAIT_OK = 0,
    STRAIT_E_INVALID = -1,     /* bad argument (null, out of range, misaligned)            */
    STRAIT_E_HIP = -2,         /* a HIP call failed; message has hipGetErrorString          */
    STRAIT_E_FORMAT = -3,      /* weight container malformed or a tensor missing/misshaped  */
    STRAIT_E_NOMEM = -4,       /* host or device allocation failed                          */
    STRAIT_E_SHAPE = -5,       /* operand shapes the kernels do not support                 */
    STRAIT_E_BUSY = -6,        /* no idle instance (submit) / work still in flight (free)   */
    STRAIT_E_BATCH = -7        /* batch < 1 or batch > max_batch                            */
};

typedef enum { STRAIT_PRIO_HIGH = 0, STRAIT_PRIO_LOW = 1 } strait_priority;

typedef enum {
    STRAIT_ARCH_TINY_CNN = 0,      /* conv3x3 x3 + GAP + FC + softmax                        */
    STRAIT_ARCH_RESNET50 = 1,      /* ResNet-50 v1.5, BatchNorm folded at load               */
    STRAIT_ARCH_MOBILENETV2 = 2,   /* MobileNetV2 1.0                                        */
    STRAIT_ARCH_ENCODER = 3,       /* post-LayerNorm Transformer encoder stack               */
    STRAIT_ARCH_VGG19 = 4,         /* VGG-19 (configuration E, no normalisation); hyper = {H, W, 3, classes, fc width} */
    STRAIT_ARCH_VIT = 5            /* Vision Transformer, 16x16 patches, pre-LayerNorm blocks; hyper = {H, W, 3,
                                      classes, layers, hidden, heads, ffn}; input and output as the CNNs'      */
} strait_arch;

typedef enum { STRAIT_ACT_NONE = 0, STRAIT_ACT_RELU = 1, STRAIT_ACT_RELU6 = 2, STRAIT_ACT_GELU = 3 } strait_act;

typedef struct strait_ctx strait_ctx;
typedef struct strait_model strait_model;
typedef struct strait_ticket_s* strait_ticket;

#define STRAIT_MAX_STREAMS 8

/* Context: one GPU plus the streams the caller created for it (Section 3.1: the priority of a
 * model selects the stream its batches run on).  n_hp/n_lp >= 1, n_copy >= 1, each at most
 * STRAIT_MAX_STREAMS.  A batch of priority p is issued on compute stream p[i % n_p] and its
 * host-to-device copy on copy_streams[j % n_copy] (i, j: running counters). */
typedef struct {
    int32_t device;
    int32_t n_hp, n_lp, n_copy;
    void* hp_streams[STRAIT_MAX_STREAMS];
    void* lp_streams[STRAIT_MAX_STREAMS];
    void* copy_streams[STRAIT_MAX_STREAMS];
} strait_ctx_desc;

/* Model: `weights` is a host pointer to a weight container ("STRW" v1: 48-byte header
 * {magic, version, arch, n_tensors, hyper[8]}, 80-byte tensor entries {name[40], dtype, ndim,
 * shape[4], offset, nbytes}, fp16 payloads; conv weights OIHW, linear weights [out,in],
 * BatchNorm as separate gamma/beta/mean/var vectors).  The container is read during the call
 * only.  Load folds BatchNorm (scale = gamma/sqrt(var+1e-5) in fp32; weight*scale rounded once
 * to fp16; bias = beta - mean*scale kept fp32), re-lays weights for the kernels, uploads them
 * and creates `n_instances` instances, each with pinned staging and device buffers sized for
 * `max_batch` (Section 3, first paragraph after Figure 3; Section 4). */
typedef struct {
    const void* weights;
    size_t weights_bytes;
    int32_t max_batch;
    int32_t n_instances;
} strait_model_desc;

/* Completion record of one batch (Section 5.1: latency runs from enqueue to the result being
 * back in host memory; Section 3.2: measured H2D time; Section 3.3: measured kernel latency).
 * Times in ms are device-side (hipEventElapsedTime); *_ns are host CLOCK_MONOTONIC. */
typedef struct {
    int32_t model_id, priority, batch, instance;
    int64_t t_enqueue_ns;      /* host time at entry of strait_submit                       */
    int64_t t_issued_ns;       /* host time when everything had been enqueued               */
    int64_t t_done_ns;         /* host time the completion thread saw the D2H copy finish   */
    float h2d_ms;              /* input copy                                                */
    float kernel_ms;           /* first kernel start to last kernel end                     */
    float d2h_ms;              /* output copy                                               */
    float total_ms;            /* start of input copy to end of output copy                 */
} strait_record;

/* Per-layer accounting (pure query, valid after load). */
typedef struct {
    char name[40];
    int32_t kind;              /* 0 conv/gemm (MFMA), 1 depthwise, 2 pool, 3 softmax, 4 layernorm,
                                  5 attention, 6 pack                                       */
    int64_t macs_per_sample;   /* multiply-accumulates per image / sequence (unmasked)      */
    int64_t bytes_per_sample;  /* activation bytes read + written once, per image / sequence */
    int64_t weight_bytes;      /* parameter bytes read once per launch                      */
    int32_t gemm_m_per_sample, gemm_n, gemm_k;  /* implicit-GEMM shape (kind 0), else 0     */
} strait_layer_info;

const char* strait_last_error(void);
int32_t strait_version(void);

strait_status strait_ctx_create(const strait_ctx_desc* desc, strait_ctx** out);
strait_status strait_ctx_destroy(strait_ctx* ctx);      /* E_BUSY while models are loaded   */
/* Whether kernels of high-priority batches raise their wave priority (default on).  Turning it
 * off leaves the two levels distinguished by their streams only: the A/B for the paper's
 * ablation "without stream priority" (Appendix A.3). */
strait_status strait_ctx_set_wave_priority(strait_ctx* ctx, int32_t enabled);
/* Whether strait_submit and strait_run replay the kernel sequence of a batch from a captured
 * HIP graph (default off).  The paper's runtime executes a compiled graph "from the first kernel to
 * the last without interruption" (Section 2); here one graph per (instance, batch size, wave
 * priority) is captured on the second use of that key (kernel launches only: copies and events
 * stay outside) and replayed with one launch call afterwards.  Results are those of the
 * kernel-by-kernel path, bit for bit. */
strait_status strait_ctx_set_graphs(strait_ctx* ctx, int32_t enabled);

/* From how many output pixels (batch x height x width) on a residual block's closing 1x1 convolution and the next
 * block's opening 1x1 convolution, which reads nothing but the first one's output, run as one launch
 * (strait_k_pointwise_pair).  Default 40000 (ResNet-50 at batch 16 and above: batch 128 2.29 -> 2.20 ms, batch 64 1.233 ->
 * 1.210 ms, batch 16 0.552 -> 0.543 ms; at batch 8 and below the two launches, which may split their reductions, are 1 %
 * faster); 0 = always two launches, and every other fusion of launches off as well (projection shortcuts, the first
 * block's opening convolution inside the stem launch): the layer-by-layer plan.  Results are the same bit for bit.  A graph that strait_ctx_set_graphs has
 * already captured keeps the launches it was captured with: set this before the first batch. */
strait_status strait_ctx_set_pair_fusion(strait_ctx* ctx, int64_t min_pixels);
/* From how many output pixels on the closing 1x1 convolution of a residual stage's first block absorbs the block's 1x1
 * projection shortcut as a second source of its reduction (strait_k_conv1x1_proj; in ResNet-50's first stage, where the
 * projection has stride 1, as part of the fused pair, strait_k_pointwise_pair_proj): the projection's launch disappears,
 * and neither the projected tensor nor its read-back exists.  Default 1, i.e. always (ResNet-50: batch 128 2.21 -> 2.06 ms,
 * batch 16 0.610 -> 0.531 ms, batch 8 0.491 -> 0.468 ms, batch 1 0.452 -> 0.436 ms).  Not bit-identical to separate launches: the sum of the two
 * products is rounded to fp16 once instead of the projection first.  With strait_ctx_set_pair_fusion(ctx, 0) no pair
 * is fused, this kind included. */
strait_status strait_ctx_set_proj_fusion(strait_ctx* ctx, int64_t min_pixels);
/* Yielding of low-priority batches.  The paper separates the two levels by stream priority, "a hardware-level hint"
 * without preemption (Section 3.1), and bounds what low-priority work may take of a GPU (Section 3.3).  Where stream
 * priorities are not available this is the library's own lever: with layers_per_segment > 0 the kernel sequence of a
 * low-priority batch is enqueued in segments of that many layers, at most two segments ahead of the GPU, and no
 * further segment is enqueued while a high-priority batch is in flight on this context (for at most 5 ms per segment).
 * A high-priority batch then shares the GPU with at most the rest of two short segments.  strait_submit stays
 * non-blocking (the stream's completion thread does the issuing); results do not change.  0 (default) = the whole
 * sequence is enqueued at once. */
strait_status strait_ctx_set_lp_yield(strait_ctx* ctx, int32_t layers_per_segment);
/* Whether a plan's independent branches (the projection shortcut of a residual stage's first block) run on the
 * instance's side stream beside the main sequence (default on).  Off keeps every launch on the one compute stream, in
 * plan order: kernel traces of such a run add up to the step time. */
strait_status strait_ctx_set_branch_streams(strait_ctx* ctx, int32_t enabled);

/* How inputs travel from the instance's pinned buffer to the device (Section 2 of the paper: inputs are
 * "copied to the GPU's memory" before the kernels run; the first-in first-out link of Section 3.2).
 * Inputs of at most max_bytes are read over the host link by a copy kernel on the copy stream; larger
 * ones go by hipMemcpyAsync on the same stream.  Both sit between the same two events, so records and
 * the link model see no difference.  Default 8 MiB (every serving-sized batch): under concurrent
 * serving the asynchronous copy call of such sizes was measured to block its caller for milliseconds
 * now and then, a kernel launch never.  0 = always hipMemcpyAsync. */
strait_status strait_ctx_set_h2d_kernel_limit(strait_ctx* ctx, int64_t max_bytes);

strait_status strait_model_load(strait_ctx* ctx, const strait_model_desc* desc, strait_model** out);
strait_status strait_model_free(strait_model* m);       /* E_BUSY with batches in flight    */

/* Sizes of one batch's host input and output.
 * CNN input : fp16 [batch][H][W][3].  CNN output: fp32 logits [batch][classes], then fp32
 *             probabilities [batch][classes], then int32 top-1 [batch] (lowest index on ties).
 * Encoder in: fp16 [batch][seq][hidden] (seq <= 256, head dimension 64) (+ int32 valid_len[batch] passed separately);
 *        out: fp16 hidden states [batch][seq][hidden], then int32 argmax over the features of
 *             token 0 [batch]. */
strait_status strait_model_io(const strait_model* m, int32_t batch, size_t* in_bytes, size_t* out_bytes);
strait_status strait_model_info(const strait_model* m, int32_t* arch, int32_t* n_layers,
                                int32_t* max_batch, int32_t* n_instances, int32_t hyper[8]);
strait_status strait_model_layer(const strait_model* m, int32_t layer, strait_layer_info* out);
/* The pinned input buffer of one instance (Section 3.2 step (1): "input data is written to pinned host
 * memory"): a producer may write a batch there directly; strait_submit given this very pointer uses that
 * instance and skips its own copy into pinned memory.  capacity = bytes of a max_batch input.  The buffer
 * belongs to the library and must not be written while a batch submitted from it is in flight. */
strait_status strait_model_staging(const strait_model* m, int32_t instance, void** host_in, size_t* capacity);

/* Submit a batch at a priority level: picks an idle instance (E_BUSY if none -- never blocks),
 * copies `host_in` into the instance's pinned buffer, enqueues H2D copy, kernel sequence and
 * D2H copy without any host synchronisation, and returns a ticket.  `host_in` may be reused
 * as soon as the call returns; `host_out` must stay valid until strait_wait returns.
 * If `host_in` is the staging buffer of an instance (strait_model_staging), that instance is the one
 * used (E_BUSY if it is not idle) and the data are taken from there without a host copy; they must
 * then stay untouched until strait_wait returns.
 * `valid_len` (host, int32[batch]) is required for the encoder and ignored otherwise. */
strait_status strait_submit(strait_model* m, strait_priority prio, int32_t batch, const void* host_in,
                            const int32_t* valid_len, void* host_out, strait_ticket* ticket);
strait_status strait_poll(strait_ticket ticket, int32_t* done);
/* Blocks until the batch is complete, fills `rec` (may be NULL) and releases the ticket and
 * its instance. */
strait_status strait_wait(strait_ticket ticket, strait_record* rec);

/* Sub-steps on an explicit instance (0 <= instance < n_instances), for tests, profiling and
 * throughput runs with the input already resident in device memory.  They do not take the
 * instance from the pool: the caller must not mix them with strait_submit on the same model
 * concurrently.  All are asynchronous on the priority's compute stream (copy_in: on a copy
 * stream, with the compute stream made to wait for it); strait_sync waits for the instance. */
strait_status strait_copy_in(strait_model* m, int32_t instance, strait_priority prio, int32_t batch,
                             const void* host_in, const int32_t* valid_len);
strait_status strait_run(strait_model* m, int32_t instance, strait_priority prio, int32_t batch);
strait_status strait_copy_out(strait_model* m, int32_t instance, strait_priority prio, int32_t batch, void* host_out);
strait_status strait_sync(strait_model* m, int32_t instance, strait_priority prio);
/* Like strait_run, with a hipEvent pair around every layer; after an internal synchronise,
 * layer_ms[i] (host, float[n_layers]) holds layer i's device time: exactly 0 for a layer that was computed inside
 * another layer's launch at this batch size (its time is in that layer's figure). */
strait_status strait_run_timed(strait_model* m, int32_t instance, strait_priority prio, int32_t batch,
                               float* layer_ms);
/* Copies an intermediate activation (the output of layer `layer`) of the instance's last run
 * to host memory as fp16; `bytes` must equal the layer's output size for `batch`. */
strait_status strait_read_activation(strait_model* m, int32_t instance, int32_t layer, int32_t batch,
                                     void* host_out, size_t bytes, size_t* needed);

/* ---- kernel-level entry points: device pointers + stream -------------------------------
 * Each is one launch of one of the library's kernels, for per-operator parity checks.
 * All tensors fp16 unless noted.  `hp` != 0 raises the wave priority inside the kernel. */

/* y[n,p,q,k] = act(bias[k] + sum_{r,s,c} x[n,p*stride+r-pad,q*stride+s-pad,c] * w[k,r,s,c] (+ res[n,p,q,k]))
 * x [N,H,W,C], w [K][R][S][C] ("KRSC"), bias fp32 [K] or NULL, res [N,P,Q,K] or NULL, y [N,P,Q,K]
 * (fp32 when out_f32 != 0).  The operator of Section 3.2 step (2) for convolution layers. */
strait_status strait_k_conv2d(void* stream, const void* x, int32_t N, int32_t H, int32_t W, int32_t C,
                              const void* w_krsc, const float* bias, int32_t K, int32_t R, int32_t S,
                              int32_t stride, int32_t pad, int32_t act, const void* res, void* y,
                              int32_t out_f32, int32_t hp);
/* Y[M,N] = act(X[M,K] W[N,K]^T + bias (+ res)); same kernel as the 1x1 convolution. */
strait_status strait_k_gemm(void* stream, const void* x, const void* w, const float* bias, int32_t M,
                            int32_t N, int32_t K, int32_t act, const void* res, void* y, int32_t out_f32,
                            int32_t hp);
/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc): strait_k_gemm for products of at most 128 * 4096 outputs (M * N; E_SHAPE beyond -- larger products
 * use no workspace and strait_k_gemm allocates nothing for them), with the split-K workspace of 16 MiB taken from a
 * static device array instead of hipMalloc.  Same kernels, same results bit for bit.  Calls no allocating routine and
 * does not synchronise; the launch is asynchronous on `stream`, whose device must be the current one.  Every call on
 * a GPU shares that GPU's array (held until the process ends), so calls that overlap on one GPU race; calls ordered
 * by a stream or an event do not. */
strait_status strait_k_gemm_noalloc(void* stream, const void* x, const void* w, const float* bias, int32_t M,
                                    int32_t N, int32_t K, int32_t act, const void* res, void* y, int32_t out_f32,
                                    int32_t hp);
/* Two chained pointwise convolutions in one launch (Section 3.2 step (2): consecutive kernels of a batch's sequence):
 *     y[m, 0:N1] = act1(x[m, 0:K1] w3^T + b3 (+ res[m, 0:N1]));     z[m, 0:N2] = act2(y[m, 0:N1] w1^T + b1)
 * x [M][K1], w3 [N1][K1], res (or NULL) and y [M][N1], w1 [N2][N1], z [M][N2], dense fp16; b3 [N1], b1 [N2] fp32 or NULL;
 * act1/act2 NONE, RELU or RELU6.  res is required.  K1 = 64, N1 = 256, N2 in {64, 128}: the shapes whose two weight
 * matrices fit in a compute unit's LDS together (E_SHAPE otherwise).  y is
 * rounded to fp16 before it enters the second product, as if the two layers had run one after the other.  z must not
 * overlap x or res. */
strait_status strait_k_pointwise_pair(void* stream, const void* x, const void* w3, const float* b3, const void* res, void* y,
                                      const void* w1, const float* b1, void* z, int32_t M, int32_t K1, int32_t N1, int32_t N2,
                                      int32_t act1, int32_t act2, int32_t hp);
/* A block-closing 1x1 convolution that absorbs the block's 1x1 projection shortcut (Section 3.2 step (2): two members of
 * the kernel sequence as one): the projection, which may subsample its input, is a second source of the reduction,
 *     y[n,p,q,k] = act(bias[k] + sum_{c<C} x[n,p,q,c] w[k][c] + sum_{c<K2} x2[n, p*stride2, q*stride2, c] w[k][C + c])
 * x [N][P][Q][C], x2 [N][H2][W2][K2] with (P-1)*stride2 < H2 and (Q-1)*stride2 < W2, w [Cout][C + K2], y [N][P][Q][Cout], dense
 * fp16 device memory; bias fp32 [Cout] or NULL (the sum of the two layers' biases); act NONE, RELU or RELU6.  C and K2
 * multiples of 64, Cout of 8 (E_SHAPE otherwise).  The sum is rounded to fp16 once. */
strait_status strait_k_conv1x1_proj(void* stream, const void* x, int32_t N, int32_t P, int32_t Q, int32_t C, const void* x2,
                                    int32_t H2, int32_t W2, int32_t K2, int32_t stride2, const void* w, const float* bias,
                                    int32_t Cout, int32_t act, void* y, int32_t hp);
/* The same pair where the first block's shortcut is a 1x1 projection of a second tensor (the first block of a residual
 * stage; Section 3.2 step (2)): the projection joins the first product's reduction instead of being written out and read
 * back as a residual,
 *     y[m, 0:N1] = act1([x[m, 0:K1] | x2[m, 0:K2]] w3^T + b3);     z[m, 0:N2] = act2(y[m, 0:N1] w1^T + b1)
 * x [M][K1], x2 [M][K2], w3 [N1][K1 + K2] (the closing convolution's weights beside the projection's; b3 the sum of the
 * two biases), y [M][N1], w1 [N2][N1], z [M][N2], dense fp16 device memory.  K1 = K2 = 64, N1 = 256, N2 = 64 (E_SHAPE
 * otherwise); x2 NULL is E_INVALID.  The sum is rounded to fp16 once, where two launches round the projection first.
 * z must not overlap x or x2. */
strait_status strait_k_pointwise_pair_proj(void* stream, const void* x, const void* x2, const void* w3, const float* b3, void* y,
                                           const void* w1, const float* b1, void* z, int32_t M, int32_t K1, int32_t K2, int32_t N1,
                                           int32_t N2, int32_t act1, int32_t act2, int32_t hp);
/* Depthwise 3x3: y[n,p,q,c] = act(bias[c] + sum_{r,s} x[..,c] * w[r][s][c]); w fp16 [3][3][C]; C % 8 == 0. */
strait_status strait_k_dwconv3x3(void* stream, const void* x, int32_t N, int32_t H, int32_t W, int32_t C,
                                 const void* w_rsc, const float* bias, int32_t stride, int32_t act, void* y,
                                 int32_t hp);
/* The first two layers of an inverted residual block in one launch (Section 3.2 step (2): two members of MobileNetV2's
 * kernel sequence): a 1x1 convolution x [N,H,W,Cin] -> Chid channels, + b1, act1, and the depthwise 3x3 convolution of
 * stride 1 or 2 and padding 1 behind it, + bd, act2 -> y [N,P,Q,Chid] with P = (H-1)/stride+1, Q = (W-1)/stride+1.  The
 * expanded tensor exists only tile by tile in LDS.  w1 fp16 [Chid][Cin], wd_rsc fp16 [3][3][Chid], b1 and bd fp32 [Chid] or
 * NULL; activations NONE, RELU or RELU6.  Cin a multiple of 8 up to 160, Chid a multiple of 8 (E_SHAPE otherwise); all
 * pointers 16-byte aligned (E_INVALID).  Results are bit-identical to strait_k_conv2d followed by strait_k_dwconv3x3. */
strait_status strait_k_expand_dw(void* stream, const void* x, int32_t N, int32_t H, int32_t W, int32_t Cin, const void* w1,
                                 const float* b1, int32_t Chid, int32_t act1, const void* wd_rsc, const float* bd, int32_t stride,
                                 int32_t act2, void* y, int32_t hp);
/* MobileNetV2's stem in one launch that reads the image as it lies in memory (Section 3.2 step (2): the first kernel of that
 * network's sequence): 3x3 convolution, stride 2, pad 1, of x [N,H,W,3] to Kout channels, + bias, activation (NONE, RELU,
 * RELU6) -> y [N,P,Q,Kout] with P = (H-1)/2+1, Q = (W-1)/2+1.  W even; Kout 8, 16, 24 or 32 (E_SHAPE otherwise).
 * wf fp16 [32][48]: row k is three filter rows of 16 halfs, {0, w[k][r][0][c=0..2], w[k][r][1][0..2], w[k][r][2][0..2],
 * 0, 0, 0, 0, 0, 0} (w indexed [k][r][s][c]); rows from Kout on are zero.  bias fp32 [Kout] or NULL.  Finite inputs give the
 * sums of the definition; a non-finite pixel can reach a neighbouring window through a zero weight. */
strait_status strait_k_stem3x3s2(void* stream, const void* x, int32_t N, int32_t H, int32_t W, const void* wf, const float* bias,
                                 int32_t Kout, int32_t act, void* y, int32_t hp);
/* The same stem with 32 output channels and the stride-1 depthwise 3x3 convolution of MobileNetV2's first block behind it
 * (padding 1, wd_rsc fp16 [3][3][32], + bd fp32 [32] or NULL, act2) in one launch: y [N,P,Q,32]; the stem's output stays in
 * LDS.  wf, bias, act1 as for strait_k_stem3x3s2.  W even (E_SHAPE otherwise), pointers 16-byte aligned.  Results are
 * bit-identical to strait_k_stem3x3s2 followed by strait_k_dwconv3x3. */
strait_status strait_k_stem3x3s2_dw(void* stream, const void* x, int32_t N, int32_t H, int32_t W, const void* wf, const float* bias,
                                    int32_t act1, const void* wd_rsc, const float* bd, int32_t act2, void* y, int32_t hp);
/* ResNet stem in one launch: 7x7 convolution, stride 2, pad 3, of x [N,H,W,3] to 64 channels, + bias, ReLU, then 3x3
 * max pooling, stride 2, pad 1 -> y [N,P2,Q2,64] (P = (H-1)/2+1, P2 = (P-1)/2+1, likewise Q).  W even.
 * wf fp16 [64][176]: row k is 22 fragments of 8 halfs; fragment 3r + j holds halfs 8j..8j+7 of the 24-half window
 * of filter row r, {0, w[k][r][0][c=0..2], w[k][r][1][0..2], ..., w[k][r][6][0..2], 0, 0} (w indexed [k][r][s][c]);
 * the 22nd fragment is zero.  bias fp32 [64]. */
strait_status strait_k_stem_pool(void* stream, const void* x, int32_t N, int32_t H, int32_t W, const void* wf,
                                 const float* bias, void* y, int32_t hp);
/* Max pooling 2x2, stride 2, no padding; C % 8 == 0, H and W even. */
strait_status strait_k_maxpool2x2s2(void* stream, const void* x, int32_t N, int32_t H, int32_t W, int32_t C,
                                    void* y, int32_t hp);
/* Token assembly of a Vision Transformer: z[n][0] = cls + pos[0], z[n][1+t] = patch[n][t] + pos[1+t];
 * patch fp16 [N][T][D], cls fp32 [D], pos fp32 [T+1][D], z fp16 [N][T+1][D]; D % 8 == 0. */
strait_status strait_k_vit_tokens(void* stream, const void* patch, const float* cls, const float* pos, int32_t N,
                                  int32_t T, int32_t D, void* z, int32_t hp);
/* Max pooling 3x3, stride 2, pad 1 (padding never wins); C % 8 == 0. */
strait_status strait_k_maxpool3x3s2(void* stream, const void* x, int32_t N, int32_t H, int32_t W, int32_t C,
                                    void* y, int32_t hp);
/* Global average pooling [N,HW,C] -> fp16 [N,C], fp32 accumulation; C % 8 == 0. */
strait_status strait_k_global_avgpool(void* stream, const void* x, int32_t N, int32_t HW, int32_t C, void* y,
                                      int32_t hp);
/* Row softmax of fp32 logits [rows][n] -> fp32 probs, int32 top1 (argmax of the logits, lowest
 * index on ties). */
strait_status strait_k_softmax_top1(void* stream, const float* logits, int32_t rows, int32_t n, float* probs,
                                    int32_t* top1, int32_t hp);
/* LayerNorm over the last axis, biased variance, eps inside the square root:
 * y = (x - mean)/sqrt(var + eps) * gamma + beta; x,y fp16 [rows][n], gamma/beta fp32; n % 8 == 0, n <= 8192. */
strait_status strait_k_layernorm(void* stream, const void* x, const float* gamma, const float* beta,
                                 int32_t rows, int32_t n, float eps, void* y, int32_t hp);
/* Fused masked multi-head attention.  qkv fp16 [B][S][3*hidden] (Q | K | V along the last
 * axis), valid_len int32 [B] (device), out fp16 [B][S][hidden]; head dim must be 64,
 * 1 <= S <= 256.  Keys j >= valid_len[b] get probability exactly 0; query rows in 32-row
 * blocks that lie entirely at or beyond valid_len[b] are written as zeros. */
strait_status strait_k_attention(void* stream, const void* qkv, const int32_t* valid_len, int32_t B, int32_t S,
                                 int32_t heads, void* out, int32_t hp);
/* fp16 argmax over the first `n` features of row (b * row_stride) -> int32 top1[b]. */
strait_status strait_k_argmax_f16(void* stream, const void* x, int32_t rows, int32_t n, int64_t row_stride,
                                  int32_t* top1, int32_t hp);

/* ---- host-to-device link model (host only; no GPU needed) -----------------------------------
 * Section 3.2 of the paper, "Interference in data transfer": pinned transfers of concurrent
 * batches are served first-in first-out, so
 *     T_data = max(0, t_available - t_current)                        (Eq. 2)
 *     t_available <- max(t_current, t_available) + t_HtoD(i,j)        (Eq. 3)
 * and ("Online calibration") once a transfer has been timed, its measured end replaces the
 * estimate: Eq. 3 is then carried forward from the measured end over the transfers scheduled
 * after it.  All times are int64 nanoseconds on one clock of the caller's choice.  Thread-safe. */
typedef struct strait_link strait_link;
strait_status strait_link_create(strait_link** out);
strait_status strait_link_destroy(strait_link* link);
/* t_available as it stands (INT64_MIN before the first transfer). */
strait_status strait_link_available(const strait_link* link, int64_t* t_available_ns);
/* Eq. 2 for a batch that would be submitted at t_current. */
strait_status strait_link_predict(const strait_link* link, int64_t t_current_ns, int64_t* t_data_ns);
/* Eq. 2 (optional output) followed by Eq. 3 for a batch whose isolated transfer takes t_htod. */
strait_status strait_link_schedule(strait_link* link, int64_t t_current_ns, int64_t t_htod_ns,
                                   uint64_t* transfer_id, int64_t* t_data_ns);
/* Online calibration: transfer `transfer_id` was observed to end at t_end.  E_INVALID for an id
 * that is unknown or older than an already calibrated transfer. */
strait_status strait_link_complete(strait_link* link, uint64_t transfer_id, int64_t t_end_ns);

/* ---- kernel-interference predictor (host only; no GPU needed) -------------------------------
 * Section 3.2 of the paper, "Interference in kernel execution" and "Self-adaptive model":
 *     kernel_eff = k * b^LR(m_avg^1..n | m_self^cmp, m_self^mem) + C          (Eq. 4)
 *     Intf       = 1 + kernel_eff * coeff_p                                    (Eq. 5)
 *     T_kernel   = (Intf - 1) * T_kernel^isol                                  (Eq. 6)
 * LR is a weighted sum without intercept.  The STRAIT_INTF_METRICS co-located metrics are, in
 * order, the utilisation of: LDS/L1, L2, DRAM, matrix pipes, FMA pipes (fractions of peak);
 * m_self^cmp is the batch's own matrix-pipe and m_self^mem its own L2 utilisation.  A batch
 * whose m_avg is all zero (never had a neighbour) has Intf = 1 and does not train the model.
 * coeff_p is indexed by strait_priority.  All arithmetic is fp64.  Thread-safe. */
#define STRAIT_INTF_METRICS 5
typedef struct strait_intf_params {
    double k, b, C;
    double w_avg[STRAIT_INTF_METRICS];
    double w_self_cmp, w_self_mem;
    double coeff_p[2];
} strait_intf_params;
typedef struct strait_intf strait_intf;
/* init == NULL: conservative start (k 1, b 2, C -1, w_avg 0.5 each, w_self 0, coeff_p 1).
 * E_INVALID if init->b < 1e-6. */
strait_status strait_intf_create(const strait_intf_params* init, strait_intf** out);
strait_status strait_intf_destroy(strait_intf* p);
strait_status strait_intf_get_params(const strait_intf* p, strait_intf_params* out);
/* Resource demand of a batch: m_out[i] = sum_j v[j][i] d[j] / sum_j d[j] over its n kernels
 * (v row-major [n][STRAIT_INTF_METRICS], d >= 0 with a positive sum). */
strait_status strait_intf_demand(const double* v, const double* d, int32_t n, double* m_out);
/* Eq. 4-6 for one batch; either output may be NULL (not both). */
strait_status strait_intf_predict(const strait_intf* p, const double* m_avg, double m_self_cmp, double m_self_mem,
                                  int32_t priority, double t_kernel_isol, double* intf_hat, double* t_kernel);
/* One online step for a completed batch whose measured slowdown (kernel latency over the
 * profiled isolated latency) was intf_actual: Adam (beta1 0.7, beta2 0.9, alpha 0.0075, eps
 * 1e-8, bias-corrected) on the Huber loss (delta 0.5) of (predicted - actual); afterwards b is
 * kept >= 1e-6.  loss (optional) receives the loss before the step. */
strait_status strait_intf_update(strait_intf* p, const double* m_avg, double m_self_cmp, double m_self_mem,
                                 int32_t priority, double intf_actual, double* loss);
/* Co-location dynamics of one GPU.  arrive: a batch of demand m[STRAIT_INTF_METRICS] starts at
 * t; depart: it ends at t, m_avg_out receives the time-weighted average, over its life, of the
 * summed demands of the batches that ran beside it.  Times are int64 nanoseconds, never
 * decreasing across calls (E_INVALID otherwise, or for an unknown id). */
strait_status strait_intf_arrive(strait_intf* p, int64_t t_ns, const double* m, uint64_t* batch_id);
strait_status strait_intf_depart(strait_intf* p, uint64_t batch_id, int64_t t_ns, double* m_avg_out);
/* Summed demand of the batches running now, leaving out exclude_id (0 = none). */
strait_status strait_intf_pressure(const strait_intf* p, uint64_t exclude_id, double* m_now);

/* ---- scheduling policy (host only; no GPU needed) ---------------------------------------------
 * Section 3.3 of the paper, Algorithm 1, on top of Eq. 1:
 *     T_inf(B_ik) = T_inf_isol(B_ik) + T_data + T_kernel(B_ik) + T_queue
 * A strait_sched owns, per GPU, a link model (Eq. 2-3) and a co-location tracker, and one interference
 * predictor (Eq. 4-6).  strait_sched_decide serves one model's queue once: requests that could not
 * finish even in isolation are dropped; a binary search finds the largest batch size k that some GPU
 * can take with not violate() and meet(); among those GPUs the one of lowest estimated T_inf gets the
 * batch, which is logged as running there.  violate(): a low-priority batch may not lift the summed peak
 * throughput (largest demand metric) of the low-priority batches on the GPU above C_low, and no running
 * batch of equal or higher priority may be pushed past its deadline (completed fraction from the elapsed
 * kernel time under its time-weighted pressure so far, the rest under the pressure with the new batch
 * added).  meet(): the new batch meets its own deadline with T_kernel taken at half of the GPU's summed
 * demand.  C_low rises by 0.25 % per full 100 ms from 75 % to 100 % and returns to 75 % when a
 * high-priority batch misses its deadline.  Times are int64 nanoseconds on one clock, never decreasing
 * across calls.  Thread-safe. */
typedef struct strait_batch_profile {          /* offline profile of one (model, batch size)           */
    double t_inf_isol_ns;                      /* p95 isolated overall latency                         */
    int64_t t_htod_ns;                         /* p95 isolated host-to-device transfer time            */
    double t_kernel_isol_ns;                   /* p95 isolated kernel latency                          */
    double m[STRAIT_INTF_METRICS];             /* resource demand (strait_intf_demand)                 */
    double m_self_cmp, m_self_mem;
} strait_batch_profile;
typedef struct strait_decision {
    int32_t n_dropped;                         /* requests removed from the front of the queue         */
    int32_t batch;                             /* size of the batch to submit (the next `batch` requests), 0 = deferred */
    int32_t gpu;                               /* where; -1 when deferred                               */
    int32_t reserved;
    double t_inf_ns;                           /* Eq. 1 for the chosen batch and GPU                   */
    int64_t t_data_ns;                         /* its Eq. 2 term                                        */
    uint64_t running_id;                       /* handle for strait_sched_complete                     */
} strait_decision;
typedef struct strait_completion {
    int32_t violated;                          /* finished after its deadline                           */
    int32_t reserved;
    double loss;                               /* Huber loss of the predictor before its update        */
    double m_avg[STRAIT_INTF_METRICS];         /* time-weighted co-located demand it ran under         */
    double c_low;
} strait_completion;
typedef struct strait_sched strait_sched;
/* init == NULL: the conservative predictor start of strait_intf_create. */
strait_status strait_sched_create(int32_t n_gpus, const strait_intf_params* init, strait_sched** out);
strait_status strait_sched_destroy(strait_sched* s);
/* table[b-1] is the profile of batch size b, b = 1..max_batch; E_BUSY while batches of the model run. */
strait_status strait_sched_set_profile(strait_sched* s, int32_t model_id, int32_t priority,
                                       const strait_batch_profile* table, int32_t max_batch);
/* Advance the AIMD clock; c_low (optional) receives the cap. */
strait_status strait_sched_tick(strait_sched* s, int64_t now_ns, double* c_low);
/* enqueue_ns / deadline_ns: the buffered requests of the model, oldest first. */
strait_status strait_sched_decide(strait_sched* s, int32_t model_id, int64_t now_ns, const int64_t* enqueue_ns,
                                  const int64_t* deadline_ns, int32_t n_requests, strait_decision* out);
/* The batch finished at now_ns with measured kernel latency kernel_ns; h2d_end_ns >= 0 calibrates the
 * link with the measured end of its transfer.  Removes it from the running list, updates the predictor
 * (Section 3.2, "Self-adaptive model") and the cap.  out may be NULL. */
strait_status strait_sched_complete(strait_sched* s, int32_t gpu, uint64_t running_id, int64_t now_ns,
                                    double kernel_ns, int64_t h2d_end_ns, strait_completion* out);
strait_status strait_sched_get_params(strait_sched* s, strait_intf_params* out);

/* ---- offline profile of one (model, batch size) (needs the GPU) --------------------------------
 * Section 3.2: the scheduler works from profiled p95 isolated latencies and from a batch's resource
 * demand, the time-weighted average throughput of its kernels.  Runs `reps` (>= 1) batches of size `batch`
 * alone on the GPU through strait_submit (the model must be otherwise idle) and fills `out`: nearest-rank
 * p95 of enqueue-to-result latency, of the input copy and of the kernel sequence; the demand vector
 * [LDS, L2, HBM, matrix pipes, vector pipes] as fractions of the chip's peaks, from the layer accounting
 * (strait_model_layer) over the p95 kernel time: HBM = activation + weight bytes against 8 TB/s; matrix =
 * 2 x MACs of the MFMA layers against 2.5 PFLOP/s; vector = depthwise MACs x 2 plus one operation per
 * element of the other layers against 157.3 TFLOP/s; L2 = operand bytes of a 128 x 128-tiled product (each
 * operand re-read once per tile row / column) plus the other layers' bytes against 64 B/clock/CU; LDS =
 * three times the MFMA layers' operand bytes (written once, read by two waves) against 128 B/clock/CU.
 * m_self_cmp is the matrix entry and m_self_mem the L2 entry (the two the paper selects). */
strait_status strait_model_profile(strait_model* m, strait_priority prio, int32_t batch, int32_t reps,
                                   strait_batch_profile* out);

/* ---- serving front end ---------------------------------------------------------------------------
 * Section 3 (system workflow), Section 4 and Section 5.1 of the paper.  A request enters the task queue
 * of its model.  A queue asks for a decision once it holds max_batch requests or its oldest request has
 * waited the model's batch formation timeout.  One scheduling thread visits the queues that ask, high
 * priority first and first come first served within a level, and takes one decision per visit
 * (strait_sched_decide): the requests the decision drops leave as violations, the chosen ones are gathered
 * into the pinned buffer of a free instance and submitted as one batch on the stream of the model's
 * priority; a queue whose batch is deferred (no capacity, no free instance, or the concurrency limit
 * reached) is visited again after the next completion, the next arrival or `retry_ns`.  Execution threads
 * wait for the batches, give every request its slice of the output and feed the measured kernel latency
 * and transfer time back (strait_sched_complete).  A request's latency runs from strait_server_request to
 * its result being in host memory; a dropped request counts as a deadline violation.
 * The scheduler given to a server must have been created for one GPU and have the profile of every
 * model added here; the server must be the only user of these models while it runs. */
typedef struct strait_server strait_server;
typedef struct strait_server_model {
    strait_model* model;                       /* NULL only with a caller-supplied executor             */
    int32_t model_id;                          /* the id its profile table is registered under          */
    int32_t priority;                          /* strait_priority                                       */
    int32_t max_batch;                         /* Section 5.1 uses 8                                    */
    int32_t n_instances;                       /* batches of this model in flight at once; 0 = the model's instances */
    int64_t deadline_ns;                       /* relative deadline of every request                    */
    int64_t formation_timeout_ns;              /* how long the oldest request waits for company         */
} strait_server_model;
/* What runs a batch when it is not the library itself (host-side tests, simulations).  submit starts batch
 * `batch_seq` and returns at once; wait blocks until it is complete and reports the measured kernel latency
 * and input transfer time in ns.  Both are called from the server's threads; nonzero return = failure. */
typedef struct strait_executor {
    void* user;
    int32_t (*submit)(void* user, uint64_t batch_seq, int32_t model_id, int32_t priority, int32_t batch,
                      const void* const* inputs, void* const* outputs, const int32_t* valid_len);
    int32_t (*wait)(void* user, uint64_t batch_seq, double* kernel_ns, double* h2d_ns);
} strait_executor;
typedef struct strait_request_record {
    uint64_t request_id;
    uint64_t batch_seq;                        /* running number of the batch it rode in, 0 if none    */
    int32_t model_id, priority;
    int32_t status;                            /* 0 served, 1 dropped early, 2 executor failure, 3 still queued at stop */
    int32_t batch;                             /* size of that batch                                   */
    int32_t position;                          /* its index in the batch (arrival order)               */
    int32_t violated;                          /* result later than the deadline, or no result         */
    int64_t t_enqueue_ns, t_dispatch_ns, t_done_ns, deadline_ns;   /* host CLOCK_MONOTONIC; deadline absolute */
    double t_inf_pred_ns;                      /* Eq. 1 estimate at dispatch                            */
    double kernel_ns, h2d_ns;                  /* measured, of its batch                                */
} strait_request_record;
typedef struct strait_server_stats {
    int64_t requests, served, dropped, failed, violated_high, violated_low, requests_high, requests_low;
    int64_t batches, batched_requests, deferrals, max_in_flight;
} strait_server_stats;
/* concurrency: batches in flight at most (Section 5.1 uses 4); retry_ns > 0; executor NULL = the library. */
strait_status strait_server_create(strait_sched* sched, int32_t concurrency, int64_t retry_ns,
                                   const strait_executor* executor, strait_server** out);
strait_status strait_server_add_model(strait_server* s, const strait_server_model* desc);   /* before start */
/* With the library's own executor, start first runs every (instance, batch size) of every model twice and one
 * burst of `concurrency` batches, so that no request pays for a first use (graph capture, runtime pools). */
strait_status strait_server_start(strait_server* s);
/* Non-blocking, thread-safe.  host_in (one sample, the model's input layout) and host_out (one sample's
 * output, the layout of strait_model_io at batch 1) must stay valid until the request's record has been
 * produced.  valid_len: encoder only.  E_INVALID before start or after stop. */
strait_status strait_server_request(strait_server* s, int32_t model_id, const void* host_in, int32_t valid_len,
                                    void* host_out, uint64_t* request_id);
/* Blocks until every queue is empty and no batch is in flight (E_BUSY after timeout_ns). */
strait_status strait_server_wait_idle(strait_server* s, int64_t timeout_ns);
/* Moves up to `capacity` finished records (oldest first) to `out`; *n = how many. */
strait_status strait_server_results(strait_server* s, strait_request_record* out, int32_t capacity, int32_t* n);
strait_status strait_server_get_stats(strait_server* s, strait_server_stats* out);
/* Stops taking requests, lets the batches in flight finish, reports what is still queued with status 3. */
strait_status strait_server_stop(strait_server* s);
strait_status strait_server_destroy(strait_server* s);   /* stops first if needed */

#ifdef __cplusplus
}
#endif
#endif /* STRAIT_H */
