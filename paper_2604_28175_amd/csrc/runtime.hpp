// Host-side runtime: weight container, BatchNorm fold and re-layout, per-architecture layer
// plans, model instances with pinned staging, dual-priority dispatch and completion records.
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>
#include <condition_variable>
#include <deque>
#include <map>
#include <mutex>
#include <set>
#include <string>
#include <thread>
#include <vector>

#include "../../include/strait.h"
#include "kernels.hpp"

namespace strait {

enum OpKind { OP_CONV = 0, OP_DWCONV = 1, OP_POOL = 2, OP_SOFTMAX = 3, OP_LAYERNORM = 4, OP_ATTENTION = 5, OP_PACK = 6, OP_TOKENS = 7, OP_STEMPOOL = 8, OP_STEM3 = 9 };
enum PoolKind { POOL_MAX3X3S2 = 0, POOL_GLOBAL_AVG = 1, POOL_ARGMAX = 2, POOL_MAX2X2S2 = 3 };

// Where an operand lives.  Slots >= 0 index the instance's activation buffers; the input and
// output slots are the instance's device input / output buffers (output at a byte offset that
// depends on the batch size).
enum { SLOT_NONE = -1, SLOT_INPUT = -2, SLOT_OUT = -3 };

struct OutRef { int kind = 0; };   // 0: start of output buffer, 1: after logits (probs), 2: after logits+probs (top1), 3: after hidden states

struct Op {
    std::string name;
    int kind = OP_CONV;
    int sub = 0;                      // PoolKind for OP_POOL
    int in = SLOT_NONE, out = SLOT_NONE, res = SLOT_NONE;
    int out_ref = 0, out_ref2 = 0;    // which region of the output buffer (when out == SLOT_OUT)
    // geometry per sample
    int H = 1, W = 1, C = 1;          // input
    int P = 1, Q = 1, K = 1;          // output
    int R = 1, S = 1, stride = 1, pad = 0, act = 0;
    int out_f32 = 0;
    // Independent branch: `side` ops run on the instance's side stream, forked off the main stream right
    // before them; the first later op with `join` set waits for the side stream before it is launched.
    int side = 0, join = 0;
    // A block-closing pointwise convolution whose output feeds the pointwise convolution `pair` ops further on (0 = none):
    // at large batches the two run as one launch (pointwise_pair.hip) and the second op is skipped.
    int pair = 0;
    // Such a pair in a block whose shortcut is a 1x1 projection of the block input with the block's own stride 1: the
    // projection can join the closing convolution's reduction (w_proj = [w | projection's w], bias_proj = the two biases
    // added), and the projection's own launch is skipped.  proj_down: on the closing convolution, the index of the
    // projection op; proj_of: on the projection op, the index of the closing convolution (-1 = none).
    int proj_down = -1, proj_of = -1;
    // on the fused stem: the index of the 1x1 convolution (64 -> 64, ReLU) that reads nothing but its output and can run inside it
    int stem_next = -1;
    // on a 1x1 expansion or the 3x3/2 stem: the next op is the depthwise 3x3 that alone reads its output, and both can run as one launch
    bool dw_next = false;
    const half_t* w_proj = nullptr;
    const float* bias_proj = nullptr;
    // implicit-GEMM addressing (elements), see ConvParams
    long long sN = 0; int sH = 0, sW = 0, stride_w = 1, pad_h = 0, pad_w = 0, vC = 0, vR = 0, vS = 0, vH = 0, vW = 0;
    int ldw = 0;
    // pack
    int Hp = 0, Wp = 0, Cpad = 0;
    // attention / layernorm
    int seq = 0, heads = 0;
    float eps = 0.f;
    long long in_row_stride = 0;      // LayerNorm: elements between input rows (0 = contiguous)
    const half_t* w = nullptr;
    const float* bias = nullptr;      // conv/gemm bias, LayerNorm gamma, class token (OP_TOKENS)
    const float* beta = nullptr;      // LayerNorm beta, position embeddings (OP_TOKENS)
    strait_layer_info info{};
};

struct Instance {
    void* pinned_in = nullptr;
    void* pinned_in_dev = nullptr;     // the same memory as the GPU addresses it
    void* pinned_out = nullptr;
    void* pinned_out_dev = nullptr;    // the same memory as the GPU addresses it
    void* dev_in = nullptr;
    void* dev_out = nullptr;
    int32_t* dev_valid = nullptr;
    float* splitk_ws = nullptr;        // fp32 slabs of split-K convolutions (small batches)
    std::vector<void*> bufs;
    hipEvent_t ev_h2d0 = nullptr, ev_h2d1 = nullptr, ev_k0 = nullptr, ev_k1 = nullptr, ev_done = nullptr;
    hipEvent_t ev_seg[2] = {nullptr, nullptr};   // ends of the two plan segments a yielding low-priority batch has in flight
    hipStream_t side = nullptr;        // default priority, non-blocking: carries branches that do not depend on each other
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    std::vector<hipEvent_t> layer_ev;
    std::vector<char> layer_skipped;    // by the last timed run: layers that were computed inside another layer's launch
    // Captured kernel sequences, keyed by (batch, wave-priority flag); a key is captured on its second
    // use, after one eager pass has set the kernels' attributes outside of any capture.
    std::map<std::pair<int, int>, hipGraphExec_t> graphs;
    std::set<std::pair<int, int>> warmed;
    bool busy = false;
};

constexpr size_t SPLITK_WS_BYTES = 16u << 20;

struct Context;

struct Model {
    Context* ctx = nullptr;
    int id = 0;
    int arch = 0;
    int hyper[8] = {0};
    int max_batch = 0;
    std::vector<Op> ops;
    std::vector<size_t> buf_elems;     // per-sample elements of each activation buffer
    size_t in_elems = 0;               // per-sample fp16 input elements
    int classes = 0;                   // CNN
    int seq = 0, hidden = 0;           // encoder
    std::vector<void*> dev_allocs;     // weights
    std::vector<Instance> inst;
    std::mutex mu;
    int in_flight = 0;

    size_t in_bytes(int b) const { return (size_t)b * in_elems * 2; }
    size_t out_bytes(int b) const;
    size_t out_offset(int ref, int b) const;
};

struct Ticket {
    Model* model = nullptr;
    int instance = 0, prio = 0, batch = 0;
    void* host_out = nullptr;
    strait_record rec{};
    bool done = false;
    int status = 0;
    bool deferred = false;             // kernels not enqueued yet: the stream's worker issues them segment by segment
    int hp = 0;                        // wave-priority flag its kernels are launched with
};

struct StreamWorker {
    hipStream_t stream = nullptr;
    std::thread th;
    std::deque<Ticket*> q;
};

struct Context {
    int device = 0;
    std::vector<hipStream_t> hp, lp, copy;
    std::vector<StreamWorker*> workers;     // one per compute stream: hp first, then lp
    // A batch's operations on a stream (event, copy, event / event, kernels, event, copy, event) are enqueued
    // under that stream's mutex, so that batches submitted from several threads do not interleave on it and
    // every record times its own batch only.
    std::deque<std::mutex> compute_mu, copy_mu;
    std::mutex mu;                          // guards worker queues, ticket completion, counters
    std::condition_variable cv_work, cv_done;
    bool stop = false;
    bool wave_priority = true;
    bool use_graphs = false;
    long long proj_min_pixels = 1;          // the same for pairs that absorb a projection shortcut: three launches become one
    long long pair_min_pixels = 40000;      // from this many output pixels on, marked pairs of pointwise convolutions run as one launch (0 = never)
    int lp_yield_layers = 0;                // > 0: low-priority batches are issued in segments of this many layers and yield between them
    std::atomic<int> hp_in_flight{0};       // high-priority batches submitted and not yet complete
    bool branch_streams = true;             // independent branches of a plan go to the instance's side stream
    size_t h2d_kernel_limit = 8u << 20;   // inputs up to this size go in by a copy kernel, larger ones by hipMemcpyAsync
    unsigned n_hp_sub = 0, n_lp_sub = 0, n_copy_sub = 0;
    int n_models = 0, next_model_id = 0;
};

int build_plan(Model& m, const void* blob, size_t bytes);
// Enqueues layers first_layer..last_layer (last_layer < 0: up to the end) of the plan for `batch` samples on `stream`.
int run_plan(Model& m, Instance& in, int batch, hipStream_t stream, int hp, int last_layer, bool timed, int first_layer = 0);

}  // namespace strait
