// C ABI (strait.h): contexts, model instances, dual-priority submission, completion records.
//
// A submitted batch follows the paper's three steps (Section 3.2): input into the instance's
// pinned buffer and an asynchronous host-to-device copy on a copy stream; the kernel sequence
// on the compute stream that belongs to the batch's priority level (Section 3.1), made to wait
// for the copy through an event; the device-to-host copy of the result into pinned memory.
// Nothing synchronises with the host in between.  One completion thread per compute stream
// waits for batches in issue order, stamps the host completion time (Section 5.1: latency ends
// when the result is back in host memory), reads the event timings that Strait's predictor
// would be fed (measured H2D time, measured kernel latency) and hands the result over.
#include <time.h>

#include <cstdio>
#include <cstring>
#include <new>

#include "runtime.hpp"

namespace strait {
const char* last_error();
}
using namespace strait;

#define HIP_TRY(expr)                                                                   \
    do {                                                                                \
        hipError_t e_ = (expr);                                                         \
        if (e_ != hipSuccess) { set_error("%s: %s", #expr, hipGetErrorString(e_)); return STRAIT_E_HIP; } \
    } while (0)

struct strait_ctx : Context {};
struct strait_model : Model {};
struct strait_ticket_s : Ticket {};

static int64_t now_ns() {
    timespec ts;
    clock_gettime(CLOCK_MONOTONIC, &ts);
    return (int64_t)ts.tv_sec * 1000000000LL + ts.tv_nsec;
}

// A yielding low-priority batch (strait_ctx_set_lp_yield): its kernel sequence is enqueued by the stream's worker thread
// in segments of a few layers, at most two segments in flight, and before each further segment the thread waits while a
// high-priority batch is in flight on the GPU (at most kMaxYieldNs per segment, so that the wait always ends).  What
// the GPU runs beside a high-priority batch is then at most the rest of two short segments instead of a whole batch.
static const int64_t kMaxYieldNs = 5000000;
static int issue_in_segments(Context* ctx, StreamWorker* w, Ticket* t) {
    Model& m = *t->model;
    Instance& in = m.inst[t->instance];
    hipStream_t s = w->stream;
    const int n = (int)m.ops.size();
    int seg;
    { std::lock_guard<std::mutex> lk(ctx->mu); seg = ctx->lp_yield_layers > 0 ? ctx->lp_yield_layers : n; }
    if (hipStreamWaitEvent(s, in.ev_h2d1, 0) != hipSuccess || hipEventRecord(in.ev_k0, s) != hipSuccess) return STRAIT_E_HIP;
    int k = 0;
    for (int first = 0; first < n; first += seg, ++k) {
        if (k >= 1) {
            const int64_t t0 = now_ns();
            while (ctx->hp_in_flight.load(std::memory_order_acquire) > 0 && now_ns() - t0 < kMaxYieldNs) {
                timespec ts{0, 20000};
                nanosleep(&ts, nullptr);
            }
        }
        const int last = first + seg - 1 < n - 1 ? first + seg - 1 : n - 1;
        if (run_plan(m, in, t->batch, s, t->hp, last, false, first)) return STRAIT_E_HIP;
        if (hipEventRecord(in.ev_seg[k & 1], s) != hipSuccess) return STRAIT_E_HIP;
        if (k >= 1 && hipEventSynchronize(in.ev_seg[(k - 1) & 1]) != hipSuccess) return STRAIT_E_HIP;   // one segment of look-ahead
    }
    if (hipEventRecord(in.ev_k1, s) != hipSuccess) return STRAIT_E_HIP;
    if (launch_copy_mapped(in.dev_out, in.pinned_out_dev, m.out_bytes(t->batch), t->hp, s)) return STRAIT_E_HIP;
    if (hipEventRecord(in.ev_done, s) != hipSuccess) return STRAIT_E_HIP;
    return 0;
}

static void worker_loop(Context* ctx, StreamWorker* w) {
    (void)hipSetDevice(ctx->device);
    for (;;) {
        Ticket* t = nullptr;
        {
            std::unique_lock<std::mutex> lk(ctx->mu);
            ctx->cv_work.wait(lk, [&] { return ctx->stop || !w->q.empty(); });
            if (w->q.empty()) return;           // stop requested and nothing left
            t = w->q.front();
            w->q.pop_front();
        }
        Instance& in = t->model->inst[t->instance];
        int status = 0;
        if (t->deferred) status = issue_in_segments(ctx, w, t);
        hipError_t e = status ? hipSuccess : hipEventSynchronize(in.ev_done);
        const int64_t done = now_ns();
        if (t->prio == STRAIT_PRIO_HIGH) ctx->hp_in_flight.fetch_sub(1, std::memory_order_acq_rel);
        if (e != hipSuccess) status = STRAIT_E_HIP;
        else if (!status) {
            memcpy(t->host_out, in.pinned_out, t->model->out_bytes(t->batch));
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, in.ev_h2d0, in.ev_h2d1) == hipSuccess) t->rec.h2d_ms = ms;
            if (hipEventElapsedTime(&ms, in.ev_k0, in.ev_k1) == hipSuccess) t->rec.kernel_ms = ms;
            if (hipEventElapsedTime(&ms, in.ev_k1, in.ev_done) == hipSuccess) t->rec.d2h_ms = ms;
            if (hipEventElapsedTime(&ms, in.ev_h2d0, in.ev_done) == hipSuccess) t->rec.total_ms = ms;
        }
        {
            std::lock_guard<std::mutex> lk(ctx->mu);
            t->rec.t_done_ns = done;
            t->status = status;
            t->done = true;
        }
        ctx->cv_done.notify_all();
    }
}

extern "C" {

const char* strait_last_error(void) { return strait::last_error(); }
int32_t strait_version(void) { return 1; }

strait_status strait_ctx_create(const strait_ctx_desc* d, strait_ctx** out) {
    if (!d || !out) { set_error("ctx_create: null argument"); return STRAIT_E_INVALID; }
    if (d->n_hp < 1 || d->n_lp < 1 || d->n_copy < 1 || d->n_hp > STRAIT_MAX_STREAMS || d->n_lp > STRAIT_MAX_STREAMS ||
        d->n_copy > STRAIT_MAX_STREAMS) { set_error("ctx_create: stream counts must be in 1..%d", STRAIT_MAX_STREAMS); return STRAIT_E_INVALID; }
    int ndev = 0;
    HIP_TRY(hipGetDeviceCount(&ndev));
    if (d->device < 0 || d->device >= ndev) { set_error("ctx_create: device %d not present (%d devices)", d->device, ndev); return STRAIT_E_INVALID; }
    HIP_TRY(hipSetDevice(d->device));
    strait_ctx* c = new (std::nothrow) strait_ctx();
    if (!c) { set_error("out of host memory"); return STRAIT_E_NOMEM; }
    c->device = d->device;
    for (int i = 0; i < d->n_hp; ++i) c->hp.push_back((hipStream_t)d->hp_streams[i]);
    for (int i = 0; i < d->n_lp; ++i) c->lp.push_back((hipStream_t)d->lp_streams[i]);
    for (int i = 0; i < d->n_copy; ++i) c->copy.push_back((hipStream_t)d->copy_streams[i]);
    for (size_t i = 0; i < c->hp.size() + c->lp.size(); ++i) {
        StreamWorker* w = new StreamWorker();
        w->stream = i < c->hp.size() ? c->hp[i] : c->lp[i - c->hp.size()];
        c->workers.push_back(w);
    }
    c->compute_mu.resize(c->workers.size());
    c->copy_mu.resize(c->copy.size());
    for (StreamWorker* w : c->workers) w->th = std::thread(worker_loop, (Context*)c, w);
    *out = c;
    return STRAIT_OK;
}

strait_status strait_ctx_destroy(strait_ctx* c) {
    if (!c) { set_error("ctx_destroy: null"); return STRAIT_E_INVALID; }
    {
        std::lock_guard<std::mutex> lk(c->mu);
        if (c->n_models > 0) { set_error("ctx_destroy: %d models still loaded", c->n_models); return STRAIT_E_BUSY; }
        c->stop = true;
    }
    c->cv_work.notify_all();
    for (StreamWorker* w : c->workers) { if (w->th.joinable()) w->th.join(); delete w; }
    delete c;
    return STRAIT_OK;
}

strait_status strait_ctx_set_wave_priority(strait_ctx* c, int32_t enabled) {
    if (!c) { set_error("ctx_set_wave_priority: null"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(c->mu);
    c->wave_priority = enabled != 0;
    return STRAIT_OK;
}

strait_status strait_ctx_set_graphs(strait_ctx* c, int32_t enabled) {
    if (!c) { set_error("ctx_set_graphs: null"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(c->mu);
    c->use_graphs = enabled != 0;
    return STRAIT_OK;
}

strait_status strait_ctx_set_h2d_kernel_limit(strait_ctx* c, int64_t max_bytes) {
    if (!c || max_bytes < 0) { set_error("ctx_set_h2d_kernel_limit: null context or negative size"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(c->mu);
    c->h2d_kernel_limit = (size_t)max_bytes;
    return STRAIT_OK;
}

strait_status strait_ctx_set_pair_fusion(strait_ctx* c, int64_t min_pixels) {
    if (!c || min_pixels < 0) { set_error("ctx_set_pair_fusion: null context or negative size"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(c->mu);
    c->pair_min_pixels = min_pixels;
    return STRAIT_OK;
}

strait_status strait_ctx_set_proj_fusion(strait_ctx* c, int64_t min_pixels) {
    if (!c || min_pixels < 0) { set_error("ctx_set_proj_fusion: null context or negative size"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(c->mu);
    c->proj_min_pixels = min_pixels;
    return STRAIT_OK;
}

strait_status strait_ctx_set_lp_yield(strait_ctx* c, int32_t layers_per_segment) {
    if (!c || layers_per_segment < 0) { set_error("ctx_set_lp_yield: null context or negative segment length"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(c->mu);
    c->lp_yield_layers = layers_per_segment;
    return STRAIT_OK;
}

strait_status strait_ctx_set_branch_streams(strait_ctx* c, int32_t enabled) {
    if (!c) { set_error("ctx_set_branch_streams: null"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(c->mu);
    c->branch_streams = enabled != 0;
    return STRAIT_OK;
}

static int hp_flag(const Context* c, int prio) { return prio == STRAIT_PRIO_HIGH && c->wave_priority; }

// The kernel sequence of one batch on `s`: launched kernel by kernel, or, when the context asks for
// graphs, as one replay of the sequence captured for this (instance, batch, wave-priority) key.
// Only kernel launches are captured (no copies, events or memsets).
static int run_batch(Model& m, Instance& in, int batch, hipStream_t s, int hp) {
    if (!m.ctx->use_graphs) return run_plan(m, in, batch, s, hp, -1, false);
    const std::pair<int, int> key(batch, hp);
    auto it = in.graphs.find(key);
    if (it == in.graphs.end()) {
        if (in.warmed.insert(key).second) return run_plan(m, in, batch, s, hp, -1, false);
        hipGraph_t g = nullptr;
        HIP_TRY(hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal));
        const int rc = run_plan(m, in, batch, s, hp, -1, false);
        const hipError_t e = hipStreamEndCapture(s, &g);
        if (rc || e != hipSuccess) {
            if (g) (void)hipGraphDestroy(g);
            if (!rc) set_error("graph capture failed: %s", hipGetErrorString(e));
            return rc ? rc : STRAIT_E_HIP;
        }
        hipGraphExec_t ex = nullptr;
        const hipError_t ei = hipGraphInstantiate(&ex, g, nullptr, nullptr, 0);
        (void)hipGraphDestroy(g);
        if (ei != hipSuccess) { set_error("graph instantiate failed: %s", hipGetErrorString(ei)); return STRAIT_E_HIP; }
        it = in.graphs.emplace(key, ex).first;
    }
    HIP_TRY(hipGraphLaunch(it->second, s));
    return 0;
}

static void free_instance(Instance& in) {
    if (in.pinned_in) (void)hipHostFree(in.pinned_in);
    if (in.pinned_out) (void)hipHostFree(in.pinned_out);
    if (in.dev_in) (void)hipFree(in.dev_in);
    if (in.dev_out) (void)hipFree(in.dev_out);
    if (in.dev_valid) (void)hipFree(in.dev_valid);
    if (in.splitk_ws) (void)hipFree(in.splitk_ws);
    for (void* b : in.bufs) if (b) (void)hipFree(b);
    if (in.side) { (void)hipStreamSynchronize(in.side); (void)hipStreamDestroy(in.side); }
    hipEvent_t evs[9] = {in.ev_h2d0, in.ev_h2d1, in.ev_k0, in.ev_k1, in.ev_done, in.ev_fork, in.ev_join, in.ev_seg[0], in.ev_seg[1]};
    for (hipEvent_t e : evs) if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : in.layer_ev) if (e) (void)hipEventDestroy(e);
    for (auto& kv : in.graphs) (void)hipGraphExecDestroy(kv.second);
    in = Instance();
}

static void free_model(strait_model* m) {
    for (Instance& in : m->inst) free_instance(in);
    for (void* d : m->dev_allocs) (void)hipFree(d);
    delete m;
}

strait_status strait_model_load(strait_ctx* c, const strait_model_desc* d, strait_model** out) {
    if (!c || !d || !out || !d->weights) { set_error("model_load: null argument"); return STRAIT_E_INVALID; }
    if (d->max_batch < 1 || d->max_batch > 4096 || d->n_instances < 1 || d->n_instances > 64) {
        set_error("model_load: max_batch must be in 1..4096 and n_instances in 1..64"); return STRAIT_E_INVALID;
    }
    HIP_TRY(hipSetDevice(c->device));
    strait_model* m = new (std::nothrow) strait_model();
    if (!m) { set_error("out of host memory"); return STRAIT_E_NOMEM; }
    m->ctx = c;
    m->max_batch = d->max_batch;
    int rc = build_plan(*m, d->weights, d->weights_bytes);
    if (rc) { free_model(m); return rc; }
    m->inst.resize(d->n_instances);
    const size_t inb = (m->in_bytes(d->max_batch) + 255) / 256 * 256, outb = (m->out_bytes(d->max_batch) + 255) / 256 * 256;
    for (Instance& in : m->inst) {
        bool ok = hipHostMalloc(&in.pinned_in, inb + (size_t)d->max_batch * 4, hipHostMallocDefault) == hipSuccess &&
                  hipHostMalloc(&in.pinned_out, outb, hipHostMallocDefault) == hipSuccess &&
                  hipHostGetDevicePointer(&in.pinned_in_dev, in.pinned_in, 0) == hipSuccess &&
                  hipHostGetDevicePointer(&in.pinned_out_dev, in.pinned_out, 0) == hipSuccess &&
                  hipMalloc(&in.dev_in, inb) == hipSuccess && hipMalloc(&in.dev_out, outb) == hipSuccess &&
                  hipMalloc((void**)&in.dev_valid, (size_t)d->max_batch * 4 + 256) == hipSuccess &&
                  hipMalloc((void**)&in.splitk_ws, SPLITK_WS_BYTES) == hipSuccess;
        for (size_t i = 0; ok && i < m->buf_elems.size(); ++i) {
            void* b = nullptr;
            const size_t bytes = (m->buf_elems[i] * 2 * (size_t)d->max_batch + 255) / 256 * 256;
            ok = hipMalloc(&b, bytes) == hipSuccess;
            in.bufs.push_back(b);
        }
        ok = ok && hipEventCreate(&in.ev_h2d0) == hipSuccess && hipEventCreate(&in.ev_h2d1) == hipSuccess &&
             hipEventCreate(&in.ev_k0) == hipSuccess && hipEventCreate(&in.ev_k1) == hipSuccess &&
             hipEventCreate(&in.ev_done) == hipSuccess &&
             hipEventCreateWithFlags(&in.ev_seg[0], hipEventDisableTiming) == hipSuccess &&
             hipEventCreateWithFlags(&in.ev_seg[1], hipEventDisableTiming) == hipSuccess &&
             hipStreamCreateWithFlags(&in.side, hipStreamNonBlocking) == hipSuccess &&      // default priority
             hipEventCreateWithFlags(&in.ev_fork, hipEventDisableTiming) == hipSuccess &&
             hipEventCreateWithFlags(&in.ev_join, hipEventDisableTiming) == hipSuccess;
        if (ok) {
            in.layer_ev.resize(m->ops.size() + 1, nullptr);
            for (hipEvent_t& e : in.layer_ev) ok = ok && hipEventCreate(&e) == hipSuccess;
        }
        if (!ok) {
            (void)hipGetLastError();
            set_error("model_load: allocating an instance (%zu B in, %zu B out, %zu activation buffers) failed", inb, outb, m->buf_elems.size());
            free_model(m);
            return STRAIT_E_NOMEM;
        }
        // The runtime sets a stream's hardware queue up at the first launch on it, which takes milliseconds:
        // do that here and not under the first batch that happens to use this instance's side stream.
        if (launch_fill_zero(in.splitk_ws, 256, in.side) != 0) { free_model(m); return STRAIT_E_HIP; }
        // valid lengths default to the full sequence
        if (m->arch == STRAIT_ARCH_ENCODER || m->arch == STRAIT_ARCH_VIT) {
            std::vector<int32_t> full(d->max_batch, m->seq);
            HIP_TRY(hipMemcpy(in.dev_valid, full.data(), full.size() * 4, hipMemcpyHostToDevice));
        }
    }
    HIP_TRY(hipDeviceSynchronize());
    {
        std::lock_guard<std::mutex> lk(c->mu);
        m->id = c->next_model_id++;
        c->n_models++;
    }
    *out = m;
    return STRAIT_OK;
}

strait_status strait_model_free(strait_model* m) {
    if (!m) { set_error("model_free: null"); return STRAIT_E_INVALID; }
    {
        std::lock_guard<std::mutex> lk(m->mu);
        if (m->in_flight > 0) { set_error("model_free: %d batches in flight", m->in_flight); return STRAIT_E_BUSY; }
    }
    Context* c = m->ctx;
    (void)hipSetDevice(c->device);
    (void)hipDeviceSynchronize();
    free_model(m);
    std::lock_guard<std::mutex> lk(c->mu);
    c->n_models--;
    return STRAIT_OK;
}

strait_status strait_model_io(const strait_model* m, int32_t batch, size_t* in_bytes, size_t* out_bytes) {
    if (!m) { set_error("model_io: null"); return STRAIT_E_INVALID; }
    if (batch < 1 || batch > m->max_batch) { set_error("batch %d outside 1..%d", batch, m->max_batch); return STRAIT_E_BATCH; }
    if (in_bytes) *in_bytes = m->in_bytes(batch);
    if (out_bytes) *out_bytes = m->out_bytes(batch);
    return STRAIT_OK;
}

strait_status strait_model_info(const strait_model* m, int32_t* arch, int32_t* n_layers, int32_t* max_batch,
                                int32_t* n_instances, int32_t hyper[8]) {
    if (!m) { set_error("model_info: null"); return STRAIT_E_INVALID; }
    if (arch) *arch = m->arch;
    if (n_layers) *n_layers = (int32_t)m->ops.size();
    if (max_batch) *max_batch = m->max_batch;
    if (n_instances) *n_instances = (int32_t)m->inst.size();
    if (hyper) for (int i = 0; i < 8; ++i) hyper[i] = m->hyper[i];
    return STRAIT_OK;
}

strait_status strait_model_staging(const strait_model* m, int32_t instance, void** host_in, size_t* capacity) {
    if (!m || !host_in) { set_error("model_staging: null"); return STRAIT_E_INVALID; }
    if (instance < 0 || instance >= (int)m->inst.size()) { set_error("instance %d outside 0..%zu", instance, m->inst.size() - 1); return STRAIT_E_INVALID; }
    *host_in = m->inst[instance].pinned_in;
    if (capacity) *capacity = m->in_bytes(m->max_batch);
    return STRAIT_OK;
}

strait_status strait_model_layer(const strait_model* m, int32_t layer, strait_layer_info* out) {
    if (!m || !out) { set_error("model_layer: null"); return STRAIT_E_INVALID; }
    if (layer < 0 || layer >= (int)m->ops.size()) { set_error("layer %d outside 0..%zu", layer, m->ops.size() - 1); return STRAIT_E_INVALID; }
    *out = m->ops[layer].info;
    return STRAIT_OK;
}

static int check_call(strait_model* m, int instance, int prio, int batch) {
    if (!m) { set_error("null model"); return STRAIT_E_INVALID; }
    if (instance < 0 || instance >= (int)m->inst.size()) { set_error("instance %d outside 0..%zu", instance, m->inst.size() - 1); return STRAIT_E_INVALID; }
    if (prio != STRAIT_PRIO_HIGH && prio != STRAIT_PRIO_LOW) { set_error("priority must be STRAIT_PRIO_HIGH or STRAIT_PRIO_LOW"); return STRAIT_E_INVALID; }
    if (batch < 1 || batch > m->max_batch) { set_error("batch %d outside 1..%d", batch, m->max_batch); return STRAIT_E_BATCH; }
    return 0;
}

static hipStream_t compute_stream(Context* c, int prio, int instance) {
    return prio == STRAIT_PRIO_HIGH ? c->hp[instance % c->hp.size()] : c->lp[instance % c->lp.size()];
}

// Index of a compute stream in Context::workers / compute_mu (hp streams first, then lp).
static size_t compute_index(const Context* c, int prio, unsigned n) {
    return prio == STRAIT_PRIO_HIGH ? n % c->hp.size() : c->hp.size() + n % c->lp.size();
}

// Stage the input in the instance's pinned buffer (no lock: this is the slow part and instances are
// independent), then enqueue event / copy / event on copy stream `ci` as one uninterrupted group.
static int enqueue_h2d(strait_model* m, Instance& in, int batch, const void* host_in, const int32_t* valid_len, size_t ci) {
    Context* c = m->ctx;
    hipStream_t cs = c->copy[ci];
    const size_t inb = m->in_bytes(batch);
    if (host_in != in.pinned_in) memcpy(in.pinned_in, host_in, inb);
    int32_t* pv = nullptr;
    if (m->arch == STRAIT_ARCH_ENCODER) {
        const size_t off = (m->in_bytes(m->max_batch) + 255) / 256 * 256;
        pv = (int32_t*)((char*)in.pinned_in + off);
        for (int i = 0; i < batch; ++i) pv[i] = valid_len[i] < 0 ? 0 : (valid_len[i] > m->seq ? m->seq : valid_len[i]);
    }
    size_t kernel_limit;
    { std::lock_guard<std::mutex> ck(c->mu); kernel_limit = c->h2d_kernel_limit; }
    std::lock_guard<std::mutex> lk(c->copy_mu[ci]);
    HIP_TRY(hipEventRecord(in.ev_h2d0, cs));
    if (inb <= kernel_limit && (inb & 3) == 0) {
        // inputs of serving-sized batches go in by a kernel that reads the pinned buffer over the host link: an
        // asynchronous copy call of this size now and then blocks its caller for milliseconds
        if (launch_copy_mapped(in.pinned_in_dev, in.dev_in, inb, 0, cs)) return STRAIT_E_HIP;
        if (pv && launch_copy_mapped((const char*)in.pinned_in_dev + ((const char*)pv - (const char*)in.pinned_in), in.dev_valid, (size_t)batch * 4, 0, cs)) return STRAIT_E_HIP;
    } else {
        HIP_TRY(hipMemcpyAsync(in.dev_in, in.pinned_in, inb, hipMemcpyHostToDevice, cs));
        if (pv) HIP_TRY(hipMemcpyAsync(in.dev_valid, pv, (size_t)batch * 4, hipMemcpyHostToDevice, cs));
    }
    HIP_TRY(hipEventRecord(in.ev_h2d1, cs));
    return 0;
}

strait_status strait_submit(strait_model* m, strait_priority prio, int32_t batch, const void* host_in,
                            const int32_t* valid_len, void* host_out, strait_ticket* ticket) {
    const int64_t t_enq = now_ns();
    int rc = check_call(m, 0, prio, batch);
    if (rc) return rc;
    if (!host_in || !host_out || !ticket) { set_error("submit: null argument"); return STRAIT_E_INVALID; }
    if (m->arch == STRAIT_ARCH_ENCODER && !valid_len) { set_error("submit: the encoder needs valid_len"); return STRAIT_E_INVALID; }
    Context* c = m->ctx;
    int idx = -1;
    {
        std::lock_guard<std::mutex> lk(m->mu);
        int staged = -1;                              // input already in an instance's pinned buffer?
        for (size_t i = 0; i < m->inst.size(); ++i)
            if (host_in == m->inst[i].pinned_in) staged = (int)i;
        if (staged >= 0) {
            if (m->inst[staged].busy) { set_error("submit: instance %d, whose staging buffer was given, is busy", staged); return STRAIT_E_BUSY; }
            idx = staged;
        } else {
            for (size_t i = 0; i < m->inst.size(); ++i)
                if (!m->inst[i].busy) { idx = (int)i; break; }
        }
        if (idx < 0) { set_error("submit: all %zu instances busy", m->inst.size()); return STRAIT_E_BUSY; }
        m->inst[idx].busy = true;
        m->in_flight++;
    }
    auto release = [&]() { std::lock_guard<std::mutex> lk(m->mu); m->inst[idx].busy = false; m->in_flight--; };
    strait_ticket_s* t = new (std::nothrow) strait_ticket_s();
    if (!t) { release(); set_error("out of host memory"); return STRAIT_E_NOMEM; }
    Instance& in = m->inst[idx];
    unsigned si, ci;
    {
        std::lock_guard<std::mutex> lk(c->mu);
        si = prio == STRAIT_PRIO_HIGH ? c->n_hp_sub++ : c->n_lp_sub++;
        ci = c->n_copy_sub++;
    }
    const size_t widx = compute_index(c, prio, si);
    const size_t cidx = ci % c->copy.size();
    hipStream_t s = c->workers[widx]->stream;
    hipStream_t cs = c->copy[cidx];
    rc = hipSetDevice(c->device) == hipSuccess ? 0 : STRAIT_E_HIP;
    if (!rc) rc = enqueue_h2d(m, in, batch, host_in, valid_len, cidx);
    t->model = m; t->instance = idx; t->prio = prio; t->batch = batch; t->host_out = host_out;
    t->rec.model_id = m->id; t->rec.priority = prio; t->rec.batch = batch; t->rec.instance = idx;
    t->rec.t_enqueue_ns = t_enq;
    bool yielding;
    { std::lock_guard<std::mutex> lk(c->mu); yielding = prio == STRAIT_PRIO_LOW && c->lp_yield_layers > 0; }
    t->hp = hp_flag(c, prio);
    if (prio == STRAIT_PRIO_HIGH) c->hp_in_flight.fetch_add(1, std::memory_order_acq_rel);
    if (yielding) {
        // the stream's worker thread enqueues the kernels, segment by segment (issue_in_segments)
        t->deferred = true;
        if (!rc) {
            t->rec.t_issued_ns = now_ns();
            std::lock_guard<std::mutex> lk(c->mu);
            c->workers[widx]->q.push_back(t);
        }
    } else {
        std::lock_guard<std::mutex> slk(c->compute_mu[widx]);
        if (!rc) rc = hipStreamWaitEvent(s, in.ev_h2d1, 0) == hipSuccess ? 0 : STRAIT_E_HIP;
        if (!rc) rc = hipEventRecord(in.ev_k0, s) == hipSuccess ? 0 : STRAIT_E_HIP;
        if (!rc) rc = run_batch(*m, in, batch, s, hp_flag(c, prio));
        if (!rc) rc = hipEventRecord(in.ev_k1, s) == hipSuccess ? 0 : STRAIT_E_HIP;
        if (!rc) rc = launch_copy_mapped(in.dev_out, in.pinned_out_dev, m->out_bytes(batch), hp_flag(c, prio), s);
        if (!rc) rc = hipEventRecord(in.ev_done, s) == hipSuccess ? 0 : STRAIT_E_HIP;
        if (!rc) {
            t->rec.t_issued_ns = now_ns();
            std::lock_guard<std::mutex> lk(c->mu);          // tickets join the worker's queue in stream order
            c->workers[widx]->q.push_back(t);
        }
    }
    if (rc) {
        if (prio == STRAIT_PRIO_HIGH) c->hp_in_flight.fetch_sub(1, std::memory_order_acq_rel);
        if (rc == STRAIT_E_HIP && !strait::last_error()[0]) set_error("submit: a HIP call failed");
        (void)hipStreamSynchronize(s);
        (void)hipStreamSynchronize(cs);
        release();
        delete t;
        return rc;
    }
    c->cv_work.notify_all();
    *ticket = t;
    return STRAIT_OK;
}

strait_status strait_poll(strait_ticket t, int32_t* done) {
    if (!t || !done) { set_error("poll: null argument"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(t->model->ctx->mu);
    *done = t->done ? 1 : 0;
    return STRAIT_OK;
}

strait_status strait_wait(strait_ticket t, strait_record* rec) {
    if (!t) { set_error("wait: null ticket"); return STRAIT_E_INVALID; }
    Model* m = t->model;
    Context* c = m->ctx;
    {
        std::unique_lock<std::mutex> lk(c->mu);
        c->cv_done.wait(lk, [&] { return t->done; });
    }
    if (rec) *rec = t->rec;
    const int status = t->status;
    {
        std::lock_guard<std::mutex> lk(m->mu);
        m->inst[t->instance].busy = false;
        m->in_flight--;
    }
    delete t;
    if (status) { set_error("wait: the batch failed on the device"); return status; }
    return STRAIT_OK;
}

strait_status strait_copy_in(strait_model* m, int32_t instance, strait_priority prio, int32_t batch,
                             const void* host_in, const int32_t* valid_len) {
    int rc = check_call(m, instance, prio, batch);
    if (rc) return rc;
    if (!host_in) { set_error("copy_in: null input"); return STRAIT_E_INVALID; }
    if (m->arch == STRAIT_ARCH_ENCODER && !valid_len) { set_error("copy_in: the encoder needs valid_len"); return STRAIT_E_INVALID; }
    Context* c = m->ctx;
    HIP_TRY(hipSetDevice(c->device));
    rc = enqueue_h2d(m, m->inst[instance], batch, host_in, valid_len, (size_t)instance % c->copy.size());
    if (rc) return rc;
    std::lock_guard<std::mutex> slk(c->compute_mu[compute_index(c, prio, (unsigned)instance)]);
    HIP_TRY(hipStreamWaitEvent(compute_stream(c, prio, instance), m->inst[instance].ev_h2d1, 0));
    return STRAIT_OK;
}

strait_status strait_run(strait_model* m, int32_t instance, strait_priority prio, int32_t batch) {
    int rc = check_call(m, instance, prio, batch);
    if (rc) return rc;
    HIP_TRY(hipSetDevice(m->ctx->device));
    std::lock_guard<std::mutex> slk(m->ctx->compute_mu[compute_index(m->ctx, prio, (unsigned)instance)]);
    return run_batch(*m, m->inst[instance], batch, compute_stream(m->ctx, prio, instance), hp_flag(m->ctx, prio));
}

strait_status strait_copy_out(strait_model* m, int32_t instance, strait_priority prio, int32_t batch, void* host_out) {
    int rc = check_call(m, instance, prio, batch);
    if (rc) return rc;
    if (!host_out) { set_error("copy_out: null output"); return STRAIT_E_INVALID; }
    Instance& in = m->inst[instance];
    hipStream_t s = compute_stream(m->ctx, prio, instance);
    HIP_TRY(hipSetDevice(m->ctx->device));
    HIP_TRY(hipMemcpyAsync(in.pinned_out, in.dev_out, m->out_bytes(batch), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    memcpy(host_out, in.pinned_out, m->out_bytes(batch));
    return STRAIT_OK;
}

strait_status strait_sync(strait_model* m, int32_t instance, strait_priority prio) {
    int rc = check_call(m, instance, prio, 1);
    if (rc) return rc;
    HIP_TRY(hipSetDevice(m->ctx->device));
    HIP_TRY(hipStreamSynchronize(compute_stream(m->ctx, prio, instance)));
    return STRAIT_OK;
}

strait_status strait_run_timed(strait_model* m, int32_t instance, strait_priority prio, int32_t batch, float* layer_ms) {
    int rc = check_call(m, instance, prio, batch);
    if (rc) return rc;
    if (!layer_ms) { set_error("run_timed: null output"); return STRAIT_E_INVALID; }
    Instance& in = m->inst[instance];
    hipStream_t s = compute_stream(m->ctx, prio, instance);
    HIP_TRY(hipSetDevice(m->ctx->device));
    rc = run_plan(*m, in, batch, s, hp_flag(m->ctx, prio), -1, true);
    if (rc) return rc;
    HIP_TRY(hipStreamSynchronize(s));
    for (size_t i = 0; i < m->ops.size(); ++i) {
        HIP_TRY(hipEventElapsedTime(&layer_ms[i], in.layer_ev[i], in.layer_ev[i + 1]));
        if (in.layer_skipped[i]) layer_ms[i] = 0.f;    // its time is in the launch that computed it (between its events: nothing)
    }
    return STRAIT_OK;
}

strait_status strait_read_activation(strait_model* m, int32_t instance, int32_t layer, int32_t batch, void* host_out,
                                     size_t bytes, size_t* needed) {
    int rc = check_call(m, instance, STRAIT_PRIO_LOW, batch);
    if (rc) return rc;
    if (layer < 0 || layer >= (int)m->ops.size()) { set_error("layer %d outside 0..%zu", layer, m->ops.size() - 1); return STRAIT_E_INVALID; }
    const Op& op = m->ops[layer];
    if (op.out < 0) { set_error("layer %d ('%s') writes to the output buffer; use copy_out", layer, op.name.c_str()); return STRAIT_E_INVALID; }
    const size_t need = (size_t)batch * op.P * op.Q * op.K * 2;
    if (needed) *needed = need;
    if (!host_out) return STRAIT_OK;
    if (bytes != need) { set_error("read_activation: layer '%s' holds %zu bytes for batch %d, caller gave %zu", op.name.c_str(), need, batch, bytes); return STRAIT_E_INVALID; }
    Instance& in = m->inst[instance];
    hipStream_t s = compute_stream(m->ctx, STRAIT_PRIO_LOW, instance);
    HIP_TRY(hipSetDevice(m->ctx->device));
    rc = run_plan(*m, in, batch, s, 0, layer, false);     // re-run the prefix: later layers reuse buffers
    if (rc) return rc;
    HIP_TRY(hipStreamSynchronize(s));
    HIP_TRY(hipMemcpy(host_out, in.bufs[op.out], need, hipMemcpyDeviceToHost));
    return STRAIT_OK;
}

// ---- kernel-level entry points -----------------------------------------------------------------

strait_status strait_k_conv2d(void* stream, const void* x, int32_t N, int32_t H, int32_t W, int32_t C,
                              const void* w_krsc, const float* bias, int32_t K, int32_t R, int32_t S, int32_t stride,
                              int32_t pad, int32_t act, const void* res, void* y, int32_t out_f32, int32_t hp) {
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || K <= 0 || R <= 0 || S <= 0 || stride <= 0 || pad < 0 ||
        H + 2 * pad < R || W + 2 * pad < S) { set_error("conv2d: invalid shape"); return STRAIT_E_SHAPE; }
    const int P = (H + 2 * pad - R) / stride + 1, Q = (W + 2 * pad - S) / stride + 1;
    if ((long long)N * P * Q > 0x7fffffffLL || (long long)R * S * C > 0x7fffffffLL) { set_error("conv2d: too large"); return STRAIT_E_SHAPE; }
    ConvParams p{};
    p.x = (const half_t*)x; p.bias = bias; p.res = (const half_t*)res; p.y = y;
    p.M = N * P * Q; p.PQ = P * Q; p.Q = Q; p.H = H; p.W = W; p.C = C; p.R = R; p.S = S;
    p.stride_h = p.stride_w = stride; p.pad_h = p.pad_w = pad;
    p.sN = (long long)H * W * C; p.sH = W * C; p.sW = C;
    p.Kg = R * S * C; p.Cout = K; p.ldy = K; p.act = act; p.out_f32 = out_f32; p.hp = hp;
    void* tmp = nullptr;
    if (p.Kg % 8 == 0) { p.w = (const half_t*)w_krsc; p.ldw = p.Kg; }
    else {
        // rows padded with zeros to a multiple of 8 elements, as the kernel's 16-byte weight loads need
        p.ldw = (p.Kg + 7) / 8 * 8;
        HIP_TRY(hipMalloc(&tmp, (size_t)K * p.ldw * 2));
        hipError_t e = hipMemsetAsync(tmp, 0, (size_t)K * p.ldw * 2, (hipStream_t)stream);
        if (e == hipSuccess) e = hipMemcpy2DAsync(tmp, (size_t)p.ldw * 2, w_krsc, (size_t)p.Kg * 2, (size_t)p.Kg * 2, K, hipMemcpyDeviceToDevice, (hipStream_t)stream);
        if (e != hipSuccess) { (void)hipFree(tmp); set_error("conv2d: padding the weights failed: %s", hipGetErrorString(e)); return STRAIT_E_HIP; }
        p.w = (const half_t*)tmp;
    }
    // small problems may take the split-K path, which needs an fp32 workspace
    void* ws = nullptr;
    if ((long long)p.M * K <= 128LL * 4096) {
        if (hipMalloc(&ws, SPLITK_WS_BYTES) != hipSuccess) { (void)hipGetLastError(); ws = nullptr; }
        p.ws = (float*)ws; p.ws_bytes = ws ? SPLITK_WS_BYTES : 0;
    }
    int rc = launch_conv(p, (hipStream_t)stream);
    if (tmp || ws) { (void)hipStreamSynchronize((hipStream_t)stream); if (tmp) (void)hipFree(tmp); if (ws) (void)hipFree(ws); }
    return rc;
}

strait_status strait_k_conv1x1_proj(void* stream, const void* x, int32_t N, int32_t P, int32_t Q, int32_t C, const void* x2,
                                    int32_t H2, int32_t W2, int32_t K2, int32_t stride2, const void* w, const float* bias,
                                    int32_t Cout, int32_t act, void* y, int32_t hp) {
    if (N <= 0 || P <= 0 || Q <= 0 || C <= 0 || K2 <= 0 || Cout <= 0 || stride2 <= 0 || H2 <= 0 || W2 <= 0 ||
        (long long)(P - 1) * stride2 >= H2 || (long long)(Q - 1) * stride2 >= W2 || (long long)N * P * Q > 0x7fffffffLL) {
        set_error("conv1x1_proj: invalid shape (every output pixel needs its pixel of the second tensor)"); return STRAIT_E_SHAPE;
    }
    if (!x2) { set_error("conv1x1_proj: x2 is required"); return STRAIT_E_INVALID; }
    ConvParams p{};
    p.x = (const half_t*)x; p.w = (const half_t*)w; p.bias = bias; p.y = y;
    p.M = N * P * Q; p.PQ = P * Q; p.Q = Q; p.H = P; p.W = Q; p.C = C; p.R = 1; p.S = 1;
    p.stride_h = p.stride_w = 1; p.pad_h = p.pad_w = 0;
    p.sN = (long long)P * Q * C; p.sH = Q * C; p.sW = C;
    p.x2 = (const half_t*)x2; p.K2 = K2; p.stride2 = stride2; p.sN2 = (long long)H2 * W2 * K2; p.sH2 = W2 * K2; p.sW2 = K2;
    p.Kg = C + K2; p.ldw = C + K2; p.Cout = Cout; p.ldy = Cout; p.act = act; p.hp = hp;
    void* ws = nullptr;                                // small problems may take the split-K path, which needs an fp32 workspace
    if ((long long)p.M * Cout <= 128LL * 4096) {
        if (hipMalloc(&ws, SPLITK_WS_BYTES) != hipSuccess) { (void)hipGetLastError(); ws = nullptr; }
        p.ws = (float*)ws; p.ws_bytes = ws ? SPLITK_WS_BYTES : 0;
    }
    const int rc = launch_conv(p, (hipStream_t)stream);
    if (ws) { (void)hipStreamSynchronize((hipStream_t)stream); (void)hipFree(ws); }
    return rc;
}

strait_status strait_k_gemm(void* stream, const void* x, const void* w, const float* bias, int32_t M, int32_t N,
                            int32_t K, int32_t act, const void* res, void* y, int32_t out_f32, int32_t hp) {
    if (M <= 0 || N <= 0 || K <= 0 || K % 8 != 0) { set_error("gemm: needs positive sizes and K %% 8 == 0"); return STRAIT_E_SHAPE; }
    ConvParams p{};
    p.x = (const half_t*)x; p.w = (const half_t*)w; p.bias = bias; p.res = (const half_t*)res; p.y = y;
    p.M = M; p.PQ = 1; p.Q = 1; p.H = 1; p.W = 1; p.C = K; p.R = 1; p.S = 1;
    p.stride_h = p.stride_w = 1; p.pad_h = p.pad_w = 0;
    p.sN = K; p.sH = K; p.sW = K; p.Kg = K; p.ldw = K; p.Cout = N; p.ldy = N; p.act = act; p.out_f32 = out_f32; p.hp = hp;
    void* ws = nullptr;
    if ((long long)M * N <= 128LL * 4096) {
        if (hipMalloc(&ws, SPLITK_WS_BYTES) != hipSuccess) { (void)hipGetLastError(); ws = nullptr; }
        p.ws = (float*)ws; p.ws_bytes = ws ? SPLITK_WS_BYTES : 0;
    }
    int rc = launch_conv(p, (hipStream_t)stream);
    if (ws) { (void)hipStreamSynchronize((hipStream_t)stream); (void)hipFree(ws); }
    return rc;
}

strait_status strait_k_pointwise_pair(void* stream, const void* x, const void* w3, const float* b3, const void* res, void* y,
                                      const void* w1, const float* b1, void* z, int32_t M, int32_t K1, int32_t N1, int32_t N2,
                                      int32_t act1, int32_t act2, int32_t hp) {
    PairParams p{};
    p.x = (const half_t*)x; p.w3 = (const half_t*)w3; p.b3 = b3; p.res = (const half_t*)res; p.y = (half_t*)y;
    p.w1 = (const half_t*)w1; p.b1 = b1; p.z = (half_t*)z;
    p.M = M; p.K1 = K1; p.N1 = N1; p.N2 = N2; p.act1 = act1; p.act2 = act2; p.hp = hp;
    return launch_pointwise_pair(p, (hipStream_t)stream);
}

strait_status strait_k_pointwise_pair_proj(void* stream, const void* x, const void* x2, const void* w3, const float* b3, void* y,
                                           const void* w1, const float* b1, void* z, int32_t M, int32_t K1, int32_t K2, int32_t N1,
                                           int32_t N2, int32_t act1, int32_t act2, int32_t hp) {
    if (!x2) { set_error("pointwise pair with projection: x2 is required"); return STRAIT_E_INVALID; }
    PairParams p{};
    p.x = (const half_t*)x; p.x2 = (const half_t*)x2; p.w3 = (const half_t*)w3; p.b3 = b3; p.y = (half_t*)y;
    p.w1 = (const half_t*)w1; p.b1 = b1; p.z = (half_t*)z;
    p.M = M; p.K1 = K1; p.K2 = K2; p.N1 = N1; p.N2 = N2; p.act1 = act1; p.act2 = act2; p.hp = hp;
    return launch_pointwise_pair(p, (hipStream_t)stream);
}

strait_status strait_k_dwconv3x3(void* stream, const void* x, int32_t N, int32_t H, int32_t W, int32_t C,
                                 const void* w_rsc, const float* bias, int32_t stride, int32_t act, void* y, int32_t hp) {
    return launch_dwconv3x3((const half_t*)x, N, H, W, C, (const half_t*)w_rsc, bias, stride, act, (half_t*)y, hp, (hipStream_t)stream);
}
strait_status strait_k_stem3x3s2(void* stream, const void* x, int32_t N, int32_t H, int32_t W, const void* wf, const float* bias,
                                 int32_t Kout, int32_t act, void* y, int32_t hp) {
    return launch_stem3x3s2((const half_t*)x, (const half_t*)wf, bias, N, H, W, Kout, act, (half_t*)y, hp, (hipStream_t)stream);
}
strait_status strait_k_stem3x3s2_dw(void* stream, const void* x, int32_t N, int32_t H, int32_t W, const void* wf, const float* bias,
                                    int32_t act1, const void* wd_rsc, const float* bd, int32_t act2, void* y, int32_t hp) {
    return launch_stem3x3s2_dw((const half_t*)x, (const half_t*)wf, bias, act1, (const half_t*)wd_rsc, bd, act2, N, H, W, (half_t*)y, hp,
                               (hipStream_t)stream);
}
strait_status strait_k_expand_dw(void* stream, const void* x, int32_t N, int32_t H, int32_t W, int32_t Cin, const void* w1,
                                 const float* b1, int32_t Chid, int32_t act1, const void* wd_rsc, const float* bd, int32_t stride,
                                 int32_t act2, void* y, int32_t hp) {
    return launch_expand_dw((const half_t*)x, N, H, W, Cin, (const half_t*)w1, Cin, b1, Chid, act1, (const half_t*)wd_rsc, bd, stride, act2,
                            (half_t*)y, hp, (hipStream_t)stream);
}
strait_status strait_k_maxpool3x3s2(void* stream, const void* x, int32_t N, int32_t H, int32_t W, int32_t C, void* y, int32_t hp) {
    return launch_maxpool3x3s2((const half_t*)x, N, H, W, C, (half_t*)y, hp, (hipStream_t)stream);
}
strait_status strait_k_stem_pool(void* stream, const void* x, int32_t N, int32_t H, int32_t W, const void* wf, const float* bias,
                                 void* y, int32_t hp) {
    return launch_stem_pool((const half_t*)x, (const half_t*)wf, bias, N, H, W, (half_t*)y, hp, (hipStream_t)stream);
}
strait_status strait_k_maxpool2x2s2(void* stream, const void* x, int32_t N, int32_t H, int32_t W, int32_t C, void* y, int32_t hp) {
    return launch_maxpool2x2s2((const half_t*)x, N, H, W, C, (half_t*)y, hp, (hipStream_t)stream);
}
strait_status strait_k_vit_tokens(void* stream, const void* patch, const float* cls, const float* pos, int32_t N, int32_t T,
                                  int32_t D, void* z, int32_t hp) {
    return launch_vit_tokens((const half_t*)patch, cls, pos, N, T, D, (half_t*)z, hp, (hipStream_t)stream);
}
strait_status strait_k_global_avgpool(void* stream, const void* x, int32_t N, int32_t HW, int32_t C, void* y, int32_t hp) {
    return launch_global_avgpool((const half_t*)x, N, HW, C, (half_t*)y, hp, (hipStream_t)stream);
}
strait_status strait_k_softmax_top1(void* stream, const float* logits, int32_t rows, int32_t n, float* probs, int32_t* top1, int32_t hp) {
    return launch_softmax_top1(logits, rows, n, probs, top1, hp, (hipStream_t)stream);
}
strait_status strait_k_layernorm(void* stream, const void* x, const float* gamma, const float* beta, int32_t rows,
                                 int32_t n, float eps, void* y, int32_t hp) {
    return launch_layernorm((const half_t*)x, gamma, beta, rows, n, eps, (half_t*)y, hp, (hipStream_t)stream);
}
strait_status strait_k_attention(void* stream, const void* qkv, const int32_t* valid_len, int32_t B, int32_t S,
                                 int32_t heads, void* out, int32_t hp) {
    return launch_attention((const half_t*)qkv, valid_len, B, S, heads, (half_t*)out, hp, (hipStream_t)stream);
}
strait_status strait_k_argmax_f16(void* stream, const void* x, int32_t rows, int32_t n, int64_t row_stride, int32_t* top1, int32_t hp) {
    return launch_argmax_f16((const half_t*)x, rows, n, row_stride, top1, hp, (hipStream_t)stream);
}

}  // extern "C"
