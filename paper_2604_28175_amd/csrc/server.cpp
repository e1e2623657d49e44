// Serving front end and offline profiling (paper Section 3, system workflow; Section 4; Section 5.1).
//
// Requests wait in one task queue per model.  A queue asks for a decision when it holds a full batch or
// its oldest request has waited the model's batch formation timeout.  The scheduling thread visits the
// asking queues in descending priority (first come first served within a level), takes one decision per
// visit from the scheduling policy (Algorithm 1), drops what the policy drops, gathers the chosen requests
// into the pinned buffer of a free instance and submits them as one batch.  Execution threads wait for the
// batches, scatter the outputs and report the measured kernel latency and transfer time to the policy.
//
// Layering: this file uses the library's own C entry points (strait_model_*, strait_submit, strait_wait,
// strait_sched_*) and nothing beneath them.
#include <time.h>

#include <algorithm>
#include <chrono>
#include <cmath>
#include <condition_variable>
#include <cstring>
#include <deque>
#include <limits>
#include <map>
#include <mutex>
#include <new>
#include <thread>
#include <vector>

#include "../../include/strait.h"
#include "kernels.hpp"

using strait::set_error;

namespace {

int64_t now_ns() {
    timespec ts;
    clock_gettime(CLOCK_MONOTONIC, &ts);
    return (int64_t)ts.tv_sec * 1000000000LL + ts.tv_nsec;
}

struct Request {
    uint64_t id;
    const void* in;
    void* out;
    int32_t valid_len;
    int64_t t_enq, deadline;
};

struct ModelQ {
    strait_server_model d{};
    int arch = 0, classes = 0, seq = 0, hidden = 0;
    size_t in1 = 0, out1 = 0;                 // bytes of one sample's input / output
    std::deque<Request> q;
    std::vector<int> free_inst;
    std::vector<std::vector<char>> out_buf;   // per instance: a whole batch's output
    bool deferred = false;                    // asked, could not be placed: asks again
};

struct Batch {
    ModelQ* mq = nullptr;
    std::vector<Request> reqs;
    std::vector<int32_t> valid;
    strait_decision dec{};
    int instance = -1;
    int64_t t_dispatch = 0;
    uint64_t seq = 0;
    strait_ticket ticket = nullptr;
};

}  // namespace

struct strait_server {
    strait_sched* sched = nullptr;
    int concurrency = 4;
    int64_t retry_ns = 200000;
    bool external = false;
    strait_executor ex{};

    std::mutex mu;                            // queues, batches in flight, results, counters
    std::mutex sched_mu;                      // every call into the policy, with the time taken inside
    std::condition_variable cv_sched, cv_exec, cv_idle;
    std::map<int, ModelQ> models;
    std::deque<Batch*> dispatched;
    std::deque<strait_request_record> results;
    strait_server_stats stats{};
    int in_flight = 0;
    bool running = false, stopping = false, kick = false;
    bool sched_done = false;                  // the scheduling thread has ended: no batch will be dispatched any more
    uint64_t next_req = 1, next_batch = 1;
    int64_t last_h2d_end = 0;
    std::thread sched_th;
    std::vector<std::thread> exec_th;

    void record(const ModelQ& mq, const Request& r, int status, const Batch* b, int pos, int64_t t_done,
                double kernel_ns, double h2d_ns) {
        strait_request_record rec{};
        rec.request_id = r.id;
        rec.batch_seq = b ? b->seq : 0;
        rec.model_id = mq.d.model_id;
        rec.priority = mq.d.priority;
        rec.status = status;
        rec.batch = b ? (int32_t)b->reqs.size() : 0;
        rec.position = pos;
        rec.violated = (status != 0 || t_done > r.deadline) ? 1 : 0;
        rec.t_enqueue_ns = r.t_enq;
        rec.t_dispatch_ns = b ? b->t_dispatch : 0;
        rec.t_done_ns = t_done;
        rec.deadline_ns = r.deadline;
        rec.t_inf_pred_ns = b ? b->dec.t_inf_ns : 0.0;
        rec.kernel_ns = kernel_ns;
        rec.h2d_ns = h2d_ns;
        results.push_back(rec);
        if (status == 0) ++stats.served;
        else if (status == 1) ++stats.dropped;
        else if (status == 2) ++stats.failed;
        if (rec.violated) { if (mq.d.priority == STRAIT_PRIO_HIGH) ++stats.violated_high; else ++stats.violated_low; }
    }

    bool idle() const {
        if (in_flight > 0) return false;
        for (const auto& kv : models) if (!kv.second.q.empty()) return false;
        return true;
    }

    // -- executor ---------------------------------------------------------------------------------------
    int submit(Batch& b) {
        ModelQ& mq = *b.mq;
        const int n = (int)b.reqs.size();
        if (external) {
            std::vector<const void*> ins(n);
            std::vector<void*> outs(n);
            for (int i = 0; i < n; ++i) { ins[i] = b.reqs[i].in; outs[i] = b.reqs[i].out; }
            return ex.submit(ex.user, b.seq, mq.d.model_id, mq.d.priority, n, ins.data(), outs.data(), b.valid.data());
        }
        void* stage = nullptr;
        size_t cap = 0;
        int rc = strait_model_staging(mq.d.model, b.instance, &stage, &cap);
        if (rc != STRAIT_OK) return rc;
        for (int i = 0; i < n; ++i) memcpy((char*)stage + (size_t)i * mq.in1, b.reqs[i].in, mq.in1);
        return strait_submit(mq.d.model, (strait_priority)mq.d.priority, n, stage, b.valid.data(),
                             mq.out_buf[b.instance].data(), &b.ticket);
    }

    int wait(Batch& b, double* kernel_ns, double* h2d_ns, int64_t* t_done) {
        ModelQ& mq = *b.mq;
        const int n = (int)b.reqs.size();
        if (external) {
            const int rc = ex.wait(ex.user, b.seq, kernel_ns, h2d_ns);
            *t_done = now_ns();
            return rc;
        }
        strait_record rec{};
        const int rc = strait_wait(b.ticket, &rec);
        if (rc != STRAIT_OK) { *t_done = now_ns(); return rc; }
        *kernel_ns = (double)rec.kernel_ms * 1e6;
        *h2d_ns = (double)rec.h2d_ms * 1e6;
        const char* src = mq.out_buf[b.instance].data();
        // a batch's output is laid out region by region; a request's output is the same layout at batch 1
        if (mq.arch == STRAIT_ARCH_ENCODER) {
            const size_t hs = (size_t)mq.seq * mq.hidden * 2;
            for (int i = 0; i < n; ++i) {
                char* dst = (char*)b.reqs[i].out;
                memcpy(dst, src + (size_t)i * hs, hs);
                memcpy(dst + hs, src + (size_t)n * hs + (size_t)i * 4, 4);
            }
        } else {
            const size_t row = (size_t)mq.classes * 4;
            for (int i = 0; i < n; ++i) {
                char* dst = (char*)b.reqs[i].out;
                memcpy(dst, src + (size_t)i * row, row);
                memcpy(dst + row, src + (size_t)n * row + (size_t)i * row, row);
                memcpy(dst + 2 * row, src + 2 * (size_t)n * row + (size_t)i * 4, 4);
            }
        }
        *t_done = now_ns();      // the result is in the requests' own memory now
        return STRAIT_OK;
    }

    // -- scheduling thread ------------------------------------------------------------------------------
    // One visit to every asking queue.  Returns whether a batch left or a request was dropped.
    bool pass(std::unique_lock<std::mutex>& lk) {
        const int64_t t = now_ns();
        std::vector<ModelQ*> asking;
        for (auto& kv : models) {
            ModelQ& mq = kv.second;
            if (mq.q.empty()) { mq.deferred = false; continue; }
            if ((int)mq.q.size() >= mq.d.max_batch || t - mq.q.front().t_enq >= mq.d.formation_timeout_ns || mq.deferred)
                asking.push_back(&mq);
        }
        std::stable_sort(asking.begin(), asking.end(), [](const ModelQ* a, const ModelQ* b) {
            if (a->d.priority != b->d.priority) return a->d.priority < b->d.priority;
            return a->q.front().t_enq < b->q.front().t_enq;
        });
        bool progress = false;
        for (ModelQ* mq : asking) {
            if (in_flight >= concurrency || mq->free_inst.empty()) {
                if (!mq->deferred) ++stats.deferrals;
                mq->deferred = true;
                continue;
            }
            const int n = (int)std::min<size_t>(mq->q.size(), 1024);
            std::vector<int64_t> enq(n), ddl(n);
            for (int i = 0; i < n; ++i) { enq[i] = mq->q[i].t_enq; ddl[i] = mq->q[i].deadline; }
            strait_decision dec{};
            int64_t t_dec = 0;
            int rc;
            {
                std::lock_guard<std::mutex> sl(sched_mu);
                t_dec = now_ns();
                rc = strait_sched_decide(sched, mq->d.model_id, t_dec, enq.data(), ddl.data(), n, &dec);
            }
            if (rc != STRAIT_OK) { mq->deferred = true; continue; }
            for (int i = 0; i < dec.n_dropped; ++i) {
                record(*mq, mq->q.front(), 1, nullptr, 0, t_dec, 0.0, 0.0);
                mq->q.pop_front();
                progress = true;
            }
            if (dec.batch <= 0) {
                if (!mq->q.empty() && !mq->deferred) ++stats.deferrals;
                mq->deferred = !mq->q.empty();
                continue;
            }
            Batch* b = new Batch;
            b->mq = mq;
            b->dec = dec;
            b->t_dispatch = t_dec;
            b->seq = next_batch++;
            for (int i = 0; i < dec.batch; ++i) {
                b->reqs.push_back(mq->q.front());
                b->valid.push_back(mq->q.front().valid_len);
                mq->q.pop_front();
            }
            b->instance = mq->free_inst.back();
            mq->free_inst.pop_back();
            mq->deferred = false;
            ++in_flight;
            if (in_flight > stats.max_in_flight) stats.max_in_flight = in_flight;
            ++stats.batches;
            stats.batched_requests += dec.batch;
            lk.unlock();
            rc = submit(*b);
            lk.lock();
            progress = true;
            if (rc != 0) {
                int64_t t_fail;
                {
                    std::lock_guard<std::mutex> sl(sched_mu);
                    t_fail = now_ns();
                    (void)strait_sched_complete(sched, dec.gpu, dec.running_id, t_fail, std::numeric_limits<double>::quiet_NaN(), -1, nullptr);
                }
                for (size_t i = 0; i < b->reqs.size(); ++i) record(*mq, b->reqs[i], 2, b, (int)i, t_fail, 0.0, 0.0);
                mq->free_inst.push_back(b->instance);
                --in_flight;
                delete b;
                cv_idle.notify_all();
                continue;
            }
            dispatched.push_back(b);
            cv_exec.notify_one();
        }
        return progress;
    }

    void sched_loop() {
        std::unique_lock<std::mutex> lk(mu);
        while (!stopping) {
            kick = false;
            if (pass(lk)) continue;
            if (idle()) cv_idle.notify_all();
            int64_t wake = std::numeric_limits<int64_t>::max();
            const int64_t t = now_ns();
            for (const auto& kv : models) {
                const ModelQ& mq = kv.second;
                if (mq.q.empty()) continue;
                const int64_t w = mq.deferred ? t + retry_ns : mq.q.front().t_enq + mq.d.formation_timeout_ns;
                wake = std::min(wake, w);
            }
            if (kick || stopping) continue;
            if (wake == std::numeric_limits<int64_t>::max()) cv_sched.wait(lk, [&] { return kick || stopping; });
            else if (wake > t) cv_sched.wait_for(lk, std::chrono::nanoseconds(wake - t), [&] { return kick || stopping; });
        }
    }

    // -- execution threads ------------------------------------------------------------------------------
    void exec_loop() {
        for (;;) {
            Batch* b = nullptr;
            {
                std::unique_lock<std::mutex> lk(mu);
                cv_exec.wait(lk, [&] { return !dispatched.empty() || (sched_done && in_flight == 0); });
                if (dispatched.empty()) return;
                b = dispatched.front();
                dispatched.pop_front();
            }
            double kernel_ns = 0.0, h2d_ns = 0.0;
            int64_t t_done = 0;
            const int rc = wait(*b, &kernel_ns, &h2d_ns, &t_done);
            int64_t h2d_end = -1;
            {
                std::lock_guard<std::mutex> lk(mu);
                if (rc == 0 && h2d_ns > 0.0) {
                    // transfers of one GPU are served first in, first out (Eq. 3): this one started when it was
                    // issued or when its predecessor ended, whichever came later
                    h2d_end = std::max(b->t_dispatch, last_h2d_end) + (int64_t)h2d_ns;
                    last_h2d_end = h2d_end;
                }
            }
            {
                std::lock_guard<std::mutex> sl(sched_mu);
                (void)strait_sched_complete(sched, b->dec.gpu, b->dec.running_id, now_ns(),
                                            rc == 0 ? kernel_ns : std::numeric_limits<double>::quiet_NaN(), h2d_end, nullptr);
            }
            {
                std::lock_guard<std::mutex> lk(mu);
                for (size_t i = 0; i < b->reqs.size(); ++i)
                    record(*b->mq, b->reqs[i], rc == 0 ? 0 : 2, b, (int)i, t_done, kernel_ns, h2d_ns);
                b->mq->free_inst.push_back(b->instance);
                --in_flight;
                kick = true;
                if (idle()) cv_idle.notify_all();
            }
            cv_sched.notify_one();
            cv_exec.notify_all();
            delete b;
        }
    }
};

extern "C" {

strait_status strait_server_create(strait_sched* sched, int32_t concurrency, int64_t retry_ns,
                                   const strait_executor* executor, strait_server** out) {
    if (!sched || !out) { set_error("server_create: null argument"); return STRAIT_E_INVALID; }
    if (concurrency < 1 || concurrency > 64 || retry_ns <= 0) { set_error("server_create: concurrency must be in 1..64 and retry_ns positive"); return STRAIT_E_INVALID; }
    if (executor && (!executor->submit || !executor->wait)) { set_error("server_create: executor without submit or wait"); return STRAIT_E_INVALID; }
    strait_server* s = new (std::nothrow) strait_server;
    if (!s) { set_error("out of host memory"); return STRAIT_E_NOMEM; }
    s->sched = sched;
    s->concurrency = concurrency;
    s->retry_ns = retry_ns;
    if (executor) { s->external = true; s->ex = *executor; }
    *out = s;
    return STRAIT_OK;
}

strait_status strait_server_add_model(strait_server* s, const strait_server_model* d) {
    if (!s || !d) { set_error("server_add_model: null argument"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(s->mu);
    if (s->running || s->stopping) { set_error("server_add_model: server already started"); return STRAIT_E_BUSY; }
    if (s->models.count(d->model_id)) { set_error("server_add_model: model id %d added twice", d->model_id); return STRAIT_E_INVALID; }
    if ((d->priority != STRAIT_PRIO_HIGH && d->priority != STRAIT_PRIO_LOW) || d->max_batch < 1 || d->deadline_ns <= 0 ||
        d->formation_timeout_ns < 0 || d->n_instances < 0) { set_error("server_add_model: bad priority, batch limit, deadline, timeout or instance count"); return STRAIT_E_INVALID; }
    if (!d->model && !s->external) { set_error("server_add_model: no model and no executor"); return STRAIT_E_INVALID; }
    ModelQ mq;
    mq.d = *d;
    int n_inst = d->n_instances;
    if (d->model) {
        int32_t arch = 0, n_layers = 0, max_batch = 0, inst = 0, hyper[8] = {0};
        int rc = strait_model_info(d->model, &arch, &n_layers, &max_batch, &inst, hyper);
        if (rc != STRAIT_OK) return rc;
        if (d->max_batch > max_batch) { set_error("server_add_model: max_batch %d above the model's %d", d->max_batch, max_batch); return STRAIT_E_BATCH; }
        if (n_inst == 0) n_inst = inst;
        if (n_inst > inst) { set_error("server_add_model: %d instances asked, the model has %d", n_inst, inst); return STRAIT_E_INVALID; }
        rc = strait_model_io(d->model, 1, &mq.in1, &mq.out1);
        if (rc != STRAIT_OK) return rc;
        mq.arch = arch;
        if (arch == STRAIT_ARCH_ENCODER) { mq.hidden = hyper[1]; mq.seq = hyper[4]; }
        else mq.classes = (int)((mq.out1 - 4) / 8);
        size_t in_b = 0, out_b = 0;
        rc = strait_model_io(d->model, d->max_batch, &in_b, &out_b);
        if (rc != STRAIT_OK) return rc;
        if (!s->external) mq.out_buf.assign(n_inst, std::vector<char>(out_b));
    } else if (n_inst == 0) {
        n_inst = 1;
    }
    mq.d.n_instances = n_inst;
    for (int i = n_inst - 1; i >= 0; --i) mq.free_inst.push_back(i);
    s->models.emplace(d->model_id, std::move(mq));
    return STRAIT_OK;
}

strait_status strait_server_start(strait_server* s) {
    if (!s) { set_error("server_start: null"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(s->mu);
    if (s->running || s->stopping) { set_error("server_start: already started"); return STRAIT_E_BUSY; }
    if (s->models.empty()) { set_error("server_start: no models"); return STRAIT_E_INVALID; }
    if (!s->external) {
        // Warm-up, so that no request pays for a first use: every (instance, batch size) runs twice (with graph
        // replay switched on in the context, the second run captures that key's graph), then every instance of every model
        // is submitted at once, three times over (the runtime grows its per-stream pools the first time streams are
        // that deep, which stalls the submitting thread for milliseconds).
        std::vector<strait_ticket> burst;
        for (auto& kv : s->models) {
            ModelQ& mq = kv.second;
            std::vector<int32_t> valid(mq.d.max_batch, mq.seq);
            for (int inst = 0; inst < mq.d.n_instances; ++inst) {
                void* stage = nullptr;
                size_t cap = 0;
                int rc = strait_model_staging(mq.d.model, inst, &stage, &cap);
                if (rc != STRAIT_OK) return rc;
                memset(stage, 0, mq.in1 * (size_t)mq.d.max_batch);
                for (int b = 1; b <= mq.d.max_batch; ++b)
                    for (int rep = 0; rep < 2; ++rep) {
                        strait_ticket tk = nullptr;
                        rc = strait_submit(mq.d.model, (strait_priority)mq.d.priority, b, stage, valid.data(), mq.out_buf[inst].data(), &tk);
                        if (rc == STRAIT_OK) rc = strait_wait(tk, nullptr);
                        if (rc != STRAIT_OK) return rc;
                    }
            }
        }
        int rc = STRAIT_OK;
        for (int round = 0; round < 3 && rc == STRAIT_OK; ++round) {
            // every instance of every model at once, models interleaved: all streams as deep as they will ever be
            burst.clear();
            int max_inst = 0;
            for (auto& kv : s->models) max_inst = std::max(max_inst, kv.second.d.n_instances);
            for (int inst = 0; inst < max_inst && rc == STRAIT_OK; ++inst)
                for (auto& kv : s->models) {
                    ModelQ& mq = kv.second;
                    if (inst >= mq.d.n_instances || rc != STRAIT_OK) continue;
                    std::vector<int32_t> valid(mq.d.max_batch, mq.seq);
                    void* stage = nullptr;
                    size_t cap = 0;
                    rc = strait_model_staging(mq.d.model, inst, &stage, &cap);
                    strait_ticket tk = nullptr;
                    if (rc == STRAIT_OK) rc = strait_submit(mq.d.model, (strait_priority)mq.d.priority, mq.d.max_batch, stage, valid.data(), mq.out_buf[inst].data(), &tk);
                    if (rc == STRAIT_OK) burst.push_back(tk);
                }
            for (strait_ticket tk : burst) { const int r2 = strait_wait(tk, nullptr); if (rc == STRAIT_OK) rc = r2; }
        }
        if (rc != STRAIT_OK) return rc;
    }
    s->running = true;
    s->sched_th = std::thread([s] { s->sched_loop(); });
    for (int i = 0; i < s->concurrency; ++i) s->exec_th.emplace_back([s] { s->exec_loop(); });
    return STRAIT_OK;
}

strait_status strait_server_request(strait_server* s, int32_t model_id, const void* host_in, int32_t valid_len,
                                    void* host_out, uint64_t* request_id) {
    if (!s) { set_error("server_request: null"); return STRAIT_E_INVALID; }
    const int64_t t = now_ns();
    {
        std::lock_guard<std::mutex> lk(s->mu);
        if (!s->running || s->stopping) { set_error("server_request: server not running"); return STRAIT_E_INVALID; }
        auto it = s->models.find(model_id);
        if (it == s->models.end()) { set_error("server_request: unknown model id %d", model_id); return STRAIT_E_INVALID; }
        ModelQ& mq = it->second;
        if (!s->external && (!host_in || !host_out)) { set_error("server_request: null buffer"); return STRAIT_E_INVALID; }
        if (mq.arch == STRAIT_ARCH_ENCODER && mq.d.model && (valid_len < 1 || valid_len > mq.seq)) {
            set_error("server_request: valid_len %d outside 1..%d", valid_len, mq.seq); return STRAIT_E_SHAPE;
        }
        Request r{s->next_req++, host_in, host_out, valid_len, t, t + mq.d.deadline_ns};
        mq.q.push_back(r);
        ++s->stats.requests;
        if (mq.d.priority == STRAIT_PRIO_HIGH) ++s->stats.requests_high; else ++s->stats.requests_low;
        if (request_id) *request_id = r.id;
        s->kick = true;
    }
    s->cv_sched.notify_one();
    return STRAIT_OK;
}

strait_status strait_server_wait_idle(strait_server* s, int64_t timeout_ns) {
    if (!s) { set_error("server_wait_idle: null"); return STRAIT_E_INVALID; }
    std::unique_lock<std::mutex> lk(s->mu);
    if (!s->cv_idle.wait_for(lk, std::chrono::nanoseconds(timeout_ns), [&] { return s->idle(); })) {
        set_error("server_wait_idle: still busy after %lld ns", (long long)timeout_ns);
        return STRAIT_E_BUSY;
    }
    return STRAIT_OK;
}

strait_status strait_server_results(strait_server* s, strait_request_record* out, int32_t capacity, int32_t* n) {
    if (!s || !n || (capacity > 0 && !out) || capacity < 0) { set_error("server_results: bad arguments"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(s->mu);
    int k = 0;
    while (k < capacity && !s->results.empty()) { out[k++] = s->results.front(); s->results.pop_front(); }
    *n = k;
    return STRAIT_OK;
}

strait_status strait_server_get_stats(strait_server* s, strait_server_stats* out) {
    if (!s || !out) { set_error("server_get_stats: null"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(s->mu);
    *out = s->stats;
    return STRAIT_OK;
}

strait_status strait_server_stop(strait_server* s) {
    if (!s) { set_error("server_stop: null"); return STRAIT_E_INVALID; }
    {
        std::lock_guard<std::mutex> lk(s->mu);
        if (!s->running) return STRAIT_OK;
        s->stopping = true;
    }
    s->cv_sched.notify_all();
    s->cv_exec.notify_all();
    if (s->sched_th.joinable()) s->sched_th.join();   // no batch leaves after this
    {
        std::lock_guard<std::mutex> lk(s->mu);
        s->sched_done = true;                         // only now may idle execution threads end
    }
    s->cv_exec.notify_all();
    for (auto& th : s->exec_th) if (th.joinable()) th.join();
    s->exec_th.clear();
    std::lock_guard<std::mutex> lk(s->mu);
    const int64_t t = now_ns();
    for (auto& kv : s->models) {
        for (const Request& r : kv.second.q) s->record(kv.second, r, 3, nullptr, 0, t, 0.0, 0.0);
        kv.second.q.clear();
    }
    s->running = false;
    return STRAIT_OK;
}

strait_status strait_server_destroy(strait_server* s) {
    if (!s) { set_error("server_destroy: null"); return STRAIT_E_INVALID; }
    (void)strait_server_stop(s);
    delete s;
    return STRAIT_OK;
}

// ---- offline profile --------------------------------------------------------------------------------
static double p95(std::vector<double> v) {
    std::sort(v.begin(), v.end());
    size_t rank = (size_t)std::ceil(0.95 * (double)v.size());      // nearest rank
    if (rank < 1) rank = 1;
    return v[rank - 1];
}

strait_status strait_model_profile(strait_model* m, strait_priority prio, int32_t batch, int32_t reps,
                                   strait_batch_profile* out) {
    if (!m || !out || reps < 1) { set_error("model_profile: bad arguments"); return STRAIT_E_INVALID; }
    int32_t arch = 0, n_layers = 0, max_batch = 0, inst = 0, hyper[8] = {0};
    int rc = strait_model_info(m, &arch, &n_layers, &max_batch, &inst, hyper);
    if (rc != STRAIT_OK) return rc;
    size_t in_b = 0, out_b = 0;
    rc = strait_model_io(m, batch, &in_b, &out_b);
    if (rc != STRAIT_OK) return rc;
    void* stage = nullptr;
    size_t cap = 0;
    rc = strait_model_staging(m, 0, &stage, &cap);
    if (rc != STRAIT_OK) return rc;
    memset(stage, 0, in_b);                        // latency of these networks does not depend on the values
    std::vector<char> host_out(out_b);
    std::vector<int32_t> valid(batch, arch == STRAIT_ARCH_ENCODER ? hyper[4] : 0);
    std::vector<double> t_inf, t_h2d, t_ker;
    const int warm = 3;
    for (int i = 0; i < warm + reps; ++i) {
        strait_ticket tk = nullptr;
        rc = strait_submit(m, prio, batch, stage, valid.data(), host_out.data(), &tk);
        if (rc != STRAIT_OK) return rc;
        strait_record rec{};
        rc = strait_wait(tk, &rec);
        if (rc != STRAIT_OK) return rc;
        if (i < warm) continue;
        t_inf.push_back((double)(rec.t_done_ns - rec.t_enqueue_ns));
        t_h2d.push_back((double)rec.h2d_ms * 1e6);
        t_ker.push_back((double)rec.kernel_ms * 1e6);
    }
    *out = strait_batch_profile{};
    out->t_inf_isol_ns = p95(t_inf);
    out->t_htod_ns = (int64_t)p95(t_h2d);
    out->t_kernel_isol_ns = p95(t_ker);
    // demand: algorithmic traffic and work of the kernel sequence over its p95 duration, as fractions of the
    // chip's peaks (256 compute units at 2.4 GHz)
    double hbm = 0, mfma = 0, valu = 0, l2 = 0, lds = 0;
    for (int l = 0; l < n_layers; ++l) {
        strait_layer_info li{};
        rc = strait_model_layer(m, l, &li);
        if (rc != STRAIT_OK) return rc;
        const double act = (double)li.bytes_per_sample * batch, w = (double)li.weight_bytes;
        const double macs = (double)li.macs_per_sample * batch;
        hbm += act + w;
        if (li.kind == 0 || li.kind == 5) {
            mfma += 2.0 * macs;
            if (li.kind == 0 && li.gemm_n > 0) {
                const double M = (double)li.gemm_m_per_sample * batch, N = li.gemm_n, K = li.gemm_k;
                const double operands = 2.0 * (M * K * std::ceil(N / 128.0) + N * K * std::ceil(M / 128.0));
                l2 += operands + 2.0 * M * N;
                lds += 3.0 * operands;
                valu += 2.0 * M * N;
            } else {
                l2 += act + w;
                lds += 3.0 * (act + w);
            }
        } else {
            l2 += act + w;
            valu += (li.kind == 1 ? 2.0 * macs : 0.0) + act / 2.0;
        }
    }
    const double t = out->t_kernel_isol_ns * 1e-9;
    const double cu_clk = 256.0 * 2.4e9;
    if (t > 0) {
        out->m[0] = lds / t / (128.0 * cu_clk);
        out->m[1] = l2 / t / (64.0 * cu_clk);
        out->m[2] = hbm / t / 8.0e12;
        out->m[3] = mfma / t / 2.5e15;
        out->m[4] = valu / t / 157.3e12;
    }
    out->m_self_cmp = out->m[3];
    out->m_self_mem = out->m[1];
    return STRAIT_OK;
}

}  // extern "C"
