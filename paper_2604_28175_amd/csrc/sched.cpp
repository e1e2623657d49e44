// Scheduling policy (paper Section 3.3, Algorithm 1) on top of the latency estimate of Eq. 1,
//     T_inf(B_ik) = T_inf_isol(B_ik) + T_data + T_kernel(B_ik) + T_queue,
// with T_data from the link model (Eq. 2-3) and T_kernel from the interference model (Eq. 4-6).
// One decision serves one model's queue: early dropping, binary search for the largest batch size that
// some GPU can take without violate() and with meet(), the GPU of lowest estimated latency gets it.
// Where the paper leaves a choice: a batch's peak throughput is the largest of its five demand metrics;
// a running batch's kernel time counts from submission + T_data + its isolated transfer time; C_low is
// one value per scheduler; the search probes mid = (lo + hi + 1) / 2 starting from lo = 1, hi = limit.
#include <map>
#include <mutex>
#include <new>
#include <vector>

#include "host_models.hpp"
#include "runtime.hpp"

namespace strait {

constexpr int NM = IntfModel::NM;
constexpr double kCLowMin = 0.75, kCLowMax = 1.00, kCLowStep = 0.0025;
constexpr int64_t kCLowPeriodNs = 100000000;

struct Profile { strait_batch_profile p; double peak; };
struct ModelProfiles { int prio; std::vector<Profile> by_batch; };
struct RunRec { int prio; const Profile* prof; int64_t t0, deadline, t_kernel_start; uint64_t link_id; };

struct Sched {
    std::mutex mu;
    IntfModel intf;                                   // parameters + learning state (tracker part unused)
    std::vector<LinkModel> links;
    std::vector<IntfModel> track;                     // per GPU: who runs beside whom
    std::vector<std::map<uint64_t, RunRec>> running;  // per GPU, keyed by tracker id
    std::map<int, ModelProfiles> models;
    double c_low = kCLowMin;
    int64_t t_aimd = 0;
    bool have_aimd = false;

    void tick(int64_t now) {
        if (!have_aimd) { t_aimd = now; have_aimd = true; }
        const int64_t steps = (now - t_aimd) / kCLowPeriodNs;
        if (steps > 0) {
            c_low += (double)steps * kCLowStep;
            if (c_low > kCLowMax) c_low = kCLowMax;
            t_aimd += steps * kCLowPeriodNs;
        }
    }
    bool violate(int g, int prio, const Profile& np, int64_t now) const {
        if (prio == STRAIT_PRIO_LOW) {
            double lp = 0.0;
            for (const auto& kv : running[g]) if (kv.second.prio == STRAIT_PRIO_LOW) lp += kv.second.prof->peak;
            if (lp + np.peak > c_low) return true;
        }
        for (const auto& kv : running[g]) {
            const RunRec& r = kv.second;
            if (r.prio > prio) continue;              // lower priority than the new batch: it may be hurt
            const strait_batch_profile& rp = r.prof->p;
            const double elapsed = now > r.t_kernel_start ? (double)(now - r.t_kernel_start) : 0.0;
            double m_sofar[NM], m_new[NM];
            track[g].pressure_so_far(kv.first, now, m_sofar);
            const double intf_sofar = intf.predict(m_sofar, rp.m_self_cmp, rp.m_self_mem, r.prio);
            double done = 1.0;
            if (rp.t_kernel_isol_ns > 0) { done = elapsed / (intf_sofar * rp.t_kernel_isol_ns); if (done > 1.0) done = 1.0; }
            track[g].pressure(kv.first, m_new);
            for (int i = 0; i < NM; ++i) m_new[i] += np.p.m[i];
            const double intf_new = intf.predict(m_new, rp.m_self_cmp, rp.m_self_mem, r.prio);
            const double start = (double)(now > r.t_kernel_start ? now : r.t_kernel_start);
            if (start + (1.0 - done) * rp.t_kernel_isol_ns * intf_new > (double)r.deadline) return true;
        }
        return false;
    }
    // Eq. 1 for a candidate batch.  Its co-located pressure over its coming life is unknown at scheduling time; the
    // paper's meet() (Section 3.3) settles it by judging the batch "under half of that GPU's runtime throughput", so
    // Eq. 4 is fed half of the summed demand of the batches running on the GPU now.  (violate() is different on
    // purpose: for batches already running it uses the full pressure with the candidate added.)
    double t_inf(int g, int prio, const Profile& np, int64_t now, int64_t t_queue) const {
        const int64_t t_data = links[g].predict(now);
        double half[NM];
        track[g].pressure(0, half);
        for (int i = 0; i < NM; ++i) half[i] *= 0.5;
        const double t_kernel = (intf.predict(half, np.p.m_self_cmp, np.p.m_self_mem, prio) - 1.0) * np.p.t_kernel_isol_ns;   // Eq. 6
        return np.p.t_inf_isol_ns + (double)t_data + t_kernel + (double)t_queue;                                                // Eq. 1
    }
};

}  // namespace strait

using namespace strait;
struct strait_sched : Sched {};

extern "C" {

strait_status strait_sched_create(int32_t n_gpus, const strait_intf_params* init, strait_sched** out) {
    if (!out || n_gpus < 1 || n_gpus > 64) { set_error("sched_create: bad arguments"); return STRAIT_E_INVALID; }
    strait_intf_params d;
    if (init) d = *init; else IntfModel::conservative(&d);
    if (!(d.b >= IntfModel::kBMin)) { set_error("sched_create: base b must be >= 1e-6"); return STRAIT_E_INVALID; }
    strait_sched* s = new (std::nothrow) strait_sched();
    if (!s) { set_error("out of host memory"); return STRAIT_E_NOMEM; }
    s->intf.set_params(d);
    s->links.resize(n_gpus);
    s->track.resize(n_gpus);
    s->running.resize(n_gpus);
    *out = s;
    return STRAIT_OK;
}

strait_status strait_sched_destroy(strait_sched* s) {
    if (!s) { set_error("sched_destroy: null"); return STRAIT_E_INVALID; }
    delete s;
    return STRAIT_OK;
}

strait_status strait_sched_set_profile(strait_sched* s, int32_t model_id, int32_t priority, const strait_batch_profile* table,
                                       int32_t max_batch) {
    if (!s || !table || max_batch < 1 || (priority != STRAIT_PRIO_HIGH && priority != STRAIT_PRIO_LOW)) { set_error("sched_set_profile: bad arguments"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(s->mu);
    for (const auto& g : s->running)
        for (const auto& kv : g)
            if (s->models.count(model_id) && kv.second.prof >= s->models[model_id].by_batch.data() &&
                kv.second.prof < s->models[model_id].by_batch.data() + s->models[model_id].by_batch.size()) {
                set_error("sched_set_profile: model %d has batches running", model_id); return STRAIT_E_BUSY;
            }
    ModelProfiles mp;
    mp.prio = priority;
    for (int b = 0; b < max_batch; ++b) {
        const strait_batch_profile& t = table[b];
        if (!(t.t_inf_isol_ns >= 0) || t.t_htod_ns < 0 || !(t.t_kernel_isol_ns >= 0)) { set_error("sched_set_profile: negative latency at batch %d", b + 1); return STRAIT_E_INVALID; }
        Profile pr{t, t.m[0]};
        for (int i = 1; i < NM; ++i) if (t.m[i] > pr.peak) pr.peak = t.m[i];
        mp.by_batch.push_back(pr);
    }
    s->models[model_id] = std::move(mp);
    return STRAIT_OK;
}

strait_status strait_sched_tick(strait_sched* s, int64_t now_ns, double* c_low) {
    if (!s) { set_error("sched_tick: null"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(s->mu);
    s->tick(now_ns);
    if (c_low) *c_low = s->c_low;
    return STRAIT_OK;
}

strait_status strait_sched_decide(strait_sched* s, int32_t model_id, int64_t now_ns, const int64_t* enqueue_ns,
                                  const int64_t* deadline_ns, int32_t n_requests, strait_decision* out) {
    if (!s || !out || n_requests < 0 || (n_requests > 0 && (!enqueue_ns || !deadline_ns))) { set_error("sched_decide: bad arguments"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(s->mu);
    auto mit = s->models.find(model_id);
    if (mit == s->models.end()) { set_error("sched_decide: model %d has no profile", model_id); return STRAIT_E_INVALID; }
    for (const IntfModel& t : s->track) if (!t.time_ok(now_ns)) { set_error("sched_decide: time runs backwards"); return STRAIT_E_INVALID; }
    const ModelProfiles& mp = mit->second;
    const int prio = mp.prio;
    s->tick(now_ns);
    int dropped = 0;                                   // early dropping: could not finish even alone
    while (dropped < n_requests && (double)(deadline_ns[dropped] - now_ns) < mp.by_batch[0].p.t_inf_isol_ns) ++dropped;
    *out = strait_decision{};
    out->n_dropped = dropped;
    out->gpu = -1;
    const int avail = n_requests - dropped;
    const int limit = avail < (int)mp.by_batch.size() ? avail : (int)mp.by_batch.size();
    if (limit == 0) return STRAIT_OK;
    const int64_t t_front = enqueue_ns[dropped], d_front = deadline_ns[dropped];
    const int64_t t_queue = now_ns - t_front;
    const int ng = (int)s->links.size();
    auto feasible = [&](int k, std::vector<int>& gpus) {
        gpus.clear();
        const Profile& np = mp.by_batch[k - 1];
        for (int g = 0; g < ng; ++g)
            if (!s->violate(g, prio, np, now_ns) && (double)t_front + s->t_inf(g, prio, np, now_ns, t_queue) <= (double)d_front) gpus.push_back(g);
        return !gpus.empty();
    };
    int best = 0, lo = 1, hi = limit;
    std::vector<int> gpus, best_gpus;
    while (lo <= hi) {
        const int mid = (lo + hi + 1) / 2;
        if (feasible(mid, gpus)) { best = mid; best_gpus = gpus; lo = mid + 1; } else hi = mid - 1;
    }
    if (best == 0) return STRAIT_OK;                   // deferred: no GPU can take even the smallest probe
    const Profile& np = mp.by_batch[best - 1];
    int g_best = -1;
    double lat_best = 0.0;
    for (int g : best_gpus) {
        const double lat = s->t_inf(g, prio, np, now_ns, t_queue);
        if (g_best < 0 || lat < lat_best) { g_best = g; lat_best = lat; }
    }
    int64_t t_data = 0;
    const uint64_t link_id = s->links[g_best].schedule(now_ns, np.p.t_htod_ns, &t_data);
    const uint64_t rid = s->track[g_best].arrive(now_ns, np.p.m);
    s->running[g_best][rid] = RunRec{prio, &np, now_ns, d_front, now_ns + t_data + np.p.t_htod_ns, link_id};
    out->batch = best;
    out->gpu = g_best;
    out->t_inf_ns = lat_best;
    out->t_data_ns = t_data;
    out->running_id = rid;
    return STRAIT_OK;
}

strait_status strait_sched_complete(strait_sched* s, int32_t gpu, uint64_t running_id, int64_t now_ns, double kernel_ns,
                                    int64_t h2d_end_ns, strait_completion* out) {
    if (!s || gpu < 0) { set_error("sched_complete: bad arguments"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(s->mu);
    if (gpu >= (int)s->links.size()) { set_error("sched_complete: no GPU %d", gpu); return STRAIT_E_INVALID; }
    auto it = s->running[gpu].find(running_id);
    if (it == s->running[gpu].end()) { set_error("sched_complete: unknown batch"); return STRAIT_E_INVALID; }
    if (!s->track[gpu].time_ok(now_ns)) { set_error("sched_complete: time runs backwards"); return STRAIT_E_INVALID; }
    const RunRec r = it->second;
    s->running[gpu].erase(it);
    double m_avg[NM];
    s->track[gpu].depart(running_id, now_ns, m_avg);
    if (h2d_end_ns >= 0) (void)s->links[gpu].complete(r.link_id, h2d_end_ns);   // older than a calibrated transfer: nothing to add
    const strait_batch_profile& rp = r.prof->p;
    double loss = 0.0;
    if (rp.t_kernel_isol_ns > 0 && std::isfinite(kernel_ns)) loss = s->intf.update(m_avg, rp.m_self_cmp, rp.m_self_mem, r.prio, kernel_ns / rp.t_kernel_isol_ns);
    const bool violated = now_ns > r.deadline;
    if (violated && r.prio == STRAIT_PRIO_HIGH) { s->c_low = kCLowMin; s->t_aimd = now_ns; s->have_aimd = true; }
    if (out) {
        out->violated = violated ? 1 : 0;
        out->loss = loss;
        for (int i = 0; i < NM; ++i) out->m_avg[i] = m_avg[i];
        out->c_low = s->c_low;
    }
    return STRAIT_OK;
}

strait_status strait_sched_get_params(strait_sched* s, strait_intf_params* out) {
    if (!s || !out) { set_error("sched_get_params: null"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(s->mu);
    s->intf.get_params(out);
    return STRAIT_OK;
}

}  // extern "C"
