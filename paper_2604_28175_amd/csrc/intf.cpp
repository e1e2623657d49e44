// Kernel-interference predictor (paper Section 3.2, "Interference in kernel execution" and
// "Self-adaptive model"), host side, fp64:
//   Eq. 4   kernel_eff = k * b^LR + C,  LR = w_avg . m_avg + w_cmp * m_self_cmp + w_mem * m_self_mem
//   Eq. 5   Intf = 1 + kernel_eff * coeff_p
//   Eq. 6   T_kernel = (Intf - 1) * T_kernel_isol
// m_avg of a batch is the time-weighted average, over the batch's life, of the summed demands of the
// batches running beside it, re-evaluated at every arrival and departure.  After every completed
// batch the parameters take one Adam step (beta1 0.7, beta2 0.9, alpha 0.0075) on the Huber loss
// (delta 0.5) between the predicted and the measured slowdown.
// Where the paper leaves a choice: LR has no intercept (k absorbs it); a batch that never had a
// neighbour has Intf = 1 and does not train the model; Adam is the published algorithm with bias
// correction and eps 1e-8 over the whole parameter vector; the base b is kept >= 1e-6.
#include <cmath>
#include <cstring>
#include <map>
#include <mutex>
#include <new>

#include "runtime.hpp"

namespace strait {

constexpr int NM = STRAIT_INTF_METRICS;
constexpr int NP = 3 + NM + 2 + 2;            // k, b, C, w_avg[NM], w_cmp, w_mem, coeff_p[2]
constexpr double kBeta1 = 0.7, kBeta2 = 0.9, kAlpha = 0.0075, kEps = 1e-8, kDelta = 0.5, kBMin = 1e-6;

struct Running { double m[NM]; double acc[NM]; int64_t t0; };

struct Intf {
    mutable std::mutex mu;
    double p[NP];
    double mom[NP], var[NP];
    uint64_t steps = 0;
    std::map<uint64_t, Running> running;      // batches on the GPU now
    double total[NM];                          // sum of their demands
    int64_t t_last = 0;
    bool have_t = false;
    uint64_t next_id = 1;

    static bool isolated(const double* m_avg) {
        for (int i = 0; i < NM; ++i) if (m_avg[i] != 0.0) return false;
        return true;
    }
    double lr(const double* m_avg, double sc, double sm) const {
        double s = 0.0;
        for (int i = 0; i < NM; ++i) s += p[3 + i] * m_avg[i];
        return s + p[3 + NM] * sc + p[4 + NM] * sm;
    }
    // every running batch has had the others beside it since t_last
    void advance(int64_t t) {
        if (have_t) {
            const double dt = (double)(t - t_last);
            for (auto& kv : running)
                for (int i = 0; i < NM; ++i) kv.second.acc[i] += (total[i] - kv.second.m[i]) * dt;
        }
        t_last = t;
        have_t = true;
    }
    void recompute_total() {                   // summed afresh so that rounding does not drift
        for (int i = 0; i < NM; ++i) total[i] = 0.0;
        for (auto& kv : running)
            for (int i = 0; i < NM; ++i) total[i] += kv.second.m[i];
    }
};

static void params_to_vec(const strait_intf_params& s, double* p) {
    p[0] = s.k; p[1] = s.b; p[2] = s.C;
    for (int i = 0; i < NM; ++i) p[3 + i] = s.w_avg[i];
    p[3 + NM] = s.w_self_cmp; p[4 + NM] = s.w_self_mem;
    p[5 + NM] = s.coeff_p[0]; p[6 + NM] = s.coeff_p[1];
}
static void vec_to_params(const double* p, strait_intf_params* s) {
    s->k = p[0]; s->b = p[1]; s->C = p[2];
    for (int i = 0; i < NM; ++i) s->w_avg[i] = p[3 + i];
    s->w_self_cmp = p[3 + NM]; s->w_self_mem = p[4 + NM];
    s->coeff_p[0] = p[5 + NM]; s->coeff_p[1] = p[6 + NM];
}

}  // namespace strait

using namespace strait;
struct strait_intf : Intf {};

static bool bad_prio(int32_t prio) { return prio != STRAIT_PRIO_HIGH && prio != STRAIT_PRIO_LOW; }

extern "C" {

strait_status strait_intf_create(const strait_intf_params* init, strait_intf** out) {
    if (!out) { set_error("intf_create: null"); return STRAIT_E_INVALID; }
    strait_intf_params d;
    if (init) d = *init;
    else {                                     // conservative start: zero pressure -> no slowdown, every metric counts
        d.k = 1.0; d.b = 2.0; d.C = -1.0;
        for (int i = 0; i < NM; ++i) d.w_avg[i] = 0.5;
        d.w_self_cmp = d.w_self_mem = 0.0;
        d.coeff_p[0] = d.coeff_p[1] = 1.0;
    }
    if (!(d.b >= kBMin)) { set_error("intf_create: base b must be >= 1e-6"); return STRAIT_E_INVALID; }
    strait_intf* o = new (std::nothrow) strait_intf();
    if (!o) { set_error("out of host memory"); return STRAIT_E_NOMEM; }
    params_to_vec(d, o->p);
    std::memset(o->mom, 0, sizeof o->mom);
    std::memset(o->var, 0, sizeof o->var);
    std::memset(o->total, 0, sizeof o->total);
    *out = o;
    return STRAIT_OK;
}

strait_status strait_intf_destroy(strait_intf* o) {
    if (!o) { set_error("intf_destroy: null"); return STRAIT_E_INVALID; }
    delete o;
    return STRAIT_OK;
}

strait_status strait_intf_get_params(const strait_intf* o, strait_intf_params* out) {
    if (!o || !out) { set_error("intf_get_params: null"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(o->mu);
    vec_to_params(o->p, out);
    return STRAIT_OK;
}

strait_status strait_intf_demand(const double* v, const double* d, int32_t n, double* m_out) {
    if (!v || !d || !m_out || n < 1) { set_error("intf_demand: bad arguments"); return STRAIT_E_INVALID; }
    double acc[NM] = {0}, dsum = 0.0;
    for (int j = 0; j < n; ++j) {
        if (!(d[j] >= 0.0)) { set_error("intf_demand: negative duration"); return STRAIT_E_INVALID; }
        for (int i = 0; i < NM; ++i) acc[i] += v[(size_t)j * NM + i] * d[j];
        dsum += d[j];
    }
    if (!(dsum > 0.0)) { set_error("intf_demand: zero total duration"); return STRAIT_E_INVALID; }
    for (int i = 0; i < NM; ++i) m_out[i] = acc[i] / dsum;
    return STRAIT_OK;
}

strait_status strait_intf_predict(const strait_intf* o, const double* m_avg, double self_cmp, double self_mem,
                                  int32_t prio, double t_kernel_isol, double* intf_hat, double* t_kernel) {
    if (!o || !m_avg || bad_prio(prio) || (!intf_hat && !t_kernel)) { set_error("intf_predict: bad arguments"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(o->mu);
    double intf = 1.0;
    if (!Intf::isolated(m_avg)) {
        const double eff = o->p[0] * std::pow(o->p[1], o->lr(m_avg, self_cmp, self_mem)) + o->p[2];   // Eq. 4
        intf = 1.0 + eff * o->p[5 + NM + prio];                                                        // Eq. 5
    }
    if (intf_hat) *intf_hat = intf;
    if (t_kernel) *t_kernel = (intf - 1.0) * t_kernel_isol;                                            // Eq. 6
    return STRAIT_OK;
}

strait_status strait_intf_update(strait_intf* o, const double* m_avg, double self_cmp, double self_mem, int32_t prio,
                                 double intf_actual, double* loss_out) {
    if (!o || !m_avg || bad_prio(prio) || !std::isfinite(intf_actual)) { set_error("intf_update: bad arguments"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(o->mu);
    if (loss_out) *loss_out = 0.0;
    if (Intf::isolated(m_avg)) return STRAIT_OK;
    double* p = o->p;
    const double k = p[0], b = p[1];
    const double lr = o->lr(m_avg, self_cmp, self_mem);
    const double pw = std::pow(b, lr);
    const double coeff = p[5 + NM + prio];
    const double eff = k * pw + p[2];
    const double e = 1.0 + eff * coeff - intf_actual;
    const double ae = std::fabs(e);
    const double dl = ae <= kDelta ? e : (e > 0 ? kDelta : -kDelta);        // derivative of the Huber loss
    if (loss_out) *loss_out = ae <= kDelta ? 0.5 * e * e : kDelta * (ae - 0.5 * kDelta);
    double g[NP] = {0};
    g[0] = pw * coeff;
    g[1] = k * lr * std::pow(b, lr - 1.0) * coeff;
    g[2] = coeff;
    const double dlr = k * pw * std::log(b) * coeff;
    for (int i = 0; i < NM; ++i) g[3 + i] = dlr * m_avg[i];
    g[3 + NM] = dlr * self_cmp;
    g[4 + NM] = dlr * self_mem;
    g[5 + NM + prio] = eff;
    o->steps += 1;
    const double c1 = 1.0 - std::pow(kBeta1, (double)o->steps), c2 = 1.0 - std::pow(kBeta2, (double)o->steps);
    for (int i = 0; i < NP; ++i) {
        const double gi = dl * g[i];
        o->mom[i] = kBeta1 * o->mom[i] + (1.0 - kBeta1) * gi;
        o->var[i] = kBeta2 * o->var[i] + (1.0 - kBeta2) * gi * gi;
        p[i] -= kAlpha * (o->mom[i] / c1) / (std::sqrt(o->var[i] / c2) + kEps);
    }
    if (!(p[1] >= kBMin)) p[1] = kBMin;
    return STRAIT_OK;
}

strait_status strait_intf_arrive(strait_intf* o, int64_t t_ns, const double* m, uint64_t* batch_id) {
    if (!o || !m || !batch_id) { set_error("intf_arrive: null"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(o->mu);
    if (o->have_t && t_ns < o->t_last) { set_error("intf_arrive: time runs backwards"); return STRAIT_E_INVALID; }
    o->advance(t_ns);
    Running r;
    for (int i = 0; i < NM; ++i) { r.m[i] = m[i]; r.acc[i] = 0.0; }
    r.t0 = t_ns;
    *batch_id = o->next_id++;
    o->running.emplace(*batch_id, r);
    o->recompute_total();
    return STRAIT_OK;
}

strait_status strait_intf_depart(strait_intf* o, uint64_t batch_id, int64_t t_ns, double* m_avg_out) {
    if (!o || !m_avg_out) { set_error("intf_depart: null"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(o->mu);
    auto it = o->running.find(batch_id);
    if (it == o->running.end()) { set_error("intf_depart: unknown batch id"); return STRAIT_E_INVALID; }
    if (t_ns < o->t_last) { set_error("intf_depart: time runs backwards"); return STRAIT_E_INVALID; }
    o->advance(t_ns);
    const double life = (double)(t_ns - it->second.t0);
    for (int i = 0; i < NM; ++i) m_avg_out[i] = life > 0.0 ? it->second.acc[i] / life : 0.0;
    o->running.erase(it);
    o->recompute_total();
    return STRAIT_OK;
}

strait_status strait_intf_pressure(const strait_intf* o, uint64_t exclude_id, double* m_now) {
    if (!o || !m_now) { set_error("intf_pressure: null"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(o->mu);
    for (int i = 0; i < NM; ++i) m_now[i] = 0.0;
    for (const auto& kv : o->running)
        if (kv.first != exclude_id)
            for (int i = 0; i < NM; ++i) m_now[i] += kv.second.m[i];
    return STRAIT_OK;
}

}  // extern "C"
