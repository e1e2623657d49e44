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
#include <mutex>
#include <new>

#include "host_models.hpp"
#include "runtime.hpp"

using namespace strait;
struct strait_intf { mutable std::mutex mu; IntfModel m; };
static constexpr int NM = IntfModel::NM;

static bool bad_prio(int32_t prio) { return prio != STRAIT_PRIO_HIGH && prio != STRAIT_PRIO_LOW; }

extern "C" {

strait_status strait_intf_create(const strait_intf_params* init, strait_intf** out) {
    if (!out) { set_error("intf_create: null"); return STRAIT_E_INVALID; }
    strait_intf_params d;
    if (init) d = *init; else IntfModel::conservative(&d);
    if (!(d.b >= IntfModel::kBMin)) { set_error("intf_create: base b must be >= 1e-6"); return STRAIT_E_INVALID; }
    strait_intf* o = new (std::nothrow) strait_intf();
    if (!o) { set_error("out of host memory"); return STRAIT_E_NOMEM; }
    o->m.set_params(d);
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
    o->m.get_params(out);
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
    const double intf = o->m.predict(m_avg, self_cmp, self_mem, prio);
    if (intf_hat) *intf_hat = intf;
    if (t_kernel) *t_kernel = (intf - 1.0) * t_kernel_isol;                                            // Eq. 6
    return STRAIT_OK;
}

strait_status strait_intf_update(strait_intf* o, const double* m_avg, double self_cmp, double self_mem, int32_t prio,
                                 double intf_actual, double* loss_out) {
    if (!o || !m_avg || bad_prio(prio) || !std::isfinite(intf_actual)) { set_error("intf_update: bad arguments"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(o->mu);
    const double loss = o->m.update(m_avg, self_cmp, self_mem, prio, intf_actual);
    if (loss_out) *loss_out = loss;
    return STRAIT_OK;
}

strait_status strait_intf_arrive(strait_intf* o, int64_t t_ns, const double* m, uint64_t* batch_id) {
    if (!o || !m || !batch_id) { set_error("intf_arrive: null"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(o->mu);
    if (!o->m.time_ok(t_ns)) { set_error("intf_arrive: time runs backwards"); return STRAIT_E_INVALID; }
    *batch_id = o->m.arrive(t_ns, m);
    return STRAIT_OK;
}

strait_status strait_intf_depart(strait_intf* o, uint64_t batch_id, int64_t t_ns, double* m_avg_out) {
    if (!o || !m_avg_out) { set_error("intf_depart: null"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(o->mu);
    if (!o->m.known(batch_id)) { set_error("intf_depart: unknown batch id"); return STRAIT_E_INVALID; }
    if (!o->m.time_ok(t_ns)) { set_error("intf_depart: time runs backwards"); return STRAIT_E_INVALID; }
    o->m.depart(batch_id, t_ns, m_avg_out);
    return STRAIT_OK;
}

strait_status strait_intf_pressure(const strait_intf* o, uint64_t exclude_id, double* m_now) {
    if (!o || !m_now) { set_error("intf_pressure: null"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(o->mu);
    o->m.pressure(exclude_id, m_now);
    return STRAIT_OK;
}

}  // extern "C"
