// C entry points of the host-to-device link model (paper Section 3.2, "Interference in data transfer":
// Eq. 2, Eq. 3 and the online calibration); the model itself is LinkModel.
#include <mutex>
#include <new>

#include "host_models.hpp"
#include "runtime.hpp"

using namespace strait;
struct strait_link { mutable std::mutex mu; LinkModel m; };

extern "C" {

strait_status strait_link_create(strait_link** out) {
    if (!out) { set_error("link_create: null"); return STRAIT_E_INVALID; }
    *out = new (std::nothrow) strait_link();
    if (!*out) { set_error("out of host memory"); return STRAIT_E_NOMEM; }
    return STRAIT_OK;
}

strait_status strait_link_destroy(strait_link* l) {
    if (!l) { set_error("link_destroy: null"); return STRAIT_E_INVALID; }
    delete l;
    return STRAIT_OK;
}

strait_status strait_link_available(const strait_link* l, int64_t* t_available_ns) {
    if (!l || !t_available_ns) { set_error("link_available: null"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(l->mu);
    *t_available_ns = l->m.available();
    return STRAIT_OK;
}

strait_status strait_link_predict(const strait_link* l, int64_t t_current_ns, int64_t* t_data_ns) {
    if (!l || !t_data_ns) { set_error("link_predict: null"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(l->mu);
    *t_data_ns = l->m.predict(t_current_ns);
    return STRAIT_OK;
}

strait_status strait_link_schedule(strait_link* l, int64_t t_current_ns, int64_t t_htod_ns, uint64_t* transfer_id,
                                   int64_t* t_data_ns) {
    if (!l || !transfer_id) { set_error("link_schedule: null"); return STRAIT_E_INVALID; }
    if (t_htod_ns < 0) { set_error("link_schedule: negative transfer time"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(l->mu);
    *transfer_id = l->m.schedule(t_current_ns, t_htod_ns, t_data_ns);
    return STRAIT_OK;
}

strait_status strait_link_complete(strait_link* l, uint64_t transfer_id, int64_t t_end_ns) {
    if (!l) { set_error("link_complete: null"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(l->mu);
    if (!l->m.complete(transfer_id, t_end_ns)) { set_error("link_complete: unknown transfer %llu", (unsigned long long)transfer_id); return STRAIT_E_INVALID; }
    return STRAIT_OK;
}

}  // extern "C"
