// Host-to-device link model (paper Section 3.2, "Interference in data transfer"):
//   Eq. 2   T_data = max(0, t_available - t_current)
//   Eq. 3   t_available <- max(t_current, t_available) + t_HtoD(i,j)
// and the online calibration of the same section: once a transfer has been timed, its measured end
// replaces the estimate, and the recurrence of Eq. 3 is carried forward from there over the
// transfers scheduled after it (pinned transfers are served first-in first-out).
#include <deque>
#include <mutex>
#include <new>

#include "runtime.hpp"

namespace strait {

struct Transfer { uint64_t id; int64_t t_sched, t_htod, t_end; bool measured; };

struct Link {
    mutable std::mutex mu;
    std::deque<Transfer> pending;     // in schedule order; entries before the newest measured one are dropped
    int64_t base = INT64_MIN;         // link-free time implied by everything already dropped
    uint64_t next_id = 1;

    // fold Eq. 3 over the pending transfers (measured ends override the estimate)
    int64_t available_locked() const {
        int64_t a = base;
        for (const Transfer& t : pending) a = t.measured ? t.t_end : (t.t_sched > a ? t.t_sched : a) + t.t_htod;
        return a;
    }
};

}  // namespace strait

using namespace strait;
struct strait_link : Link {};

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
    *t_available_ns = l->available_locked();
    return STRAIT_OK;
}

strait_status strait_link_predict(const strait_link* l, int64_t t_current_ns, int64_t* t_data_ns) {
    if (!l || !t_data_ns) { set_error("link_predict: null"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(l->mu);
    const int64_t a = l->available_locked();
    *t_data_ns = a > t_current_ns ? a - t_current_ns : 0;
    return STRAIT_OK;
}

strait_status strait_link_schedule(strait_link* l, int64_t t_current_ns, int64_t t_htod_ns, uint64_t* transfer_id,
                                   int64_t* t_data_ns) {
    if (!l || !transfer_id) { set_error("link_schedule: null"); return STRAIT_E_INVALID; }
    if (t_htod_ns < 0) { set_error("link_schedule: negative transfer time"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(l->mu);
    const int64_t a = l->available_locked();
    if (t_data_ns) *t_data_ns = a > t_current_ns ? a - t_current_ns : 0;
    Transfer t{l->next_id++, t_current_ns, t_htod_ns, 0, false};
    l->pending.push_back(t);
    *transfer_id = t.id;
    return STRAIT_OK;
}

strait_status strait_link_complete(strait_link* l, uint64_t transfer_id, int64_t t_end_ns) {
    if (!l) { set_error("link_complete: null"); return STRAIT_E_INVALID; }
    std::lock_guard<std::mutex> lk(l->mu);
    size_t idx = l->pending.size();
    for (size_t i = 0; i < l->pending.size(); ++i)
        if (l->pending[i].id == transfer_id) { idx = i; break; }
    if (idx == l->pending.size()) { set_error("link_complete: unknown transfer %llu", (unsigned long long)transfer_id); return STRAIT_E_INVALID; }
    l->pending[idx].measured = true;
    l->pending[idx].t_end = t_end_ns;
    // everything up to the newest measured transfer is history: fold it into `base`
    size_t last = 0;
    bool any = false;
    for (size_t i = 0; i < l->pending.size(); ++i)
        if (l->pending[i].measured) { last = i; any = true; }
    if (any) {
        l->base = l->pending[last].t_end;
        l->pending.erase(l->pending.begin(), l->pending.begin() + (long)last + 1);
    }
    return STRAIT_OK;
}

}  // extern "C"
