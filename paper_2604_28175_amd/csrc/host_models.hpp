// Host-side models shared by the C entry points and the scheduler: the first-in first-out link model
// (paper Eq. 2-3 with online calibration) and the kernel-interference predictor (Eq. 4-6 with its
// co-location tracker and Adam/Huber online step).  Plain classes without locking: the owners lock.
#pragma once
#include <cmath>
#include <cstdint>
#include <cstring>
#include <deque>
#include <map>

#include "../../include/strait.h"

namespace strait {

// ---- Eq. 2-3 ---------------------------------------------------------------------------------------
class LinkModel {
public:
    // fold Eq. 3 over the pending transfers (measured ends override the estimate)
    int64_t available() const {
        int64_t a = base_;
        for (const Transfer& t : pending_) a = t.measured ? t.t_end : (t.t_sched > a ? t.t_sched : a) + t.t_htod;
        return a;
    }
    int64_t predict(int64_t t_current) const {                       // Eq. 2
        const int64_t a = available();
        return a > t_current ? a - t_current : 0;
    }
    uint64_t schedule(int64_t t_current, int64_t t_htod, int64_t* t_data) {   // Eq. 2, then Eq. 3
        if (t_data) *t_data = predict(t_current);
        Transfer t{next_id_++, t_current, t_htod, 0, false};
        pending_.push_back(t);
        return t.id;
    }
    // online calibration; false for an id that is unknown or older than an already measured transfer
    bool complete(uint64_t id, int64_t t_end) {
        size_t idx = pending_.size();
        for (size_t i = 0; i < pending_.size(); ++i)
            if (pending_[i].id == id) { idx = i; break; }
        if (idx == pending_.size()) return false;
        pending_[idx].measured = true;
        pending_[idx].t_end = t_end;
        // everything up to the newest measured transfer is history: fold it into the base
        size_t last = 0;
        for (size_t i = 0; i < pending_.size(); ++i)
            if (pending_[i].measured) last = i;
        base_ = pending_[last].t_end;
        pending_.erase(pending_.begin(), pending_.begin() + (long)last + 1);
        return true;
    }

private:
    struct Transfer { uint64_t id; int64_t t_sched, t_htod, t_end; bool measured; };
    std::deque<Transfer> pending_;    // in schedule order; entries up to the newest measured one are dropped
    int64_t base_ = INT64_MIN;        // link-free time implied by everything already dropped
    uint64_t next_id_ = 1;
};

// ---- Eq. 4-6, co-location dynamics, online step -------------------------------------------------------
class IntfModel {
public:
    static constexpr int NM = STRAIT_INTF_METRICS;
    static constexpr int NP = 3 + NM + 2 + 2;            // k, b, C, w_avg[NM], w_cmp, w_mem, coeff_p[2]
    static constexpr double kBeta1 = 0.7, kBeta2 = 0.9, kAlpha = 0.0075, kEps = 1e-8, kDelta = 0.5, kBMin = 1e-6;

    double p[NP];

    IntfModel() {
        std::memset(mom_, 0, sizeof mom_);
        std::memset(var_, 0, sizeof var_);
        std::memset(total_, 0, sizeof total_);
        std::memset(p, 0, sizeof p);
    }
    void set_params(const strait_intf_params& s) {
        p[0] = s.k; p[1] = s.b; p[2] = s.C;
        for (int i = 0; i < NM; ++i) p[3 + i] = s.w_avg[i];
        p[3 + NM] = s.w_self_cmp; p[4 + NM] = s.w_self_mem;
        p[5 + NM] = s.coeff_p[0]; p[6 + NM] = s.coeff_p[1];
    }
    void get_params(strait_intf_params* s) const {
        s->k = p[0]; s->b = p[1]; s->C = p[2];
        for (int i = 0; i < NM; ++i) s->w_avg[i] = p[3 + i];
        s->w_self_cmp = p[3 + NM]; s->w_self_mem = p[4 + NM];
        s->coeff_p[0] = p[5 + NM]; s->coeff_p[1] = p[6 + NM];
    }
    static void conservative(strait_intf_params* d) {   // zero pressure -> no slowdown, every metric counts
        d->k = 1.0; d->b = 2.0; d->C = -1.0;
        for (int i = 0; i < NM; ++i) d->w_avg[i] = 0.5;
        d->w_self_cmp = d->w_self_mem = 0.0;
        d->coeff_p[0] = d->coeff_p[1] = 1.0;
    }
    static bool isolated(const double* m_avg) {
        for (int i = 0; i < NM; ++i) if (m_avg[i] != 0.0) return false;
        return true;
    }
    double lr(const double* m_avg, double sc, double sm) const {
        double s = 0.0;
        for (int i = 0; i < NM; ++i) s += p[3 + i] * m_avg[i];
        return s + p[3 + NM] * sc + p[4 + NM] * sm;
    }
    double predict(const double* m_avg, double sc, double sm, int prio) const {
        if (isolated(m_avg)) return 1.0;
        const double eff = p[0] * std::pow(p[1], lr(m_avg, sc, sm)) + p[2];      // Eq. 4
        return 1.0 + eff * p[5 + NM + prio];                                     // Eq. 5
    }
    // one Adam step on the Huber loss of (predicted - actual); returns the loss before the step
    double update(const double* m_avg, double sc, double sm, int prio, double intf_actual) {
        if (isolated(m_avg)) return 0.0;
        const double k = p[0], b = p[1];
        const double l = lr(m_avg, sc, sm);
        const double pw = std::pow(b, l);
        const double coeff = p[5 + NM + prio];
        const double eff = k * pw + p[2];
        const double e = 1.0 + eff * coeff - intf_actual;
        const double ae = std::fabs(e);
        const double dl = ae <= kDelta ? e : (e > 0 ? kDelta : -kDelta);          // derivative of the Huber loss
        const double loss = ae <= kDelta ? 0.5 * e * e : kDelta * (ae - 0.5 * kDelta);
        double g[NP] = {0};
        g[0] = pw * coeff;
        g[1] = k * l * std::pow(b, l - 1.0) * coeff;
        g[2] = coeff;
        const double dlr = k * pw * std::log(b) * coeff;
        for (int i = 0; i < NM; ++i) g[3 + i] = dlr * m_avg[i];
        g[3 + NM] = dlr * sc;
        g[4 + NM] = dlr * sm;
        g[5 + NM + prio] = eff;
        steps_ += 1;
        const double c1 = 1.0 - std::pow(kBeta1, (double)steps_), c2 = 1.0 - std::pow(kBeta2, (double)steps_);
        for (int i = 0; i < NP; ++i) {
            const double gi = dl * g[i];
            mom_[i] = kBeta1 * mom_[i] + (1.0 - kBeta1) * gi;
            var_[i] = kBeta2 * var_[i] + (1.0 - kBeta2) * gi * gi;
            p[i] -= kAlpha * (mom_[i] / c1) / (std::sqrt(var_[i] / c2) + kEps);
        }
        if (!(p[1] >= kBMin)) p[1] = kBMin;
        return loss;
    }

    // ---- who runs beside whom ---------------------------------------------------------------------
    bool time_ok(int64_t t) const { return !have_t_ || t >= t_last_; }
    uint64_t arrive(int64_t t, const double* m) {
        advance(t);
        Running r;
        for (int i = 0; i < NM; ++i) { r.m[i] = m[i]; r.acc[i] = 0.0; }
        r.t0 = t;
        const uint64_t id = next_id_++;
        running_.emplace(id, r);
        recompute_total();
        return id;
    }
    bool known(uint64_t id) const { return running_.count(id) != 0; }
    void depart(uint64_t id, int64_t t, double* m_avg_out) {
        advance(t);
        auto it = running_.find(id);
        const double life = (double)(t - it->second.t0);
        for (int i = 0; i < NM; ++i) m_avg_out[i] = life > 0.0 ? it->second.acc[i] / life : 0.0;
        running_.erase(it);
        recompute_total();
    }
    void pressure(uint64_t exclude, double* m_now) const {
        for (int i = 0; i < NM; ++i) m_now[i] = 0.0;
        for (const auto& kv : running_)
            if (kv.first != exclude)
                for (int i = 0; i < NM; ++i) m_now[i] += kv.second.m[i];
    }
    // time-weighted pressure on batch `id` from its start up to `now` (no state change)
    void pressure_so_far(uint64_t id, int64_t now, double* m_out) const {
        const Running& r = running_.at(id);
        double others[NM];
        pressure(id, others);
        const double dt = have_t_ ? (double)(now - t_last_) : 0.0;
        const double life = (double)(now - r.t0);
        for (int i = 0; i < NM; ++i) m_out[i] = life > 0.0 ? (r.acc[i] + others[i] * dt) / life : 0.0;
    }

private:
    struct Running { double m[NM]; double acc[NM]; int64_t t0; };
    // every running batch has had the others beside it since t_last
    void advance(int64_t t) {
        if (have_t_) {
            const double dt = (double)(t - t_last_);
            for (auto& kv : running_)
                for (int i = 0; i < NM; ++i) kv.second.acc[i] += (total_[i] - kv.second.m[i]) * dt;
        }
        t_last_ = t;
        have_t_ = true;
    }
    void recompute_total() {                   // summed afresh so that rounding does not drift
        for (int i = 0; i < NM; ++i) total_[i] = 0.0;
        for (auto& kv : running_)
            for (int i = 0; i < NM; ++i) total_[i] += kv.second.m[i];
    }
    double mom_[NP], var_[NP];
    uint64_t steps_ = 0;
    std::map<uint64_t, Running> running_;
    double total_[NM];
    int64_t t_last_ = 0;
    bool have_t_ = false;
    uint64_t next_id_ = 1;
};

}  // namespace strait
