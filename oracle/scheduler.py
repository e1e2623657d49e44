"""CPU oracle of the scheduling policy.  TEST INFRASTRUCTURE ONLY.

Section 3.3 of the paper (Algorithm 1, "Priority-aware Scheduling") on top of Eq. 1:
    T_inf(B_ik) = T_inf_isol(B_ik) + T_data + T_kernel(B_ik) + T_queue
with T_data from the link oracle (Eq. 2-3) and T_kernel from the interference oracle (Eq. 4-6).

One decision, for the queue of model i holding j requests (oldest first), at time `now`:
  1. early dropping: requests whose remaining time is shorter than the isolated latency of a batch of
     one are removed (they could not finish even alone);
  2. binary search for the largest batch size k in 1..min(j, max_batch) for which some GPU satisfies
     not violate(...) and meet(...); the batch takes the k oldest requests, its deadline is the front
     request's, T_queue = now - enqueue time of the front request;
  3. among the GPUs feasible at that k the one with the smallest estimated T_inf gets the batch, which
     is logged in that GPU's running list (link model and co-location tracker advance).
violate(): (1) a low-priority batch may not lift the summed peak throughput of the low-priority batches
running on the GPU above C_low; (2) no running batch of equal or higher priority may be pushed past its
deadline: its completed fraction is (elapsed kernel time) / (Intf under its time-weighted pressure so far
x isolated kernel latency), the rest runs at the Intf predicted for the pressure it would see with the
new batch added.
meet(): the new batch must meet its own deadline with T_kernel predicted for half of the GPU's current
summed demand.
C_low: additive increase 0.25 % per full 100 ms up to 100 %, reset to 75 % when a high-priority batch
misses its deadline.

Readings where the paper is silent: "peak throughput" of a batch is the largest of its five demand
metrics; elapsed kernel time of a running batch counts from its predicted kernel start (submission time
plus T_data plus its isolated transfer time); feasibility is assumed monotone in k (that is what makes
a binary search valid), the probe sequence is lo = 1, hi = limit, mid = (lo + hi + 1) // 2.
"""
from __future__ import annotations

import numpy as np

from oracle.interference import ColocationOracle, PredictorOracle
from oracle.transfer import LinkOracle

HIGH, LOW = 0, 1
C_LOW_MIN, C_LOW_MAX, C_LOW_STEP, C_LOW_PERIOD_NS = 0.75, 1.00, 0.0025, 100_000_000


class Profile:
    """Offline profile of one (model, batch size): isolated p95 latencies (ns) and resource demand."""

    def __init__(self, t_inf_isol, t_htod, t_kernel_isol, m, self_cmp, self_mem):
        self.t_inf_isol, self.t_htod, self.t_kernel_isol = float(t_inf_isol), int(t_htod), float(t_kernel_isol)
        self.m = np.asarray(m, dtype=np.float64)
        self.self_cmp, self.self_mem = float(self_cmp), float(self_mem)
        self.peak = float(self.m.max())


class SchedulerOracle:
    def __init__(self, n_gpus, predictor: PredictorOracle):
        self.pred = predictor
        self.links = [LinkOracle() for _ in range(n_gpus)]
        self.track = [ColocationOracle() for _ in range(n_gpus)]
        self.running = [dict() for _ in range(n_gpus)]      # tracker id -> record
        self.models = {}                                     # model id -> (priority, [Profile] by batch-1)
        self.c_low = C_LOW_MIN
        self.t_aimd = None

    def set_profile(self, model_id, priority, profiles):
        self.models[model_id] = (priority, list(profiles))

    # ---- AIMD ------------------------------------------------------------------------------------
    def tick(self, now):
        if self.t_aimd is None:
            self.t_aimd = now
        steps = (now - self.t_aimd) // C_LOW_PERIOD_NS
        if steps > 0:
            self.c_low = min(C_LOW_MAX, self.c_low + steps * C_LOW_STEP)
            self.t_aimd += steps * C_LOW_PERIOD_NS

    # ---- the two predicates ------------------------------------------------------------------------
    def _violate(self, g, prio, prof, now):
        if prio == LOW:
            lp = sum(r["prof"].peak for r in self.running[g].values() if r["prio"] == LOW)
            if lp + prof.peak > self.c_low:
                return True
        for rid, r in self.running[g].items():
            if r["prio"] > prio:                             # lower priority than the new batch: may be hurt
                continue
            rp = r["prof"]
            elapsed = max(0, now - r["t_kernel_start"])
            # pressure so far: time-weighted average over the batch's life up to now
            life = now - r["t0"]
            tr = self.track[g]
            acc = tr.running[rid]["acc"] + (tr.pressure(rid)) * (now - tr.t_last) if tr.t_last is not None else tr.running[rid]["acc"]
            m_sofar = acc / life if life > 0 else np.zeros_like(rp.m)
            intf_sofar = self.pred.predict(m_sofar, rp.self_cmp, rp.self_mem, r["prio"])
            done = min(1.0, elapsed / (intf_sofar * rp.t_kernel_isol)) if rp.t_kernel_isol > 0 else 1.0
            m_new = tr.pressure(rid) + prof.m
            intf_new = self.pred.predict(m_new, rp.self_cmp, rp.self_mem, r["prio"])
            finish = max(now, r["t_kernel_start"]) + (1.0 - done) * rp.t_kernel_isol * intf_new
            if finish > r["deadline"]:
                return True
        return False

    def _t_inf(self, g, prio, prof, now, t_queue):
        t_data = self.links[g].predict(now)
        m_half = 0.5 * self.track[g].pressure()
        t_kernel = self.pred.t_kernel(m_half, prof.self_cmp, prof.self_mem, prio, prof.t_kernel_isol)
        return prof.t_inf_isol + t_data + t_kernel + t_queue

    def _meet(self, g, prio, prof, now, t_queue, t_front, deadline):
        return t_front + self._t_inf(g, prio, prof, now, t_queue) <= deadline

    # ---- one decision ------------------------------------------------------------------------------
    def decide(self, model_id, now, enqueue, deadline):
        """enqueue/deadline: per buffered request, oldest first.  Returns dict(dropped, batch, gpu, t_inf, id)."""
        prio, profs = self.models[model_id]
        self.tick(now)
        dropped = 0
        while dropped < len(enqueue) and deadline[dropped] - now < profs[0].t_inf_isol:
            dropped += 1
        enqueue, deadline = enqueue[dropped:], deadline[dropped:]
        out = {"dropped": dropped, "batch": 0, "gpu": -1, "t_inf": 0.0, "id": 0}
        limit = min(len(enqueue), len(profs))
        if limit == 0:
            return out
        t_front, d_front = enqueue[0], deadline[0]
        t_queue = now - t_front

        def feasible(k):
            prof = profs[k - 1]
            return [g for g in range(len(self.links))
                    if not self._violate(g, prio, prof, now) and self._meet(g, prio, prof, now, t_queue, t_front, d_front)]

        best, best_gpus = 0, []
        lo, hi = 1, limit
        while lo <= hi:
            mid = (lo + hi + 1) // 2
            gpus = feasible(mid)
            if gpus:
                best, best_gpus = mid, gpus
                lo = mid + 1
            else:
                hi = mid - 1
        if best == 0:
            return out
        prof = profs[best - 1]
        lat = [(self._t_inf(g, prio, prof, now, t_queue), g) for g in best_gpus]
        t_inf, g = min(lat)                                  # ties: lowest GPU index
        tid, t_data = self.links[g].schedule(now, prof.t_htod)
        rid = self.track[g].arrive(now, prof.m)
        self.running[g][rid] = {"prio": prio, "prof": prof, "t0": now, "deadline": d_front, "link_id": tid,
                                "t_kernel_start": now + t_data + prof.t_htod}
        out.update(batch=best, gpu=g, t_inf=t_inf, id=rid)
        return out

    def complete(self, gpu, rid, now, kernel_ns, h2d_end_ns=None):
        """The batch finished at `now` with measured kernel latency; feeds the predictor and the link."""
        r = self.running[gpu].pop(rid)
        m_avg = self.track[gpu].depart(rid, now)
        if h2d_end_ns is not None:
            self.links[gpu].complete(r["link_id"], h2d_end_ns)       # an unknown transfer id is an error and surfaces
        actual = kernel_ns / r["prof"].t_kernel_isol
        loss = self.pred.update(m_avg, r["prof"].self_cmp, r["prof"].self_mem, r["prio"], actual)
        violated = now > r["deadline"]
        if violated and r["prio"] == HIGH:
            self.c_low = C_LOW_MIN
            self.t_aimd = now
        return {"violated": violated, "loss": loss, "m_avg": m_avg}
