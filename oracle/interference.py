"""CPU oracle of the kernel-interference predictor.  TEST INFRASTRUCTURE ONLY.

Section 3.2 of the paper ("Interference in kernel execution", "Self-adaptive model"), fp64 throughout:

  demand of a batch       m = sum_i v_i d_i / sum_i d_i      (time-weighted kernel throughputs)
  Eq. 4                   kernel_eff = k * b**LR + C,   LR = w_avg . m_avg + w_cmp m_self_cmp + w_mem m_self_mem
  Eq. 5                   Intf = 1 + kernel_eff * coeff_p
  Eq. 6                   T_kernel = (Intf - 1) * T_kernel_isol
  co-location dynamics    m_avg of a batch = time-weighted average, over its life, of the summed demands
                          of the batches running beside it; re-evaluated at every arrival and departure
  online learning         after each completed batch one Adam step (beta1 0.7, beta2 0.9, alpha 0.0075) on
                          the Huber loss (delta 0.5) between the predicted and the measured Intf

Readings where the paper is silent: LR has no intercept (it would be absorbed by k); a batch that never
had a neighbour has Intf = 1 by definition and does not train the model; Adam is the published algorithm
with bias correction and eps = 1e-8 applied to the whole parameter vector (the coefficient of the other
priority level sees a zero gradient); after a step the base b is kept >= B_MIN so that b**LR stays real.
"""
from __future__ import annotations

import math

import numpy as np

N_METRICS = 5          # co-located metrics: [L1/LDS, L2, DRAM, matrix pipes, FMA pipes]
N_PRIO = 2
BETA1, BETA2, ALPHA, EPS = 0.7, 0.9, 0.0075, 1e-8
HUBER_DELTA = 0.5
B_MIN = 1e-6
# parameter vector layout: k, b, C, w_avg[5], w_cmp, w_mem, coeff_p[2]
N_PARAMS = 3 + N_METRICS + 2 + N_PRIO


def demand(v, d):
    """Time-weighted average throughput of a batch's kernels: v [n][N_METRICS], d [n] durations."""
    v = np.asarray(v, dtype=np.float64).reshape(len(d), -1)
    d = np.asarray(d, dtype=np.float64)
    return (v * d[:, None]).sum(axis=0) / d.sum()


def huber(e, delta=HUBER_DELTA):
    a = abs(e)
    return 0.5 * e * e if a <= delta else delta * (a - 0.5 * delta)


def default_params():
    """Conservative start: zero pressure -> no slowdown (C = -k), every co-located metric counts."""
    return np.array([1.0, 2.0, -1.0] + [0.5] * N_METRICS + [0.0, 0.0] + [1.0] * N_PRIO, dtype=np.float64)


class PredictorOracle:
    def __init__(self, params=None):
        self.p = default_params() if params is None else np.array(params, dtype=np.float64)
        assert self.p.shape == (N_PARAMS,)
        self.m = np.zeros(N_PARAMS)
        self.v = np.zeros(N_PARAMS)
        self.t = 0

    # ---- Eq. 4-6 ------------------------------------------------------------------------------
    def _lr(self, m_avg, self_cmp, self_mem):
        w = self.p[3:3 + N_METRICS]
        return float(np.dot(w, np.asarray(m_avg, dtype=np.float64)) + self.p[8] * self_cmp + self.p[9] * self_mem)

    def kernel_eff(self, m_avg, self_cmp, self_mem):
        k, b, c = self.p[0], self.p[1], self.p[2]
        return k * b ** self._lr(m_avg, self_cmp, self_mem) + c

    def predict(self, m_avg, self_cmp, self_mem, prio):
        if not np.any(np.asarray(m_avg) != 0.0):
            return 1.0                                       # isolation
        return 1.0 + self.kernel_eff(m_avg, self_cmp, self_mem) * self.p[10 + prio]

    def t_kernel(self, m_avg, self_cmp, self_mem, prio, t_isol):
        return (self.predict(m_avg, self_cmp, self_mem, prio) - 1.0) * t_isol

    # ---- one online step --------------------------------------------------------------------------
    def gradient(self, m_avg, self_cmp, self_mem, prio, intf_actual):
        """(loss, d loss / d params) of the Huber loss of (predicted - actual)."""
        m_avg = np.asarray(m_avg, dtype=np.float64)
        k, b = self.p[0], self.p[1]
        lr = self._lr(m_avg, self_cmp, self_mem)
        pw = b ** lr
        coeff = self.p[10 + prio]
        e = 1.0 + (k * pw + self.p[2]) * coeff - intf_actual
        dl = e if abs(e) <= HUBER_DELTA else HUBER_DELTA * math.copysign(1.0, e)
        g = np.zeros(N_PARAMS)
        g[0] = pw * coeff
        g[1] = k * lr * b ** (lr - 1.0) * coeff
        g[2] = coeff
        dlr = k * pw * math.log(b) * coeff
        g[3:3 + N_METRICS] = dlr * m_avg
        g[8] = dlr * self_cmp
        g[9] = dlr * self_mem
        g[10 + prio] = k * pw + self.p[2]
        return huber(e), dl * g

    def update(self, m_avg, self_cmp, self_mem, prio, intf_actual):
        if not np.any(np.asarray(m_avg) != 0.0):
            return 0.0
        loss, g = self.gradient(m_avg, self_cmp, self_mem, prio, intf_actual)
        self.t += 1
        self.m = BETA1 * self.m + (1.0 - BETA1) * g
        self.v = BETA2 * self.v + (1.0 - BETA2) * g * g
        mhat = self.m / (1.0 - BETA1 ** self.t)
        vhat = self.v / (1.0 - BETA2 ** self.t)
        self.p = self.p - ALPHA * mhat / (np.sqrt(vhat) + EPS)
        self.p[1] = max(self.p[1], B_MIN)
        return loss


class ColocationOracle:
    """Who ran beside whom, for how long: the time-weighted m_avg of every batch on one GPU."""

    def __init__(self):
        self.running = {}        # id -> dict(m, t0, acc)
        self.t_last = None
        self.next_id = 1

    def _advance(self, t):
        if self.t_last is not None:
            dt = t - self.t_last
            total = sum((r["m"] for r in self.running.values()), np.zeros(N_METRICS))
            for r in self.running.values():
                r["acc"] = r["acc"] + (total - r["m"]) * dt
        self.t_last = t

    def pressure(self, exclude_id=0):
        return sum((r["m"] for i, r in self.running.items() if i != exclude_id), np.zeros(N_METRICS))

    def arrive(self, t, m):
        self._advance(t)
        i = self.next_id
        self.next_id += 1
        self.running[i] = {"m": np.asarray(m, dtype=np.float64), "t0": t, "acc": np.zeros(N_METRICS)}
        return i

    def depart(self, batch_id, t):
        self._advance(t)
        r = self.running.pop(batch_id)
        life = t - r["t0"]
        return r["acc"] / life if life > 0 else np.zeros(N_METRICS)
