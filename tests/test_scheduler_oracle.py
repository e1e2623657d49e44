"""Pins of the scheduling-policy oracle (Algorithm 1, violate / meet, early dropping, AIMD cap, Eq. 1)."""
import os

import numpy as np
import pytest

from oracle import scheduler as osch
from oracle.interference import PredictorOracle

MS = 1_000_000
HIGH, LOW = osch.HIGH, osch.LOW
SIMPLE = np.array([1.0, 4.0, -1.0, 1, 0, 0, 0, 0, 0, 0, 1, 1])     # Intf = 4^(first metric) under pressure


def golden():
    out = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "scheduler_worked.txt")):
        if line[0] == "#" or not line.strip():
            continue
        f = line.split()
        out[f[0]] = {f[i]: float(f[i + 1]) for i in range(1, len(f), 2)}
    return out


def linear_profiles(n, base_ms=1.0, per_ms=0.5, kernel_ms=None, metric=0.0, htod_ms=0.0):
    return [osch.Profile((base_ms + per_ms * k) * MS, htod_ms * MS, (kernel_ms if kernel_ms is not None else base_ms + per_ms * k) * MS,
                         [metric, 0, 0, 0, 0], 0, 0) for k in range(1, n + 1)]


def make(n_gpus=1, params=SIMPLE):
    return osch.SchedulerOracle(n_gpus, PredictorOracle(params))


def test_largest_batch_closed_form():
    g = golden()["largest_batch"]
    s = make()
    s.set_profile(7, HIGH, linear_profiles(12))
    d = s.decide(7, 1 * MS, [0] * 12, [6 * MS] * 12)
    assert d["batch"] == g["batch"] and d["gpu"] == 0 and d["dropped"] == 0
    assert d["t_inf"] == pytest.approx(g["t_inf"] * MS)


def test_early_drop():
    g = golden()["early_drop"]
    s = make()
    s.set_profile(1, LOW, linear_profiles(8))
    d = s.decide(1, 5 * MS, [0, 1 * MS, 2 * MS, 3 * MS], [6 * MS, 7 * MS, 8 * MS, 9 * MS])
    assert d["dropped"] == g["dropped"] and d["batch"] == g["batch"]
    s2 = make()
    s2.set_profile(1, LOW, linear_profiles(8))
    d2 = s2.decide(1, 20 * MS, [0, 1 * MS], [6 * MS, 7 * MS])            # everything is late: all dropped, nothing scheduled
    assert d2["dropped"] == 2 and d2["batch"] == 0 and d2["gpu"] == -1


def test_eq1_terms_add_up():
    g = golden()["eq1"]
    s = make()
    s.set_profile(1, HIGH, [osch.Profile(1.5 * MS, 3 * MS, 1.0 * MS, [1, 0, 0, 0, 0], 0, 0)])
    s.set_profile(2, HIGH, [osch.Profile(1.5 * MS, 0, 1.0 * MS, [0.1, 0, 0, 0, 0], 0, 0)])
    first = s.decide(1, 0, [0], [100 * MS])                                  # occupies the link until 3 and exerts pressure 1
    assert first["batch"] == 1
    d = s.decide(2, 1 * MS, [MS // 2], [100 * MS])
    assert d["batch"] == 1 and d["t_inf"] == pytest.approx(g["t_inf"] * MS)


def protect_case(deadline_ms, running_prio, new_prio):
    s = make()
    s.set_profile(1, running_prio, [osch.Profile(4 * MS, 0, 4 * MS, [0.0, 0, 0, 0, 0], 0, 0)])
    s.set_profile(2, new_prio, [osch.Profile(1 * MS, 0, 1 * MS, [0.5, 0, 0, 0, 0], 0, 0)])
    assert s.decide(1, 0, [0], [deadline_ms * MS])["batch"] == 1
    return s.decide(2, 2 * MS, [2 * MS], [100 * MS])["batch"]


def test_running_batches_of_equal_or_higher_priority_are_protected():
    g = golden()["protect"]
    assert protect_case(7, HIGH, LOW) == g["admit_deadline_7"]
    assert protect_case(5.5, HIGH, LOW) == g["admit_deadline_5.5"]
    assert protect_case(5.5, HIGH, HIGH) == g["admit_deadline_5.5"]
    assert protect_case(5.5, LOW, LOW) == g["admit_deadline_5.5"]
    assert protect_case(5.5, LOW, HIGH) == g["hp_over_lp"]


def test_low_priority_cap():
    g = golden()["cap"]

    def run(n_gpus, prio):
        s = make(n_gpus)
        s.set_profile(1, LOW, [osch.Profile(1 * MS, 0, 1 * MS, [0.0, 0.5, 0, 0, 0], 0, 0)])
        s.set_profile(2, prio, [osch.Profile(1 * MS, 0, 1 * MS, [0.0, 0.3, 0.1, 0, 0], 0, 0)])
        assert s.decide(1, 0, [0], [100 * MS])["gpu"] == 0
        return s.decide(2, 0, [0], [100 * MS])["gpu"]

    assert run(2, LOW) == g["lp_two_gpus"] and run(1, LOW) == g["lp_one_gpu"] and run(1, HIGH) == g["hp_one_gpu"]


def test_aimd():
    g = golden()["aimd"]
    s = make()
    s.tick(0)
    assert s.c_low == 0.75
    s.tick(99 * MS)
    assert s.c_low == 0.75
    s.tick(1000 * MS)
    assert s.c_low == pytest.approx(g["after_1s"])
    s.tick(12_000 * MS)
    assert s.c_low == g["after_12s"]
    s.set_profile(1, HIGH, linear_profiles(1))
    d = s.decide(1, 12_000 * MS, [12_000 * MS], [12_010 * MS])
    res = s.complete(d["gpu"], d["id"], 12_050 * MS, 1.5 * MS)               # finished after its deadline
    assert res["violated"] and s.c_low == g["after_hp_miss"]


def test_lowest_latency_gpu_and_ties():
    s = make(3)
    s.set_profile(1, LOW, [osch.Profile(1 * MS, 2 * MS, 1 * MS, [0.1, 0, 0, 0, 0], 0, 0)])
    assert s.decide(1, 0, [0], [100 * MS])["gpu"] == 0                       # all idle: lowest index
    assert s.decide(1, 0, [0], [100 * MS])["gpu"] == 1                       # GPU 0's link is busy now
    assert s.decide(1, 0, [0], [100 * MS])["gpu"] == 2
    assert s.decide(1, 5 * MS, [5 * MS], [100 * MS])["gpu"] == 0             # links idle again; pressure equal everywhere


def test_binary_search_finds_the_largest_feasible_batch():
    rng = np.random.default_rng(2)
    for trial in range(60):
        n = int(rng.integers(1, 33))
        base, per = rng.uniform(0.2, 2.0), rng.uniform(0.05, 0.6)
        slo = rng.uniform(1.0, 12.0)
        now = rng.uniform(0, 3.0)
        profs = linear_profiles(n, base, per)
        s = make(2)
        s.set_profile(1, HIGH, profs)
        j = int(rng.integers(1, 40))
        enq = sorted(rng.uniform(0, now, j))
        enq_ns = [int(t * MS) for t in enq]
        dl_ns = [t + int(slo * MS) for t in enq_ns]
        now_ns = int(now * MS)
        # brute force on the same definitions: after early dropping, the largest k whose isolated estimate meets the front deadline
        kept = [i for i in range(j) if dl_ns[i] - now_ns >= profs[0].t_inf_isol]
        dropped = j - len(kept) if kept == list(range(j - len(kept), j)) else None
        want = 0
        if kept:
            f = kept[0]
            for k in range(1, min(len(kept), n) + 1):
                if enq_ns[f] + profs[k - 1].t_inf_isol + (now_ns - enq_ns[f]) <= dl_ns[f]:
                    want = k
        d = s.decide(1, now_ns, enq_ns, dl_ns)
        assert d["batch"] == want and (dropped is None or d["dropped"] == dropped), trial


def test_completion_feeds_predictor_and_link():
    s = make()
    ref = PredictorOracle(SIMPLE)
    s.set_profile(1, LOW, [osch.Profile(4 * MS, 1 * MS, 3 * MS, [0.5, 0.2, 0, 0, 0], 0.3, 0.1)])
    s.set_profile(2, HIGH, [osch.Profile(2 * MS, 1 * MS, 1 * MS, [0.25, 0, 0, 0, 0], 0.2, 0.2)])
    a = s.decide(1, 0, [0], [100 * MS])
    b = s.decide(2, 1 * MS, [1 * MS], [100 * MS])
    out_b = s.complete(0, b["id"], 3 * MS, 1.4 * MS, h2d_end_ns=int(2.2 * MS))   # ran 1..3 beside the first batch the whole time
    assert np.allclose(out_b["m_avg"], [0.5, 0.2, 0, 0, 0])
    assert out_b["loss"] == pytest.approx(ref.update([0.5, 0.2, 0, 0, 0], 0.2, 0.2, HIGH, 1.4))
    assert np.allclose(s.pred.p, ref.p)
    assert s.links[0].available() == int(2.2 * MS)                               # measured end replaced the estimate
    out_a = s.complete(0, a["id"], 5 * MS, 3.3 * MS)                             # beside the second batch for 2 of its 5 ms
    assert np.allclose(out_a["m_avg"], np.array([0.25, 0, 0, 0, 0]) * 2 / 5)
    assert not out_a["violated"]
