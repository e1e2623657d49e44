"""The scheduling policy behind the C ABI against its oracle (host only: runs without a GPU)."""
import numpy as np
import pytest

from oracle import scheduler as osch
from oracle.interference import PredictorOracle, default_params
from test_scheduler_oracle import MS, SIMPLE, golden, linear_profiles

HIGH, LOW = 0, 1


@pytest.fixture(scope="module")
def S():
    import paper_2604_28175_amd as strait
    return strait


def as_tuples(profiles):
    return [(p.t_inf_isol, p.t_htod, p.t_kernel_isol, p.m, p.self_cmp, p.self_mem) for p in profiles]


def test_golden_cases_through_the_abi(S):
    g = golden()
    s = S.Scheduler(1, SIMPLE)
    s.set_profile(7, HIGH, as_tuples(linear_profiles(12)))
    d = s.decide(7, 1 * MS, [0] * 12, [6 * MS] * 12)
    assert (d.batch, d.gpu, d.n_dropped) == (g["largest_batch"]["batch"], 0, 0) and d.t_inf_ns == pytest.approx(g["largest_batch"]["t_inf"] * MS)
    s.close()
    s = S.Scheduler(1, SIMPLE)
    s.set_profile(1, LOW, as_tuples(linear_profiles(8)))
    d = s.decide(1, 5 * MS, [0, 1 * MS, 2 * MS, 3 * MS], [6 * MS, 7 * MS, 8 * MS, 9 * MS])
    assert (d.n_dropped, d.batch) == (g["early_drop"]["dropped"], g["early_drop"]["batch"])
    s.close()
    s = S.Scheduler(1, SIMPLE)
    assert s.tick(0) == 0.75 and s.tick(1000 * MS) == pytest.approx(g["aimd"]["after_1s"]) and s.tick(12_000 * MS) == g["aimd"]["after_12s"]
    s.set_profile(1, HIGH, as_tuples(linear_profiles(1)))
    d = s.decide(1, 12_000 * MS, [12_000 * MS], [12_010 * MS])
    c = s.complete(d.gpu, d.running_id, 12_050 * MS, 1.5 * MS)
    assert c.violated == 1 and c.c_low == g["aimd"]["after_hp_miss"]
    s.close()


def random_model(rng, n_batch):
    base, per = rng.uniform(0.3, 2.0), rng.uniform(0.05, 0.4)
    scale = rng.uniform(0.02, 0.12)
    profs = []
    for k in range(1, n_batch + 1):
        t_inf = (base + per * k) * MS
        m = np.minimum(1.0, scale * k ** 0.5 * rng.uniform(0.5, 1.5, 5))
        profs.append(osch.Profile(t_inf, int(0.02 * k * MS), 0.85 * t_inf, m, float(m[3]), float(m[1])))
    return profs


@pytest.mark.parametrize("seed,n_gpus", [(0, 1), (1, 2), (2, 3)])
def test_simulated_serving_matches_oracle(S, seed, n_gpus):
    """A synthetic serving run: Poisson arrivals for four models, the scheduler polled every 0.2 ms, batches
    completing with noisy slowdowns.  Every decision and every completion must agree with the oracle."""
    rng = np.random.default_rng(seed)
    start = default_params() + rng.normal(0, 0.02, default_params().size)
    s, o = S.Scheduler(n_gpus, start), osch.SchedulerOracle(n_gpus, PredictorOracle(start))
    models = {}
    for mid in range(4):
        prio = HIGH if mid < 2 else LOW
        profs = random_model(rng, int(rng.integers(4, 17)))
        slo = int(rng.uniform(4, 12) * MS)
        models[mid] = (prio, profs, slo)
        s.set_profile(mid, prio, as_tuples(profs))
        o.set_profile(mid, prio, profs)
    queues = {mid: [] for mid in models}
    arrivals = []
    for mid in models:
        t = 0.0
        while t < 60.0:
            t += rng.exponential(1.0 / rng.uniform(0.8, 2.5))
            arrivals.append((int(t * MS), mid))
    arrivals.sort()
    ai, in_flight, decisions, completions = 0, [], 0, 0
    for step in range(1, 400):
        now = step * MS // 5
        while ai < len(arrivals) and arrivals[ai][0] <= now:
            t, mid = arrivals[ai]; ai += 1
            queues[mid].append((t, t + models[mid][2]))
        for f in sorted([f for f in in_flight if f[0] <= now]):            # completions first, in time order
            t_done, gpu, rid, kernel_ns, h2d = f
            in_flight.remove(f)
            c, oc = s.complete(gpu, rid, t_done, kernel_ns, h2d), o.complete(gpu, rid, t_done, kernel_ns, h2d)
            assert bool(c.violated) == oc["violated"] and c.loss == pytest.approx(oc["loss"], rel=1e-9, abs=1e-15)
            assert np.allclose(list(c.m_avg), oc["m_avg"], rtol=1e-12, atol=1e-15) and c.c_low == pytest.approx(o.c_low, rel=1e-12)
            completions += 1
        for mid in sorted(models, key=lambda m: models[m][0]):             # queues in descending priority
            q = queues[mid]
            if not q:
                continue
            enq, dl = [a for a, _ in q], [b for _, b in q]
            d, od = s.decide(mid, now, enq, dl), o.decide(mid, now, enq, dl)
            assert (d.n_dropped, d.batch, d.gpu) == (od["dropped"], od["batch"], od["gpu"]), (step, mid)
            del q[:d.n_dropped + d.batch]
            if d.batch:
                assert d.t_inf_ns == pytest.approx(od["t_inf"], rel=1e-9) and d.running_id == od["id"]
                prof = models[mid][1][d.batch - 1]
                slow = 1.0 + rng.uniform(0, 0.8)
                t_k0 = now + d.t_data_ns + prof.t_htod
                in_flight.append((int(t_k0 + prof.t_kernel_isol * slow), d.gpu, d.running_id, prof.t_kernel_isol * slow,
                                  int(now + d.t_data_ns + prof.t_htod * rng.uniform(0.9, 1.3))))
                decisions += 1
        assert s.tick(now) == pytest.approx(o.c_low, rel=1e-12)
    assert decisions > 50 and completions > 40
    assert np.allclose(s.params(), o.pred.p, rtol=1e-8, atol=1e-12)
    s.close()


def test_error_paths(S):
    s = S.Scheduler(2)
    with pytest.raises(S.StraitError):
        s.decide(9, 0, [0], [10])                                             # no profile
    s.set_profile(1, HIGH, as_tuples(linear_profiles(2)))
    d = s.decide(1, 10, [0], [100 * MS])
    assert d.batch == 1
    with pytest.raises(S.StraitError):
        s.set_profile(1, HIGH, as_tuples(linear_profiles(3)))                 # batches of the model still run
    with pytest.raises(S.StraitError):
        s.decide(1, 5, [0], [100 * MS])                                       # time runs backwards
    with pytest.raises(S.StraitError):
        s.complete(1 - d.gpu, d.running_id, 20, 1.0)                          # wrong GPU
    with pytest.raises(S.StraitError):
        s.complete(7, d.running_id, 20, 1.0)
    s.complete(d.gpu, d.running_id, 20, 1.0)
    assert s.decide(1, 30, [], []).batch == 0
    s.close()
    assert S.lib.strait_sched_create(0, None, None) == S.E_INVALID
