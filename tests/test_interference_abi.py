"""The interference predictor behind the C ABI against its oracle (host only: runs without a GPU).
Both sides compute in fp64; pow/log may differ in the last place, hence 1e-10 relative."""
import os

import numpy as np
import pytest

from oracle import interference as oi

HIGH, LOW = 0, 1
RTOL = 1e-10


@pytest.fixture(scope="module")
def S():
    import paper_2604_28175_amd as strait
    return strait


def test_defaults_and_layout(S):
    p = S.Interference()
    assert np.array_equal(p.params(), oi.default_params())
    assert S.INTF_METRICS == oi.N_METRICS
    p.close()
    v = np.arange(1, 13, dtype=np.float64)
    q = S.Interference(v)
    assert np.array_equal(q.params(), v)
    q.close()


def test_golden_values_through_the_abi(S):
    from test_interference_oracle import WORKED, golden
    g, p = golden(), S.Interference(WORKED)
    m = [1, 9, 2, 9, 9]
    assert p.predict(m, 2, 4, HIGH, 2.0) == (g["intf_high"], g["t_kernel_high"])
    assert p.predict(m, 2, 4, LOW, 2.0) == (g["intf_low"], g["t_kernel_low"])
    assert p.predict([0] * 5, 2, 4, LOW, 2.0) == (1.0, 0.0)
    assert S.intf_demand([[0.8] * 5, [0.2] * 5], [1, 3]) == pytest.approx([g["demand"]] * 5, rel=1e-15)
    mA, mB, mC = [0.2, 0.4, 0.1, 0.5, 0], [0.1, 0.2, 0.3, 0, 0.6], [0.3, 0, 0, 0, 0.1]
    a = p.arrive(0, mA); b = p.arrive(10, mB)
    assert np.allclose(p.pressure(a), mB, rtol=1e-15)
    c = p.arrive(30, mC)
    assert np.allclose(p.depart(b, 40), g["mavg_B"], rtol=1e-14)
    assert np.allclose(p.depart(a, 50), g["mavg_A"], rtol=1e-14)
    assert np.allclose(p.depart(c, 80), g["mavg_C"], rtol=1e-14)
    p.close()


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_online_learning_matches_oracle(S, seed):
    rng = np.random.default_rng(seed)
    start = oi.default_params() + rng.normal(0, 0.05, oi.N_PARAMS)
    p, o = S.Interference(start), oi.PredictorOracle(start)
    for step in range(500):
        m = rng.uniform(0, 1, 5) * (rng.random() > 0.1)          # one in ten batches ran alone
        sc, sm, prio = rng.uniform(0, 1), rng.uniform(0, 1), int(rng.integers(0, 2))
        want = o.predict(m, sc, sm, prio)
        got, tk = p.predict(m, sc, sm, prio, 3.5)
        assert got == pytest.approx(want, rel=RTOL) and tk == pytest.approx((want - 1.0) * 3.5, rel=1e-9, abs=1e-12)
        actual = float(rng.uniform(1.0, 4.0)) if step % 7 else float(rng.uniform(5.0, 30.0))    # some outliers (linear Huber zone)
        assert p.update(m, sc, sm, prio, actual) == pytest.approx(o.update(m, sc, sm, prio, actual), rel=1e-9, abs=1e-15)
        assert np.allclose(p.params(), o.p, rtol=1e-9, atol=1e-12), step
    p.close()


def test_colocation_tracker_matches_oracle(S):
    rng = np.random.default_rng(4)
    p, o = S.Interference(), oi.ColocationOracle()
    t, live = 0, []
    for step in range(2000):
        t += int(rng.integers(0, 5_000_000))
        if live and (len(live) >= 4 or rng.random() < 0.45):
            i = live.pop(int(rng.integers(0, len(live))))
            assert np.allclose(p.depart(i, t), o.depart(i, t), rtol=1e-12, atol=1e-15)
        else:
            m = rng.uniform(0, 1, 5)
            i, j = p.arrive(t, m), o.arrive(t, m)
            assert i == j
            live.append(i)
        ex = live[0] if live else 0
        assert np.allclose(p.pressure(ex), o.pressure(ex), rtol=1e-12, atol=1e-15)
    p.close()


def test_demand_matches_oracle(S):
    rng = np.random.default_rng(8)
    for n in (1, 3, 58):
        v, d = rng.uniform(0, 1, (n, 5)), rng.uniform(0, 2, n)
        assert np.allclose(S.intf_demand(v, d), oi.demand(v, d), rtol=1e-13)


def test_error_paths(S):
    p = S.Interference()
    with pytest.raises(S.StraitError):
        p.depart(99, 0)
    i = p.arrive(100, [0.1] * 5)
    with pytest.raises(S.StraitError):
        p.arrive(50, [0.1] * 5)                                  # time runs backwards
    with pytest.raises(S.StraitError):
        p.predict([0.1] * 5, 0, 0, 7)
    with pytest.raises(S.StraitError):
        p.update([0.1] * 5, 0, 0, LOW, float("nan"))
    with pytest.raises(S.StraitError):
        S.intf_demand([[0.1] * 5], [0.0])
    with pytest.raises(S.StraitError):
        S.Interference(np.array([1, 0.0, 0, 1, 1, 1, 1, 1, 0, 0, 1, 1.0]))
    p.depart(i, 100)
    p.close()
    assert S.lib.strait_intf_create(None, None) == S.E_INVALID
