"""Pins of the interference-predictor oracle (Eq. 4-6, co-location dynamics, Adam + Huber online step)."""
import math
import os

import numpy as np
import pytest

from oracle import interference as oi

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "interference_worked.txt")
WORKED = np.array([2.0, 2.0, -1.0, 1, 0, 1, 0, 0, 0.5, -0.5, 0.5, 1.5])
HIGH, LOW = 0, 1


def golden():
    out = {}
    for line in open(GOLDEN):
        if line[0] == "#" or not line.strip():
            continue
        f = line.split()
        if f[0] == "forward":
            out[f[1]] = float(f[2])
        elif f[0] == "demand":
            out["demand"] = float(f[1])
        else:
            out["mavg_" + f[1]] = np.array([float(v) for v in f[2:]])
    return out


def test_forward_hand_worked():
    g, o = golden(), oi.PredictorOracle(WORKED)
    m = [1, 9, 2, 9, 9]
    assert o.kernel_eff(m, 2, 4) == g["kernel_eff"]
    assert o.predict(m, 2, 4, HIGH) == g["intf_high"] and o.predict(m, 2, 4, LOW) == g["intf_low"]
    assert o.t_kernel(m, 2, 4, HIGH, 2.0) == g["t_kernel_high"] and o.t_kernel(m, 2, 4, LOW, 2.0) == g["t_kernel_low"]
    assert oi.demand([[0.8] * 5, [0.2] * 5], [1, 3]) == pytest.approx([g["demand"]] * 5, rel=1e-15)


def test_isolation_is_no_slowdown_and_does_not_train():
    o = oi.PredictorOracle(WORKED)
    assert o.predict([0] * 5, 0.7, 0.3, LOW) == 1.0 and o.t_kernel([0] * 5, 0.7, 0.3, HIGH, 5.0) == 0.0
    before = o.p.copy()
    assert o.update([0] * 5, 0.7, 0.3, LOW, 1.3) == 0.0 and np.array_equal(o.p, before) and o.t == 0
    d = oi.PredictorOracle()                                     # conservative default: zero exponent -> k + C = 0
    assert d.kernel_eff([0] * 5, 0, 0) == 0.0


def test_colocation_hand_worked():
    g = golden()
    mA, mB, mC = [0.2, 0.4, 0.1, 0.5, 0], [0.1, 0.2, 0.3, 0, 0.6], [0.3, 0, 0, 0, 0.1]
    c = oi.ColocationOracle()
    a = c.arrive(0, mA)
    b = c.arrive(10, mB)
    assert np.allclose(c.pressure(exclude_id=a), mB)
    cc = c.arrive(30, mC)
    assert np.allclose(c.depart(b, 40), g["mavg_B"], rtol=1e-14)
    assert np.allclose(c.depart(a, 50), g["mavg_A"], rtol=1e-14)
    assert np.allclose(c.depart(cc, 80), g["mavg_C"], rtol=1e-14)
    lone = c.arrive(100, mA)                                     # nobody beside it: zero pressure
    assert not c.depart(lone, 130).any()


def test_huber_closed_forms():
    d = oi.HUBER_DELTA
    assert d == 0.5
    assert oi.huber(0.0) == 0 and oi.huber(0.2) == pytest.approx(0.02) and oi.huber(-0.2) == pytest.approx(0.02)
    assert oi.huber(d) == pytest.approx(0.125) and oi.huber(3.0) == pytest.approx(0.5 * 2.75) == oi.huber(-3.0)
    eps = 1e-9                                                   # C1 at the threshold: value and slope continuous
    assert oi.huber(d + eps) == pytest.approx(oi.huber(d - eps), abs=1e-8)
    assert (oi.huber(d + 2 * eps) - oi.huber(d + eps)) / eps == pytest.approx(d, rel=1e-5)


def numeric_gradient(o, m, sc, sm, prio, actual, h=1e-6):
    g = np.zeros(oi.N_PARAMS)
    for i in range(oi.N_PARAMS):
        vals = []
        for s in (+1, -1):
            q = oi.PredictorOracle(o.p)
            q.p[i] += s * h
            vals.append(oi.huber(q.predict(m, sc, sm, prio) - actual))
        g[i] = (vals[0] - vals[1]) / (2 * h)
    return g


@pytest.mark.parametrize("actual", [4.3, 4.8, 9.0, 1.0])        # inside the quadratic zone, on both sides, both linear tails
def test_gradient_matches_finite_differences(actual):
    rng = np.random.default_rng(3)
    p = WORKED + rng.normal(0, 0.05, oi.N_PARAMS)
    o = oi.PredictorOracle(p)
    m, sc, sm = rng.uniform(0.1, 1.0, 5), 0.6, 0.3
    for prio in (HIGH, LOW):
        scale = o.predict(m, sc, sm, prio) / 4.5
        loss, g = o.gradient(m, sc, sm, prio, actual * scale)
        assert loss == pytest.approx(oi.huber(o.predict(m, sc, sm, prio) - actual * scale))
        assert np.allclose(g, numeric_gradient(o, m, sc, sm, prio, actual * scale), rtol=1e-5, atol=1e-8)
        assert g[10 + (1 - prio)] == 0.0                         # the other level's coefficient is untouched by this sample


def test_adam_first_step_is_alpha_against_the_gradient_sign():
    o = oi.PredictorOracle(WORKED)
    m, sc, sm = [0.3, 0.2, 0.5, 0.4, 0.1], 0.5, 0.25
    _, g = o.gradient(m, sc, sm, LOW, 1.2)
    before = o.p.copy()
    o.update(m, sc, sm, LOW, 1.2)
    step = o.p - before
    nz = g != 0
    assert nz.sum() == oi.N_PARAMS - 1
    assert np.allclose(step[nz], -oi.ALPHA * np.sign(g[nz]), rtol=1e-6) and np.all(step[~nz] == 0)
    assert (oi.BETA1, oi.BETA2, oi.ALPHA) == (0.7, 0.9, 0.0075)


def test_online_steps_match_torch_adam_and_huber():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(11)
    o = oi.PredictorOracle(WORKED)
    p = torch.tensor(WORKED, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([p], lr=0.0075, betas=(0.7, 0.9), eps=1e-8)
    lossf = torch.nn.HuberLoss(delta=0.5)
    for step in range(300):
        m, sc, sm = rng.uniform(0, 1, 5), rng.uniform(0, 1), rng.uniform(0, 1)
        prio, actual = int(rng.integers(0, 2)), float(rng.uniform(1.0, 6.0))
        o.update(m, sc, sm, prio, actual)
        opt.zero_grad()
        lr = (p[3:8] * torch.tensor(m)).sum() + p[8] * sc + p[9] * sm
        pred = 1.0 + (p[0] * p[1] ** lr + p[2]) * p[10 + prio]
        lossf(pred.reshape(1), torch.tensor([actual], dtype=torch.float64)).backward()
        opt.step()
        assert np.allclose(o.p, p.detach().numpy(), rtol=1e-9, atol=1e-12), step


def test_online_learning_recovers_a_known_interference_law():
    truth = oi.PredictorOracle(np.array([0.6, 3.0, -0.6, 0.9, 0.3, 0.5, 0.8, 0.2, 0.2, 0.1, 0.6, 1.0]))
    o = oi.PredictorOracle()
    rng = np.random.default_rng(5)

    def sample():
        return rng.uniform(0, 0.8, 5), rng.uniform(0, 1), rng.uniform(0, 1), int(rng.integers(0, 2))

    def mean_abs_error(n=300):
        r = np.random.default_rng(99)
        errs = []
        for _ in range(n):
            m, sc, sm, prio = r.uniform(0, 0.8, 5), r.uniform(0, 1), r.uniform(0, 1), int(r.integers(0, 2))
            errs.append(abs(o.predict(m, sc, sm, prio) - truth.predict(m, sc, sm, prio)))
        return float(np.mean(errs))

    e0 = mean_abs_error()
    for _ in range(6000):
        m, sc, sm, prio = sample()
        o.update(m, sc, sm, prio, truth.predict(m, sc, sm, prio))
    e1 = mean_abs_error()
    assert e1 < 0.25 * e0 and e1 < 0.15, (e0, e1)


def test_base_stays_positive():
    o = oi.PredictorOracle(np.array([1.0, 2e-6, 0.0, 1, 1, 1, 1, 1, 0, 0, 1, 1]))
    for _ in range(5):
        o.update([1, 1, 1, 1, 1], 0, 0, LOW, 0.0)                # pushes b down
    assert o.p[1] >= oi.B_MIN and math.isfinite(o.predict([1, 1, 1, 1, 1], 0, 0, LOW))
