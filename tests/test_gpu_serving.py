"""The serving front end on the GPU: offline profiles, then requests through task queues, batch formation,
the scheduling policy and the library's own executor.  Every served request's output is compared with the
CPU oracle's result for that request's input (a batch is only a vehicle: Section 2 of the paper), whatever
batch it rode in and at whatever position."""
import time

import numpy as np
import pytest

import synth
from oracle import models as omodels
from parity import check_logits

pytestmark = pytest.mark.gpu
MS = 1_000_000
HIGH, LOW = 0, 1


@pytest.fixture(scope="module")
def env():
    import paper_2604_28175_amd as strait
    ctx = strait.Context(device=0, n_hp=1, n_lp=1, n_copy=2)
    mds = {1: synth.resnet50(11, hw=64), 2: synth.mobilenet_v2(12, hw=64),
           3: synth.encoder(13, layers=2, hidden=128, heads=2, ffn=256, seq=64)}
    models = {mid: ctx.load(synth.pack(md), max_batch=8, n_instances=3) for mid, md in mds.items()}
    yield strait, ctx, mds, models
    for m in models.values():
        m.free()
    ctx.close()


def profiles(S, model, prio, max_batch, reps=12):
    return [S.profile_model(model, prio, b, reps) for b in range(1, max_batch + 1)]


def as_tuples(profs):
    return [(p.t_inf_isol_ns, p.t_htod_ns, p.t_kernel_isol_ns, list(p.m), p.m_self_cmp, p.m_self_mem) for p in profs]


def test_profile_of_a_batch(env):
    S, ctx, mds, models = env
    p1, p8 = S.profile_model(models[1], HIGH, 1, 20), S.profile_model(models[1], HIGH, 8, 20)
    for p in (p1, p8):
        assert 0 < p.t_htod_ns < p.t_inf_isol_ns and 0 < p.t_kernel_isol_ns < p.t_inf_isol_ns
        assert all(0.0 < v < 1.5 for v in p.m) and p.m_self_cmp == p.m[3] and p.m_self_mem == p.m[1]
    assert p8.m[3] > p1.m[3]                                      # eight images keep the matrix pipes busier than one
    x = synth.default_image_batch(mds[1], 8, 5)
    _, rec = models[1].infer(x, prio=HIGH)
    _, rec = models[1].infer(x, prio=HIGH)
    print(f"kernel time of one batch of 8 over its profiled p95: {rec.kernel_ms * 1e6 / p8.t_kernel_isol_ns:.2f}")   # reported only
    assert rec.kernel_ms > 0
    with pytest.raises(S.StraitError):
        S.profile_model(models[1], HIGH, 9, 5)                    # above max_batch


def test_served_requests_get_the_oracles_outputs(env):
    S, ctx, mds, models = env
    prio = {1: HIGH, 2: LOW, 3: HIGH}
    sched = S.Scheduler(1)
    srv = S.Server(sched, 4, 200_000)
    for mid, m in models.items():
        sched.set_profile(mid, prio[mid], as_tuples(profiles(S, m, prio[mid], 8)))
        srv.add_model(m, mid, prio[mid], 8, 400 * MS, 3 * MS)
    srv.start()
    n = 20
    xs = {1: synth.default_image_batch(mds[1], n, 21), 2: synth.default_image_batch(mds[2], n, 22)}
    xs[3], vl = synth.token_batch(mds[3], n, 23, min_len=32)
    outs = {mid: [models[mid].new_output(1) for _ in range(n)] for mid in models}
    ids = {}
    rng = np.random.default_rng(0)
    for i in range(n):                                            # bursts of uneven size, so that batches of many sizes form
        for mid in (1, 2, 3):
            ids[srv.request(mid, xs[mid][i], outs[mid][i], int(vl[i]) if mid == 3 else 0)] = (mid, i)
        if rng.random() < 0.35:
            time.sleep(0.006)
    srv.wait_idle(60.0)
    recs = srv.results()
    st = srv.stats()
    srv.close()
    sched.close()
    assert sorted(r.request_id for r in recs) == sorted(ids) and all(r.status == 0 for r in recs), [r.status for r in recs]
    assert st.served == 3 * n and st.max_in_flight <= 4 and st.batches < 3 * n           # some batching happened
    sizes = sorted({r.batch for r in recs})
    assert len(sizes) >= 2, sizes
    ref = {1: omodels.resnet50_forward(mds[1].tensors, xs[1]), 2: omodels.mobilenet_v2_forward(mds[2].tensors, xs[2]),
           3: omodels.encoder_forward(mds[3].tensors, xs[3], vl, mds[3].hyper)}
    for mid in (1, 2):
        got = [models[mid].decode(outs[mid][i], 1) for i in range(n)]
        logits = np.stack([g["logits"][0] for g in got])
        top1 = np.array([g["top1"][0] for g in got], dtype=np.int32)
        check_logits(logits, ref[mid].logits, top1, f"served model {mid}")
        probs = np.stack([g["probs"][0] for g in got])
        assert np.abs(probs - ref[mid].probs).max() <= 2e-2
    scale = max(float(np.abs(ref[3].logits[i, :vl[i]]).max()) for i in range(n))
    hidden0, top1 = [], []
    for i in range(n):
        g = models[3].decode(outs[3][i], 1)
        L = int(vl[i])
        assert np.abs(g["hidden"][0, :L].astype(np.float64) - ref[3].logits[i, :L]).max() <= 2e-2 * scale
        hidden0.append(g["hidden"][0, 0])
        top1.append(g["top1"][0])
    check_logits(np.stack(hidden0), ref[3].logits[:, 0, :], np.array(top1, dtype=np.int32), "served encoder token 0")
    for r in recs:                                                # latency record of a request
        assert r.t_enqueue_ns <= r.t_dispatch_ns < r.t_done_ns and r.kernel_ns > 0 and r.h2d_ns > 0
        assert r.t_inf_pred_ns > 0 and r.violated == (r.t_done_ns > r.deadline_ns)
    print(f"served {st.served} requests in {st.batches} batches (sizes {sizes}), in flight at most {st.max_in_flight}, "
          f"deferrals {st.deferrals}")


def test_overload_drops_instead_of_queueing_forever(env):
    """Far more high-priority work than the deadline allows: early dropping keeps the queue short, every request
    ends as served or dropped, and what is served late or dropped counts as violated."""
    S, ctx, mds, models = env
    sched = S.Scheduler(1)
    profs = profiles(S, models[1], HIGH, 8)
    sched.set_profile(1, HIGH, as_tuples(profs))
    srv = S.Server(sched, 2, 200_000)
    deadline = int(2.0 * profs[0].t_inf_isol_ns)
    srv.add_model(models[1], 1, HIGH, 8, deadline, 0)
    srv.start()
    x = synth.default_image_batch(mds[1], 1, 3)[0]
    outs = [models[1].new_output(1) for _ in range(600)]
    for o in outs:
        srv.request(1, x, o)
    srv.wait_idle(60.0)
    recs = srv.results()
    st = srv.stats()
    srv.close()
    sched.close()
    assert len(recs) == 600 and st.served + st.dropped == 600 and st.dropped > 0 and st.served > 0
    assert all(r.violated == 1 for r in recs if r.status == 1)
    assert st.violated_high >= st.dropped
    print(f"overload: served {st.served}, dropped {st.dropped}, violated {st.violated_high}")
