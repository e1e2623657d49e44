"""The serving front end behind the C ABI with a host-side executor in place of the GPU (runs without one).

What is checked is what Sections 3, 4 and 5.1 of the paper state about the front end: one task queue per
model served first come first served, batch formation by size or timeout, queues visited in descending
priority, a limit on the batches in flight, early-dropped requests counted as violations, latency from
enqueue to result, and the measured kernel latency fed back into the predictor."""
import threading
import time

import numpy as np
import pytest

from test_scheduler_oracle import MS, SIMPLE

HIGH, LOW = 0, 1


@pytest.fixture(scope="module")
def S():
    import paper_2604_28175_amd as strait
    return strait


def flat_profiles(n, t_ms, m=0.05):
    """Batch size hardly matters: t_inf = t_ms (+1 % per extra sample), kernels 80 % of it."""
    return [((t_ms * (1 + 0.01 * (k - 1))) * MS, int(0.01 * MS), 0.8 * t_ms * MS, [m] * 5, m, m) for k in range(1, n + 1)]


class FakeGpu:
    """Batches take `dur_ms[model]` of wall time; records what ran when."""

    def __init__(self, dur_ms, fail=()):
        self.dur_ms, self.fail = dur_ms, set(fail)
        self.lock = threading.Lock()
        self.started, self.live, self.max_live = {}, 0, 0

    def submit(self, seq, mid, prio, batch):
        if mid in self.fail:
            return 1
        with self.lock:
            self.started[seq] = (time.monotonic_ns(), mid, prio, batch)
            self.live += 1
            self.max_live = max(self.max_live, self.live)
        return 0

    def wait(self, seq):
        t0, mid, _, _ = self.started[seq]
        left = t0 + self.dur_ms[mid] * MS - time.monotonic_ns()
        if left > 0:
            time.sleep(left / 1e9)
        with self.lock:
            self.live -= 1
        return 0.8 * self.dur_ms[mid] * MS, 0.01 * MS


def make(S, gpu, models, concurrency=4, params=SIMPLE):
    """models: {id: (priority, max_batch, deadline_ms, timeout_ms, n_instances, profile t_ms)}"""
    sched = S.Scheduler(1, params)
    srv = S.Server(sched, concurrency, 200_000, gpu.submit, gpu.wait)
    for mid, (prio, mb, ddl, to, ni, t_ms) in models.items():
        sched.set_profile(mid, prio, flat_profiles(mb, t_ms))
        srv.add_model(None, mid, prio, mb, int(ddl * MS), int(to * MS), ni)
    srv.start()
    return sched, srv


def finish(sched, srv):
    srv.wait_idle(20.0)
    recs = srv.results()
    st = srv.stats()
    srv.close()
    sched.close()
    return recs, st


def test_requests_that_arrive_within_the_timeout_ride_in_one_batch(S):
    gpu = FakeGpu({1: 5})
    sched, srv = make(S, gpu, {1: (HIGH, 8, 500, 30, 1, 5)})
    ids = [srv.request(1, None, None) for _ in range(3)]
    recs, st = finish(sched, srv)
    assert [r.request_id for r in recs] == ids and all(r.status == 0 and r.batch == 3 for r in recs)
    assert [r.position for r in recs] == [0, 1, 2] and len({r.batch_seq for r in recs}) == 1     # first come first served
    waited = (recs[0].t_dispatch_ns - recs[0].t_enqueue_ns) / MS
    assert 30.0 <= waited < 45.0                                   # the oldest request waited the formation timeout
    assert all(r.t_enqueue_ns <= r.t_dispatch_ns <= r.t_done_ns and r.violated == 0 for r in recs)
    assert all(r.deadline_ns == r.t_enqueue_ns + 500 * MS for r in recs)
    assert (st.requests, st.served, st.batches, st.batched_requests) == (3, 3, 1, 3)


def test_a_full_batch_leaves_without_waiting_for_the_timeout(S):
    gpu = FakeGpu({1: 5})
    sched, srv = make(S, gpu, {1: (HIGH, 4, 2000, 1000, 2, 5)})
    for _ in range(8):
        srv.request(1, None, None)
    recs, st = finish(sched, srv)
    assert sorted(r.batch for r in recs) == [4] * 8 and st.batches == 2
    assert max(r.t_dispatch_ns - r.t_enqueue_ns for r in recs) < 200 * MS


def test_high_priority_queue_is_visited_first(S):
    gpu = FakeGpu({1: 60, 2: 5})
    sched, srv = make(S, gpu, {1: (LOW, 1, 5000, 0, 2, 60), 2: (HIGH, 1, 5000, 0, 1, 5)}, concurrency=1)
    srv.request(1, None, None)            # occupies the only slot
    time.sleep(0.01)
    lp2 = srv.request(1, None, None)      # asks first ...
    time.sleep(0.005)
    hp = srv.request(2, None, None)       # ... but this one is of higher priority
    recs, st = finish(sched, srv)
    by_id = {r.request_id: r for r in recs}
    assert by_id[hp].batch_seq < by_id[lp2].batch_seq and by_id[hp].t_dispatch_ns <= by_id[lp2].t_dispatch_ns
    assert st.max_in_flight == 1 and gpu.max_live == 1 and st.deferrals >= 1


def test_concurrency_limit_holds(S):
    gpu = FakeGpu({1: 30, 2: 30})
    sched, srv = make(S, gpu, {1: (HIGH, 1, 5000, 0, 4, 30), 2: (HIGH, 1, 5000, 0, 4, 30)}, concurrency=2)
    for i in range(8):
        srv.request(1 + i % 2, None, None)
    recs, st = finish(sched, srv)
    assert st.max_in_flight == 2 and gpu.max_live == 2 and st.served == 8


def test_instances_bound_a_models_batches_in_flight(S):
    gpu = FakeGpu({1: 30})
    sched, srv = make(S, gpu, {1: (HIGH, 1, 5000, 0, 1, 30)}, concurrency=4)
    for _ in range(3):
        srv.request(1, None, None)
    recs, st = finish(sched, srv)
    assert gpu.max_live == 1 and st.served == 3


def test_requests_that_cannot_finish_alone_are_dropped_and_count_as_violations(S):
    gpu = FakeGpu({1: 5})
    sched, srv = make(S, gpu, {1: (HIGH, 4, 2, 0, 1, 5)})       # deadline 2 ms, isolated latency 5 ms
    for _ in range(5):
        srv.request(1, None, None)
    recs, st = finish(sched, srv)
    assert len(recs) == 5 and all(r.status == 1 and r.violated == 1 and r.batch == 0 for r in recs)
    assert (st.dropped, st.violated_high, st.batches) == (5, 5, 0) and not gpu.started


def test_late_results_count_as_violations(S):
    gpu = FakeGpu({1: 40})                                          # the profile promises 5 ms, the batch takes 40
    sched, srv = make(S, gpu, {1: (HIGH, 1, 20, 0, 1, 5)})
    srv.request(1, None, None)
    recs, st = finish(sched, srv)
    assert recs[0].status == 0 and recs[0].violated == 1 and st.violated_high == 1
    assert (recs[0].t_done_ns - recs[0].t_enqueue_ns) / MS >= 40.0
    assert recs[0].kernel_ns == pytest.approx(0.8 * 40 * MS)


def test_every_request_gets_exactly_one_record(S):
    rng = np.random.default_rng(3)
    gpu = FakeGpu({1: 3, 2: 6})
    sched, srv = make(S, gpu, {1: (HIGH, 8, 60, 2, 2, 3), 2: (LOW, 8, 200, 5, 2, 6)})
    ids = []
    for _ in range(300):
        ids.append(srv.request(int(rng.integers(1, 3)), None, None))
        time.sleep(float(rng.exponential(0.0005)))
    recs, st = finish(sched, srv)
    assert sorted(r.request_id for r in recs) == sorted(ids) and len(set(ids)) == 300
    assert st.requests == 300 == st.served + st.dropped + st.failed and st.requests_high + st.requests_low == 300
    served = [r for r in recs if r.status == 0]
    assert st.batched_requests == len(served) and st.batches == len({r.batch_seq for r in served})
    for seq in {r.batch_seq for r in served}:                      # a batch: one model, positions 0..n-1 in arrival order
        rs = sorted((r for r in served if r.batch_seq == seq), key=lambda r: r.position)
        assert len({r.model_id for r in rs}) == 1 and [r.position for r in rs] == list(range(rs[0].batch))
        assert all(a.request_id < b.request_id for a, b in zip(rs, rs[1:])) and rs[0].batch <= 8
    for mid in (1, 2):                                             # first come first served inside a queue
        rs = sorted((r for r in served if r.model_id == mid), key=lambda r: r.request_id)
        assert all(a.batch_seq <= b.batch_seq for a, b in zip(rs, rs[1:]))
    assert st.max_in_flight <= 4


def test_executor_failure_is_reported_and_the_running_list_cleaned(S):
    gpu = FakeGpu({1: 5, 2: 5}, fail={1})
    sched, srv = make(S, gpu, {1: (HIGH, 2, 500, 0, 1, 5), 2: (HIGH, 2, 500, 0, 1, 5)})
    a = srv.request(1, None, None)
    b = srv.request(2, None, None)
    srv.wait_idle(10.0)
    recs = {r.request_id: r for r in srv.results()}
    assert recs[a].status == 2 and recs[a].violated == 1 and recs[b].status == 0
    sched.set_profile(1, HIGH, flat_profiles(2, 5))                # refused while a batch of the model is logged as running
    srv.close()
    sched.close()


def test_stop_reports_what_is_still_queued(S):
    gpu = FakeGpu({1: 5})
    sched, srv = make(S, gpu, {1: (HIGH, 8, 5000, 4000, 1, 5)})   # the timeout never expires in this test
    ids = [srv.request(1, None, None) for _ in range(3)]
    srv.stop()
    recs = srv.results()
    assert [r.request_id for r in recs] == ids and all(r.status == 3 and r.violated == 1 for r in recs)
    with pytest.raises(S.StraitError):
        srv.request(1, None, None)
    srv.close()
    sched.close()


def test_measured_kernel_latency_reaches_the_predictor(S):
    """Two models run side by side and take 1.5x their isolated kernel time: the parameters must move."""
    gpu = FakeGpu({1: 15, 2: 15})
    sched, srv = make(S, gpu, {1: (HIGH, 1, 5000, 0, 1, 10), 2: (LOW, 1, 5000, 0, 1, 10)})
    before = sched.params().copy()
    for _ in range(5):
        srv.request(1, None, None)
        srv.request(2, None, None)
        time.sleep(0.03)
    srv.wait_idle(10.0)
    after = sched.params()
    assert np.abs(after - before).max() > 1e-3
    recs = srv.results()
    assert all(r.t_inf_pred_ns >= 10 * MS for r in recs)          # Eq. 1: never below the isolated latency
    srv.close()
    sched.close()


def test_argument_checks(S):
    sched = S.Scheduler(1, SIMPLE)
    with pytest.raises(S.StraitError):
        S.Server(sched, 0)
    srv = S.Server(sched, 2, 200_000, lambda *a: 0, lambda s: (1.0, 1.0))
    with pytest.raises(S.StraitError):
        srv.start()                                                # no models
    with pytest.raises(S.StraitError):
        srv.add_model(None, 1, 5, 4, MS, 0)                        # bad priority
    srv.add_model(None, 1, HIGH, 4, MS, 0)
    with pytest.raises(S.StraitError):
        srv.add_model(None, 1, HIGH, 4, MS, 0)                     # twice
    with pytest.raises(S.StraitError):
        srv.request(1, None, None)                                 # not started
    srv.close()
    sched.close()


def test_requests_from_many_threads(S):
    """strait_server_request is thread-safe: eight producers, every request accounted for exactly once."""
    gpu = FakeGpu({1: 2, 2: 3})
    sched, srv = make(S, gpu, {1: (HIGH, 8, 2000, 1, 2, 2), 2: (LOW, 8, 2000, 2, 2, 3)})
    ids, lock = [], threading.Lock()

    def producer(k):
        mine = [srv.request(1 + (k + i) % 2, None, None) for i in range(100)]
        with lock:
            ids.extend(mine)

    th = [threading.Thread(target=producer, args=(k,)) for k in range(8)]
    for t in th:
        t.start()
    for t in th:
        t.join()
    recs, st = finish(sched, srv)
    assert len(set(ids)) == 800 and sorted(r.request_id for r in recs) == sorted(ids)
    assert st.requests == 800 == st.served + st.dropped + st.failed


def test_stop_lets_batches_in_flight_finish(S):
    gpu = FakeGpu({1: 80})
    sched, srv = make(S, gpu, {1: (HIGH, 1, 5000, 0, 2, 80)}, concurrency=2)
    a, b, c = (srv.request(1, None, None) for _ in range(3))      # two start at once, the third waits for an instance
    time.sleep(0.02)
    t0 = time.monotonic()
    srv.stop()                                                     # returns only when the two running batches are done
    assert time.monotonic() - t0 >= 0.04
    recs = {r.request_id: r for r in srv.results()}
    assert recs[a].status == 0 and recs[b].status == 0 and recs[c].status == 3 and gpu.live == 0
    srv.close()
    sched.close()
