"""The host-to-device link model (Eq. 2, Eq. 3 and the online calibration of Section 3.2): pins of the
oracle, and the C ABI against the oracle.  Host only: runs without a GPU."""
import os
import random

import pytest

from oracle.transfer import LinkOracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "link_fifo.txt")


def golden_ops():
    for line in open(GOLDEN):
        if line[0] == "#" or not line.strip():
            continue
        lhs, rhs = line.split("->")
        op, a, b = lhs.split()
        want_t, want_avail = rhs.split()
        yield op, int(a), int(b), (None if want_t == "-" else int(want_t)), int(want_avail)


def drive(link, op, a, b):
    if op == "schedule":
        return link.schedule(a, b)[1]
    if op == "complete":
        link.complete(a, b)
        return None
    return link.predict(a)


def test_oracle_hand_worked():
    o = LinkOracle()
    assert o.predict(123) == 0
    for op, a, b, want_t, want_avail in golden_ops():
        got = drive(o, op, a, b)
        assert got == want_t and o.available() == want_avail, (op, a, b)


def fifo_server_simulation(arrivals):
    """Independent formulation: a single server that serves jobs in arrival order."""
    waits, free_at = [], None
    for t, d in arrivals:
        start = t if free_at is None or free_at <= t else free_at
        waits.append(start - t)
        free_at = start + d
    return waits, free_at


def test_oracle_is_a_fifo_queue_and_closed_forms():
    rnd = random.Random(7)
    t, arrivals = 0, []
    for _ in range(500):
        t += rnd.randrange(0, 40)
        arrivals.append((t, rnd.randrange(1, 30)))
    o = LinkOracle()
    waits = [o.schedule(t, d)[1] for t, d in arrivals]
    want, free_at = fifo_server_simulation(arrivals)
    assert waits == want and o.available() == free_at and min(waits) >= 0
    # all at the same instant: the k-th waits for the sum of the earlier transfer times
    o = LinkOracle()
    ds = [5, 7, 11, 13]
    assert [o.schedule(100, d)[1] for d in ds] == [0, 5, 12, 23]
    # spaced further apart than they take: nobody waits
    o = LinkOracle()
    assert all(o.schedule(100 * k, 99)[1] == 0 for k in range(10))
    # calibration with the predicted ends changes nothing; a late end delays the successors by as much
    o, p = LinkOracle(), LinkOracle()
    for q in (o, p):
        q.schedule(0, 10); q.schedule(1, 10); q.schedule(2, 10)
    o.complete(1, 10)
    assert o.available() == p.available() == 30
    o.complete(2, 25)                       # predicted 20, measured 25
    assert o.available() == 35 and o.predict(3) == 32


@pytest.fixture(scope="module")
def S():
    import paper_2604_28175_amd as strait
    return strait


def test_c_abi_matches_golden_and_oracle(S):
    link = S.Link()
    for op, a, b, want_t, want_avail in golden_ops():
        assert drive(link, op, a, b) == want_t and link.available() == want_avail, (op, a, b)
    link.close()
    rnd = random.Random(11)
    for trial in range(20):
        link, o = S.Link(), LinkOracle()
        t, ids, newest_done = 0, [], 0
        for step in range(300):
            t += rnd.randrange(0, 2000)
            r = rnd.random()
            if r < 0.6 or not ids:
                d = rnd.randrange(1, 3000)
                (i1, w1), (i2, w2) = link.schedule(t, d), o.schedule(t, d)
                assert i1 == i2 and w1 == w2
                ids.append(i1)
            elif r < 0.8:
                assert link.predict(t) == o.predict(t)
            else:
                tid = rnd.choice(ids)
                end = t + rnd.randrange(0, 500)
                if tid > newest_done:
                    link.complete(tid, end); o.complete(tid, end); newest_done = tid
                else:
                    with pytest.raises(S.StraitError):      # older than a calibrated transfer: already history
                        link.complete(tid, end)
            assert link.available() == o.available()
        link.close()


def test_c_abi_link_errors(S):
    assert S.lib.strait_link_create(None) == S.E_INVALID
    link = S.Link()
    with pytest.raises(S.StraitError):
        link.complete(42, 0)
    with pytest.raises(S.StraitError):
        link.schedule(0, -1)
    assert link.predict(5) == 0
    link.close()
