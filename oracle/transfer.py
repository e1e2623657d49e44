"""CPU oracle of the host-to-device link model.  TEST INFRASTRUCTURE ONLY.

Section 3.2 of the paper ("Interference in data transfer"): pinned transfers of concurrent batches
are served first-in first-out, so the wait of a new batch is
    T_data = max(0, t_available - t_current)                         (Eq. 2)
and scheduling batch B(i,j) moves the link-free time to
    t_available <- max(t_current, t_available) + t_HtoD(i,j)         (Eq. 3)
"Online calibration": once a transfer has been timed its measured end replaces the estimate.  The
reading taken here: the whole history is kept and t_available is recomputed from scratch by running
Eq. 3 over the transfers in schedule order, a measured transfer contributing its measured end.
"""
from __future__ import annotations

NEG_INF = -(1 << 63)


class LinkOracle:
    def __init__(self):
        self.history = []            # dicts: t_sched, t_htod, t_end (None until measured)

    def available(self) -> int:
        a = NEG_INF
        for t in self.history:
            a = t["t_end"] if t["t_end"] is not None else max(t["t_sched"], a) + t["t_htod"]
        return a

    def predict(self, t_current: int) -> int:
        return max(0, self.available() - t_current)

    def schedule(self, t_current: int, t_htod: int):
        t_data = self.predict(t_current)
        self.history.append({"t_sched": t_current, "t_htod": t_htod, "t_end": None})
        return len(self.history), t_data        # ids count from 1

    def complete(self, transfer_id: int, t_end: int):
        self.history[transfer_id - 1]["t_end"] = t_end
