"""Open-loop dual-priority driver: a high-priority request stream arriving on a schedule next to
low-priority batches issued back to back, on one GPU, through strait_submit / strait_wait.

The paper's evaluation is open loop (Section 5.1 "Workloads": each request is generated
independently of earlier completions) and measures a request from its arrival to the moment
its result is back in host memory (Section 5.1 "Evaluation Metrics"); its motivation study
co-locates one high-priority and one low-priority model at concurrency two (Section 2.1).
This module only drives the C ABI and collects the completion records; every step of the
request itself (staging, copies, kernels, timing) happens inside the library.
"""
from __future__ import annotations

import gc
import threading
import time
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

from . import binding as S


@dataclass
class StreamStats:
    requests: int = 0
    dropped: int = 0
    latency_ms: List[float] = field(default_factory=list)     # arrival -> host-observed completion
    kernel_ms: List[float] = field(default_factory=list)
    h2d_ms: List[float] = field(default_factory=list)
    total_ms: List[float] = field(default_factory=list)
    images: int = 0
    wall_s: float = 0.0

    def summary(self) -> dict:
        def pct(a, q):
            return round(float(np.percentile(a, q)), 4) if len(a) else None
        return {"requests": self.requests, "dropped": self.dropped,
                "latency_ms": {"p50": pct(self.latency_ms, 50), "p95": pct(self.latency_ms, 95), "p99": pct(self.latency_ms, 99),
                               "max": pct(self.latency_ms, 100)},
                "kernel_ms": {"p50": pct(self.kernel_ms, 50), "p95": pct(self.kernel_ms, 95), "p99": pct(self.kernel_ms, 99)},
                "h2d_ms": {"p50": pct(self.h2d_ms, 50), "p99": pct(self.h2d_ms, 99)},
                "images_per_s": round(self.images / self.wall_s, 1) if self.wall_s > 0 else None}


def _back_to_back(model, prio, xs, valid_len, stop: threading.Event, stats: StreamStats):
    """Closed loop: the next batch is submitted when the previous one has completed."""
    batch = xs[0].shape[0]
    out = model.new_output(batch)
    t0 = time.monotonic()
    i = 0
    while not stop.is_set():
        x = xs[i % len(xs)]
        t_arr = time.monotonic_ns()
        rec = model.wait(model.submit(prio, x, valid_len, out))
        stats.requests += 1
        stats.images += batch
        stats.latency_ms.append((rec.t_done_ns - t_arr) * 1e-6)
        stats.kernel_ms.append(rec.kernel_ms)
        stats.h2d_ms.append(rec.h2d_ms)
        stats.total_ms.append(rec.total_ms)
        i += 1
    stats.wall_s = time.monotonic() - t0


def _open_loop(model, prio, xs, arrivals_ns: np.ndarray, stats: StreamStats):
    """Open loop: request k is submitted at t0 + arrivals_ns[k] whatever happened to earlier ones;
    a request that finds every instance busy is dropped and counted."""
    batch = xs[0].shape[0]
    outs = [model.new_output(batch) for _ in range(model.n_instances)]
    free_outs = list(range(len(outs)))
    pending = []                                  # (ticket, arrival time, out index)
    t0 = time.monotonic_ns() + 2_000_000

    def harvest(block: bool):
        for item in list(pending):
            tk, t_arr, oi = item
            if block or model.poll(tk):
                rec = model.wait(tk)
                stats.latency_ms.append((rec.t_done_ns - t_arr) * 1e-6)
                stats.kernel_ms.append(rec.kernel_ms)
                stats.h2d_ms.append(rec.h2d_ms)
                stats.total_ms.append(rec.total_ms)
                stats.images += batch
                pending.remove(item)
                free_outs.append(oi)

    for k, a in enumerate(arrivals_ns):
        t_arr = t0 + int(a)
        while True:
            now = time.monotonic_ns()
            if now >= t_arr:
                break
            harvest(False)
            if t_arr - time.monotonic_ns() > 300_000:
                time.sleep(0.0001)
        stats.requests += 1
        if not free_outs:
            harvest(False)
        tk = None
        if free_outs:
            oi = free_outs.pop()
            tk = model.try_submit(prio, xs[k % len(xs)], None, outs[oi])
            if tk is None:
                free_outs.append(oi)
        if tk is None:
            stats.dropped += 1
        else:
            pending.append((tk, t_arr, oi))
    harvest(True)
    stats.wall_s = (time.monotonic_ns() - t0) * 1e-9


def run(hp_model, hp_inputs, arrivals_ns, lp_model, lp_inputs, mode: str = "both", lp_solo_s: float = 1.0):
    """mode: 'hp_solo' (arrivals only), 'lp_solo' (back-to-back only, for lp_solo_s seconds) or
    'both'.  Returns (hp StreamStats or None, lp StreamStats or None)."""
    hp, lp = (StreamStats() if mode != "lp_solo" else None), (StreamStats() if mode != "hp_solo" else None)
    stop = threading.Event()
    th: Optional[threading.Thread] = None
    gc_was_on = gc.isenabled()
    gc.disable()                                  # a collection pause in the submitting thread would show up as request latency
    if lp is not None:
        th = threading.Thread(target=_back_to_back, args=(lp_model, S.PRIO_LOW, lp_inputs, None, stop, lp), daemon=True)
        th.start()
        time.sleep(0.05)                          # let the low-priority stream reach steady state
    try:
        if hp is not None:
            _open_loop(hp_model, S.PRIO_HIGH, hp_inputs, arrivals_ns, hp)
        else:
            time.sleep(lp_solo_s)
    finally:
        stop.set()
        if th is not None:
            th.join()
        if gc_was_on:
            gc.enable()
    return hp, lp
