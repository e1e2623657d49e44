"""Open-loop load on the serving front end: single requests for several models arrive on seeded Poisson
schedules (Section 5.1 of the paper, "Workloads": stochastic arrivals, open model), the front end batches,
schedules and runs them, and the per-request records give what the paper reports: deadline-violation rate
(dropped requests count as violations), goodput (requests per second that met their deadline) and latency
from enqueue to result.  This module only issues requests and summarises records; queues, batching,
scheduling and execution are the library's.
"""
from __future__ import annotations

import gc
import time
from typing import Dict, List

import numpy as np

from . import binding as S


def offline_profiles(model: "S.Model", prio: int, max_batch: int, reps: int = 30) -> List["S.BatchProfile"]:
    """Isolated p95 latencies and resource demand for batch sizes 1..max_batch (Section 3.2)."""
    return [S.profile_model(model, prio, b, reps) for b in range(1, max_batch + 1)]


def profile_tuples(profs):
    return [(p.t_inf_isol_ns, p.t_htod_ns, p.t_kernel_isol_ns, list(p.m), p.m_self_cmp, p.m_self_mem) for p in profs]


def run_open_loop(server: "S.Server", streams: Dict[int, dict], seconds: float) -> Dict[int, dict]:
    """streams: {model_id: {"model": Model, "arrivals_ns": int64[], "inputs": [one-sample arrays], "valid_len": int}}.
    Issues request k of a model at t0 + arrivals_ns[k] whatever happened to earlier ones; returns a summary per
    model id."""
    events = sorted((int(t), mid) for mid, s in streams.items() for t in s["arrivals_ns"])
    ring = 4096
    outs = {mid: [s["model"].new_output(1) for _ in range(ring)] for mid, s in streams.items()}
    count = {mid: 0 for mid in streams}
    recs = []
    gc_was_on = gc.isenabled()
    gc.disable()
    try:
        t0 = time.monotonic_ns() + 2_000_000
        for k, (t, mid) in enumerate(events):
            t_arr = t0 + t
            while True:
                left = t_arr - time.monotonic_ns()
                if left <= 0:
                    break
                if left > 300_000:
                    time.sleep(0.0001)
            s = streams[mid]
            i = count[mid]
            count[mid] = i + 1
            server.request(mid, s["inputs"][i % len(s["inputs"])], outs[mid][i % ring], s.get("valid_len", 0))
            if (k & 1023) == 1023:
                recs.extend(server.results())
        server.wait_idle(30.0)
        wall_s = (time.monotonic_ns() - t0) * 1e-9
        recs.extend(server.results())
    finally:
        if gc_was_on:
            gc.enable()
    out = {}
    for mid in streams:
        rs = [r for r in recs if r.model_id == mid]
        lat = np.array([(r.t_done_ns - r.t_enqueue_ns) * 1e-6 for r in rs if r.status == 0])
        ok = sum(1 for r in rs if not r.violated)
        served = [r for r in rs if r.status == 0]
        batches = {r.batch_seq: r.batch for r in served}

        def pct(q):
            return round(float(np.percentile(lat, q)), 4) if lat.size else None
        out[mid] = {"requests": len(rs), "served": len(served), "dropped": sum(1 for r in rs if r.status == 1),
                    "violation_rate": round(1.0 - ok / max(1, len(rs)), 5),
                    "goodput_per_s": round(ok / max(wall_s, 1e-9), 1),
                    "latency_ms": {"p50": pct(50), "p95": pct(95), "p99": pct(99), "max": pct(100)},
                    "mean_batch": round(float(np.mean(list(batches.values()))), 3) if batches else None,
                    "mean_abs_prediction_error_ms": round(float(np.mean([abs(r.t_inf_pred_ns - (r.t_done_ns - r.t_enqueue_ns))
                                                                         for r in served if r.position == 0])) * 1e-6, 4) if served else None}
    return out
