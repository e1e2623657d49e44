#!/usr/bin/env python3
"""Throughput of the served hot path on one MI355X.

A step is one pass of the whole kernel sequence of a batch (every layer of the plan, through
the C ABI's strait_run) over a synthetic ResNet-50 v1.5 batch of 128 fp16 224x224 images whose
input already sits in device memory.  Prints ONE JSON line:

  value         images/s over the K timed steps
  roofline      the implicit-GEMM convolution kernels (53 convolutions + FC per step; the stem convolution
                is a kernel of its own, fused with the max pooling): algorithmic
                flops of those launches divided by their device time.  Device time = HIP events
                around the K timed steps on the launch stream, minus the non-convolution kernels'
                time; a second pass of K steps with an event pair around every layer supplies the
                latter and the per-layer split (event pairs open gaps between launches, so they
                are kept out of the pass `value` is taken from)
  cpu_baseline  the CPU oracle's ResNet-50 forward timed on this host on a bounded sample
  by_batch      the other batch sizes of the workload (1, 8, 32; the paper serves at batch <= 8, Section 5.1), shorter runs:
                images/s, ms per step, TFLOP/s, and the fraction of the layer-wise roofline (sum over the layers of
                max(flops / MFMA peak, bytes / HBM peak)) at that batch size
  hbm_kernels   the bandwidth-bound kernels (depthwise convolution, pooling, softmax in MobileNetV2 b64; LayerNorm in the
                encoder b64): algorithmic bytes / per-layer event time, as GB/s and as a fraction of the HBM peak;
                depthwise_conv3x3_kernel_alone: that kernel through its C-ABI hook on the three largest depthwise layers
  two_instances images/s when the same K steps are issued alternately to two instances of the model on
                the two compute streams (the paper's servers run several instances at once); not `value`
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
# The co-location phase uses five streams; with HIP's default of 4 hardware queues per process two
# of them would share a queue and serialise.  Must be set before the HIP runtime initialises.
os.environ.setdefault("GPU_MAX_HW_QUEUES", "8")

MFMA_F16_PEAK_TFLOPS = 2500.0      # MI355X dense fp16 matrix peak
HBM_PEAK_GBS = 8000.0


TRAFFIC_FILE = "profiles/traffic_conv_igemm_resnet50_b128.json"


def measured_traffic(batch):
    """HBM bytes per step of the convolution launches from the committed hardware-counter runs (TRAFFIC_FILE: this
    process does not read counters), or None when a kernel source has changed since they were taken (or the workload
    differs)."""
    import hashlib
    try:
        rec = json.load(open(os.path.join(ROOT, TRAFFIC_FILE)))
        for src in rec["kernel_sources"]:
            if hashlib.sha256(open(os.path.join(ROOT, src["path"]), "rb").read()).hexdigest() != src["sha256"]:
                return None
    except (OSError, ValueError, KeyError, TypeError):
        return None
    if batch != 128:
        return None
    return rec.get("hbm_bytes_per_step")


def colocation(ctx, md_resnet, blob_resnet, seconds):
    """High-priority ResNet-50 b8 requests, Poisson at 200/s, next to low-priority MobileNetV2 b64
    issued back to back; per-request latency solo vs co-located, with and without wave priority."""
    import synth
    from paper_2604_28175_amd import colocate

    seed = synth.SEEDS["colocation"]
    hp = ctx.load(blob_resnet, max_batch=8, n_instances=4)
    md_lp = synth.mobilenet_v2(synth.SEEDS[synth.ARCH_MOBILENETV2])
    lp = ctx.load(synth.pack(md_lp), max_batch=64, n_instances=1)
    hp_x = [synth.default_image_batch(md_resnet, 8, seed + i) for i in range(4)]
    lp_x = [synth.default_image_batch(md_lp, 64, seed + 100 + i) for i in range(2)]
    arrivals = synth.poisson_arrivals_ns(seed, 200.0, seconds)
    res = {"hp": "resnet50_v1.5 b8, Poisson 200 req/s, open loop", "lp": "mobilenet_v2 b64, back to back",
           "seconds_per_phase": seconds}
    colocate.run(hp, hp_x, arrivals[:50], lp, lp_x, "hp_solo")            # warm-up
    h, _ = colocate.run(hp, hp_x, arrivals, lp, lp_x, "hp_solo")
    res["hp_solo"] = h.summary()
    _, l = colocate.run(hp, hp_x, arrivals, lp, lp_x, "lp_solo", lp_solo_s=min(seconds, 3.0))
    res["lp_solo"] = l.summary()
    h, l = colocate.run(hp, hp_x, arrivals, lp, lp_x, "both")
    res["colocated"] = {"hp": h.summary(), "lp": l.summary()}
    ctx.set_wave_priority(False)
    h, l = colocate.run(hp, hp_x, arrivals, lp, lp_x, "both")
    res["colocated_no_wave_priority"] = {"hp": h.summary(), "lp": l.summary()}
    ctx.set_wave_priority(True)
    # the low-priority batches issued in segments of four layers that yield while a high-priority batch is in flight
    ctx.set_lp_yield(4)
    h, l = colocate.run(hp, hp_x, arrivals, lp, lp_x, "both")
    res["colocated_lp_yield_4"] = {"hp": h.summary(), "lp": l.summary()}
    ctx.set_lp_yield(0)
    solo, co, coy = res["hp_solo"]["latency_ms"], res["colocated"]["hp"]["latency_ms"], res["colocated_lp_yield_4"]["hp"]["latency_ms"]
    res["hp_p99_colocated_over_solo"] = round(co["p99"] / solo["p99"], 3)
    res["hp_p50_colocated_over_solo"] = round(co["p50"] / solo["p50"], 3)
    res["hp_p99_colocated_over_solo_lp_yield_4"] = round(coy["p99"] / solo["p99"], 3)
    res["hp_p50_colocated_over_solo_lp_yield_4"] = round(coy["p50"] / solo["p50"], 3)
    res["lp_images_per_s_lp_yield_4_over_default"] = round(res["colocated_lp_yield_4"]["lp"]["images_per_s"] / res["colocated"]["lp"]["images_per_s"], 3)
    hp.free()
    lp.free()
    return res


def serving(ctx, md_resnet, blob_resnet, seconds, hp_rate, lp_rate):
    """The whole of the paper's system on one GPU: single requests for a high-priority ResNet-50 and a
    low-priority MobileNetV2 on Poisson schedules through the front end (maximum batch 8, four batches in
    flight, batch formation timeout a tenth of the deadline: Section 5.1), first the high-priority model
    alone, then both, then both with twice the low-priority rate (more than its one stream can serve)."""
    import synth
    import paper_2604_28175_amd as strait
    from paper_2604_28175_amd import serve

    seed = synth.SEEDS["colocation"] + 7
    hp = ctx.load(blob_resnet, max_batch=8, n_instances=4)
    md_lp = synth.mobilenet_v2(synth.SEEDS[synth.ARCH_MOBILENETV2])
    lp = ctx.load(synth.pack(md_lp), max_batch=8, n_instances=4)
    sched = strait.Scheduler(1)
    prof = {1: serve.offline_profiles(hp, strait.PRIO_HIGH, 8), 2: serve.offline_profiles(lp, strait.PRIO_LOW, 8)}
    sched.set_profile(1, strait.PRIO_HIGH, serve.profile_tuples(prof[1]))
    sched.set_profile(2, strait.PRIO_LOW, serve.profile_tuples(prof[2]))
    cfg = {1: dict(model=hp, prio=strait.PRIO_HIGH, rate=hp_rate, deadline_ms=5.0),
           2: dict(model=lp, prio=strait.PRIO_LOW, rate=lp_rate, deadline_ms=25.0)}
    xs = {1: list(synth.default_image_batch(md_resnet, 8, seed)), 2: list(synth.default_image_batch(md_lp, 8, seed + 1))}
    res = {"hp": f"resnet50_v1.5, single requests, Poisson {hp_rate:.0f}/s, deadline 5 ms",
           "lp": f"mobilenet_v2, single requests, Poisson {lp_rate:.0f}/s, deadline 25 ms",
           "max_batch": 8, "concurrency": 4, "seconds_per_phase": seconds,
           "profile_ms": {name: {"b1": [round(p[0].t_inf_isol_ns * 1e-6, 3), round(p[0].t_kernel_isol_ns * 1e-6, 3)],
                                 "b8": [round(p[7].t_inf_isol_ns * 1e-6, 3), round(p[7].t_kernel_isol_ns * 1e-6, 3)],
                                 "demand_b8": [round(v, 3) for v in p[7].m]} for name, p in (("hp", prof[1]), ("lp", prof[2]))}}
    ctx.set_graphs(True)      # a batch's kernel sequence is replayed from a captured graph: a fifth of the host time per submit
    for phase, mids, lp_scale in (("hp_alone", (1,), 1.0), ("hp_and_lp", (1, 2), 1.0), ("hp_and_lp_overload", (1, 2), 2.0)):
        srv = strait.Server(sched, 4, 200_000)
        for mid in mids:
            c = cfg[mid]
            srv.add_model(c["model"], mid, c["prio"], 8, int(c["deadline_ms"] * 1e6), int(c["deadline_ms"] * 1e5))
        srv.start()
        streams = {mid: {"model": cfg[mid]["model"], "inputs": xs[mid],
                         "arrivals_ns": synth.poisson_arrivals_ns(seed + mid, cfg[mid]["rate"] * (lp_scale if mid == 2 else 1.0), seconds)}
                   for mid in mids}
        summ = serve.run_open_loop(srv, streams, seconds)
        st = srv.stats()
        srv.close()
        res[phase] = {("hp" if mid == 1 else "lp"): summ[mid] for mid in mids}
        res[phase]["batches"] = st.batches
        res[phase]["max_in_flight"] = st.max_in_flight
        res[phase]["deferrals"] = st.deferrals
    ctx.set_graphs(False)
    sched.close()
    hp.free()
    lp.free()
    return res


def serving_mixed(models_data, seconds, scale):
    """The paper's heterogeneous workload by shape (Table 1: model, priority, deadline) on one GPU: ResNet-50 (high,
    8 ms), ViT-B/16 (high, 15 ms), VGG-19 (low, 25 ms) and a BERT-base-shaped encoder standing in for RoBERTa-B
    (low, 45 ms), single requests on independent Poisson schedules, maximum batch 8, four batches in flight, batch
    formation timeout a tenth of the deadline (Section 5.1)."""
    import synth
    import paper_2604_28175_amd as strait
    from paper_2604_28175_amd import serve

    seed = synth.SEEDS["colocation"] + 11
    table = {1: ("resnet50", synth.ARCH_RESNET50, strait.PRIO_HIGH, 8.0, 2000.0),
             2: ("vit_b16", synth.ARCH_VIT, strait.PRIO_HIGH, 15.0, 1200.0),
             3: ("vgg19", synth.ARCH_VGG19, strait.PRIO_LOW, 25.0, 1200.0),
             4: ("encoder", synth.ARCH_ENCODER, strait.PRIO_LOW, 45.0, 1500.0)}
    # four batches in flight need four compute streams to run side by side: two per priority level
    ctx = strait.Context(device=0, n_hp=2, n_lp=2, n_copy=2)
    sched = strait.Scheduler(1)
    srv = strait.Server(sched, 4, 200_000)
    ctx.set_graphs(True)
    loaded, streams = {}, {}
    for mid, (name, arch, prio, deadline_ms, rate) in table.items():
        md, blob = models_data(arch)
        m = ctx.load(blob, max_batch=8, n_instances=3)
        loaded[mid] = m
        sched.set_profile(mid, prio, serve.profile_tuples(serve.offline_profiles(m, prio, 8, reps=20)))
        srv.add_model(m, mid, prio, 8, int(deadline_ms * 1e6), int(deadline_ms * 1e5))
        if arch == synth.ARCH_ENCODER:
            xs, _ = synth.token_batch(md, 8, seed + mid)
            streams[mid] = {"model": m, "inputs": list(xs), "valid_len": 96}
        else:
            streams[mid] = {"model": m, "inputs": list(synth.default_image_batch(md, 8, seed + mid))}
        streams[mid]["arrivals_ns"] = synth.poisson_arrivals_ns(seed + mid, rate * scale, seconds)
    srv.start()
    summ = serve.run_open_loop(srv, streams, seconds)
    st = srv.stats()
    srv.close()
    sched.close()
    for m in loaded.values():
        m.free()
    ctx.close()
    res = {name: dict(priority="high" if prio == strait.PRIO_HIGH else "low", deadline_ms=deadline_ms, rate_per_s=rate * scale, **summ[mid])
           for mid, (name, arch, prio, deadline_ms, rate) in table.items()}
    res.update(seconds=seconds, batches=st.batches, max_in_flight=st.max_in_flight, deferrals=st.deferrals)
    return res


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--batch", type=int, default=128)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-by-batch", action="store_true")
    ap.add_argument("--no-gpu-state", action="store_true", help="skip the extra passes during which clocks are read (profiling runs count passes)")
    ap.add_argument("--no-other-models", action="store_true", help="skip the throughput lines of the other served models (VGG-19, ViT-B/16, MobileNetV2, encoder)")
    ap.add_argument("--only-model", choices=("vgg19", "vit_b16", "mobilenet_v2", "encoder"), default=None,
                    help="time nothing but this model at batch 64 (for kernel profiles of the second workload set)")
    ap.add_argument("--single-stream", action="store_true",
                    help="keep the projection shortcuts on the main stream (kernel traces of such a run add up to the step time)")
    ap.add_argument("--colocation-seconds", type=float, default=10.0,
                    help="length of each phase of the dual-priority co-location run (0 = skip)")
    ap.add_argument("--serving-seconds", type=float, default=2.0,
                    help="seconds per phase of the request-level serving run (0 = skip)")
    ap.add_argument("--serving-mixed-scale", type=float, default=1.0, help="multiplies the request rates of the four-model serving phase")
    ap.add_argument("--serving-hp-rate", type=float, default=4000.0, help="high-priority requests per second")
    ap.add_argument("--serving-lp-rate", type=float, default=10000.0, help="low-priority requests per second")
    ap.add_argument("--copy-calibration-mb", type=int, default=0,
                    help="also run one plain device copy of this many MiB (reference for hardware byte counters)")
    ap.add_argument("--cpu-sample", type=int, default=0, help="images the CPU oracle is timed on (0 = twelve per thread)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library serves from one GPU (the served path has no collectives); run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2604_28175_amd as strait
    import synth

    B, K, W = args.batch, args.steps, args.warmup
    seed = synth.SEEDS[synth.ARCH_RESNET50]
    md = synth.resnet50(seed)
    blob = synth.pack(md)
    ctx = strait.Context(device=0, n_hp=1, n_lp=1, n_copy=2)
    if args.single_stream:
        ctx.set_branch_streams(False)
    model = ctx.load(blob, max_batch=B, n_instances=1)
    x = synth.default_image_batch(md, B, seed + B)
    prio = strait.PRIO_HIGH
    model.copy_in(0, prio, x)
    model.sync(0, prio)
    torch.cuda.synchronize()

    stream = ctx.hp_streams[0]                    # the stream strait_run launches on at high priority
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(m, batch, steps, warmup):
        for _ in range(warmup):
            m.run(0, prio, batch)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev0.record(stream)
        for _ in range(steps):
            m.run(0, prio, batch)
        ev1.record(stream)
        torch.cuda.synchronize()
        return time.perf_counter() - t0, ev0.elapsed_time(ev1)

    data_cache = {synth.ARCH_RESNET50: (md, blob)}

    def models_data(arch):
        """(seeded tensors, weight container) of an architecture, generated once per run."""
        if arch not in data_cache:
            amd = synth.make_model(arch, synth.SEEDS[arch])
            data_cache[arch] = (amd, synth.pack(amd))
        return data_cache[arch]

    def other_model(arch, steps=20, warmup=5):
        omd, oblob = models_data(arch)
        om = ctx.load(oblob, max_batch=64, n_instances=1)
        if arch == synth.ARCH_ENCODER:
            tokens, valid = synth.token_batch(omd, 64, 5)      # (`valid` is also what the attention flops are counted with)
            om.copy_in(0, prio, tokens, valid)
        else:
            om.copy_in(0, prio, synth.default_image_batch(omd, 64, 5))
        om.sync(0, prio)
        odt, odev = timed(om, 64, steps, warmup)
        olayers = om.layers()
        # multiply-accumulates of the batch; attention counts what is computed: every query against the valid keys only
        macs = 0.0
        for l in olayers:
            if l.kind == 5 and arch == synth.ARCH_ENCODER:
                macs += float(l.macs_per_sample) * float(valid.sum()) / omd.hyper[4]
            else:
                macs += float(l.macs_per_sample) * 64
        step_s = odev / steps * 1e-3
        nbytes = sum(float(l.bytes_per_sample) * 64 + l.weight_bytes for l in olayers)
        t_roof = sum(max(2.0 * l.macs_per_sample * 64 / (MFMA_F16_PEAK_TFLOPS * 1e12),
                         (float(l.bytes_per_sample) * 64 + l.weight_bytes) / (HBM_PEAK_GBS * 1e9)) for l in olayers)
        res = {"batch": 64, "images_per_s": round(steps * 64 / odt, 1), "ms_per_step": round(odt / steps * 1e3, 4),
               "tflops": round(2.0 * macs / step_s / 1e12, 1),
               "frac_of_mfma_peak": round(2.0 * macs / step_s / 1e12 / MFMA_F16_PEAK_TFLOPS, 4),
               "algorithmic_gbs": round(nbytes / step_s / 1e9, 1),
               "frac_of_hbm_peak": round(nbytes / step_s / 1e9 / HBM_PEAK_GBS, 4),
               "bound": "hbm" if nbytes / (HBM_PEAK_GBS * 1e9) > 2.0 * macs / (MFMA_F16_PEAK_TFLOPS * 1e12) else "mfma",
               "layerwise_roofline_ms": round(t_roof * 1e3, 4), "frac_of_layerwise_roofline": round(t_roof / step_s, 4)}
        if arch in (synth.ARCH_MOBILENETV2, synth.ARCH_ENCODER):
            # the bandwidth-bound kernels one by one: an event pair around every layer (a few microseconds of gap per
            # layer are booked to the kernels this way, so these are lower bounds of the kernels' own rates)
            lms = np.zeros(len(olayers))
            for _ in range(steps):
                lms += om.run_timed(0, prio, 64)
            lms /= steps
            kinds = {1: "depthwise_conv3x3", 2: "pooling", 3: "softmax", 4: "layernorm"}
            hk = {}
            for i, l in enumerate(olayers):
                if l.kind in kinds and l.bytes_per_sample > 0 and lms[i] == 0.0:
                    # computed inside another layer's launch at this batch size (run_timed gives exactly 0): not a launch
                    hk.setdefault(kinds[l.kind], {"launches": 0, "bytes": 0.0, "ms": 0.0, "best_gbs": 0.0}).setdefault("fused_into_other_launches", 0)
                    hk[kinds[l.kind]]["fused_into_other_launches"] += 1
                elif l.kind in kinds and l.bytes_per_sample > 0:
                    e = hk.setdefault(kinds[l.kind], {"launches": 0, "bytes": 0.0, "ms": 0.0, "best_gbs": 0.0})
                    by = float(l.bytes_per_sample) * 64 + l.weight_bytes
                    e["launches"] += 1
                    e["bytes"] += by
                    e["ms"] += float(lms[i])
                    e["best_gbs"] = max(e["best_gbs"], by / (float(lms[i]) * 1e-3) / 1e9)
            for e in hk.values():
                e["gbs"] = round(e["bytes"] / (e["ms"] * 1e-3) / 1e9, 1)
                e["frac_of_hbm_peak"] = round(e["gbs"] / HBM_PEAK_GBS, 4)
                e["best_layer_gbs"] = round(e.pop("best_gbs"), 1)
                e["best_layer_frac_of_hbm_peak"] = round(e["best_layer_gbs"] / HBM_PEAK_GBS, 4)
                e["ms"] = round(e["ms"], 4)
                e["bytes"] = int(e["bytes"])
            if arch == synth.ARCH_MOBILENETV2:
                # The depthwise kernel by itself on the network's three largest depthwise layers (two of which the plan runs
                # inside other launches at this batch size): the C ABI's kernel hook on seeded random tensors, three sets of
                # buffers in rotation (0.3 to 0.6 GB: more than the 256 MB memory-side cache holds), stream events around 24 launches.
                alone = {}
                for name, hh, cc, st in (("b0.dw 112x112x32 s1", 112, 32, 1), ("b1.dw 112x112x96 s2", 112, 96, 2), ("b2.dw 56x56x144 s1", 56, 144, 1)):
                    g = torch.Generator(device="cuda").manual_seed(1234)
                    xs = [torch.randn((64, hh, hh, cc), generator=g, device="cuda", dtype=torch.float16) for _ in range(3)]
                    wd = torch.randn((3, 3, cc), generator=g, device="cuda", dtype=torch.float16) * 0.4
                    bd = torch.randn((cc,), generator=g, device="cuda", dtype=torch.float32)
                    pq = (hh - 1) // st + 1
                    ys = [torch.empty((64, pq, pq, cc), device="cuda", dtype=torch.float16) for _ in range(3)]
                    sp = torch.cuda.current_stream().cuda_stream

                    def dw(i):
                        strait.binding._check(strait.lib.strait_k_dwconv3x3(sp, xs[i % 3].data_ptr(), 64, hh, hh, cc, wd.data_ptr(), bd.data_ptr(),
                                                                           st, 2, ys[i % 3].data_ptr(), 0))
                    for i in range(6):
                        dw(i)
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    for i in range(24):
                        dw(i)
                    e1.record()
                    torch.cuda.synchronize()
                    us = e0.elapsed_time(e1) / 24 * 1e3
                    by = 2.0 * 64 * cc * (hh * hh + pq * pq)
                    alone[name] = {"us": round(us, 2), "gbs": round(by / us / 1e3, 1), "frac_of_hbm_peak": round(by / us / 1e3 / HBM_PEAK_GBS, 4)}
                    del xs, ys
                hk["depthwise_conv3x3_kernel_alone"] = alone
            res["hbm_kernels"] = hk
        om.free()
        return res

    if args.copy_calibration_mb > 0:
        src = torch.empty(args.copy_calibration_mb << 20, dtype=torch.uint8, device="cuda").zero_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # (for the encoder an "image" is a 128-token sequence with a seeded valid length)
    others = {"vgg19": synth.ARCH_VGG19, "vit_b16": synth.ARCH_VIT, "mobilenet_v2": synth.ARCH_MOBILENETV2, "encoder": synth.ARCH_ENCODER}
    if args.only_model:
        # profiling aid: nothing but this model's steps is launched (no ResNet-50 step, no headline value)
        print(json.dumps({"only_model": args.only_model, "steps": K, "warmup": W, **other_model(others[args.only_model], K, W)}))
        model.free()
        ctx.close()
        return 0

    dt, dev_ms = timed(model, B, K, W)
    value = K * B / dt

    # clock and power while the same steps run (a second, untimed pass: the query itself takes about as long as K steps)
    def gpu_state_under_load():
        import subprocess
        try:
            for _ in range(3 * K):
                model.run(0, prio, B)
            r = subprocess.run(["rocm-smi", "--showclocks", "--showpower", "--json"], capture_output=True, text=True, timeout=20)
            torch.cuda.synchronize()
            card = next(iter(json.loads(r.stdout[r.stdout.index("{"):]).values()))
            return {k.strip(": ").replace(" ", "_"): v for k, v in card.items()}
        except Exception as e:                    # no such tool, no permission, unexpected format: the figure is optional
            torch.cuda.synchronize()
            return {"unavailable": type(e).__name__}

    # ---- roofline of the dominant kernel (implicit-GEMM convolution), per-layer event pairs
    layers = model.layers()
    ms = np.zeros(len(layers))
    for _ in range(K):
        ms += model.run_timed(0, prio, B)
    ms /= K
    conv = [i for i, l in enumerate(layers) if l.kind == 0]
    conv_flops = sum(2.0 * layers[i].macs_per_sample * B for i in conv)
    # Device time of the convolution launches per step: the timed region's own device time (one HIP
    # event before and after the K steps, on the launch stream) minus the other kernels' time.  The
    # per-layer event pairs of the second pass only apportion it: an event pair around every launch
    # opens a gap of a few microseconds per launch, which would otherwise be booked to the kernels.
    other_ms = float(ms.sum()) - float(sum(ms[i] for i in conv))
    scale = (dev_ms / K - other_ms) / float(sum(ms[i] for i in conv))
    ms = np.array([ms[i] * scale if i in set(conv) else ms[i] for i in range(len(ms))])
    conv_ms = float(sum(ms[i] for i in conv))
    achieved = conv_flops / (conv_ms * 1e-3) / 1e12
    # per-class view: MFMA-bound layers (arithmetic intensity above the machine balance) vs the rest
    balance = MFMA_F16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)
    cls = {"mfma_bound": [0.0, 0.0, 0.0], "hbm_bound": [0.0, 0.0, 0.0]}
    t_roof = 0.0
    for i in conv:
        l = layers[i]
        fl = 2.0 * l.macs_per_sample * B
        by = float(l.bytes_per_sample) * B + l.weight_bytes
        key = "mfma_bound" if fl / by >= balance else "hbm_bound"
        cls[key][0] += fl
        cls[key][1] += by
        cls[key][2] += ms[i]
        t_roof += max(fl / (MFMA_F16_PEAK_TFLOPS * 1e12), by / (HBM_PEAK_GBS * 1e9))
    out = {
        "metric": "ResNet-50 fp16 images/s by batch; high-prio p99 latency solo vs co-located",
        "value": round(value, 1), "unit": "images/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(dt / K * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "gpu_state_under_load": None if args.no_gpu_state else gpu_state_under_load(),
        "config": {"workload": f"resnet50_v1.5 224x224 fp16 NHWC, batch {B}, BatchNorm folded, input resident in HBM",
                   "batch": B, "priority": "high"},
        "roofline": {"bound": "mfma", "achieved": round(achieved, 2), "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved / MFMA_F16_PEAK_TFLOPS, 4), "traffic": measured_traffic(B),
                     "traffic_source": TRAFFIC_FILE + " (rocprofv3 FETCH_SIZE and WRITE_SIZE runs of this command, committed; null when a kernel source has changed since)",
                     "algorithmic_bytes_per_step": sum(float(layers[i].bytes_per_sample) * B + layers[i].weight_bytes for i in conv),
                     "kernel": "conv_igemm_dma_kernel (all tile shapes), conv3x3_patch_kernel and its tile-walking form, pointwise_pair_wave_kernel and stem_pool_kernel: the MFMA launches of a step (53 convolutions and the classifier, in fewer launches than layers: the stem with the pooling and the first 1x1 convolution behind it, every projection shortcut inside its block's closing convolution, three block seams of the first stage as pairs)",
                     "flops_per_step": conv_flops, "kernel_ms_per_step": round(conv_ms, 4),
                     "other_kernels_ms_per_step": round(other_ms, 4),
                     "layerwise_roofline_ms": round(t_roof * 1e3, 4),
                     "frac_of_layerwise_roofline": round(t_roof * 1e3 / conv_ms, 4),
                     "classes": {k: {"tflops": round(v[0] / (v[2] * 1e-3) / 1e12, 2) if v[2] else None,
                                     "gbs": round(v[1] / (v[2] * 1e-3) / 1e9, 1) if v[2] else None,
                                     "ms": round(v[2], 4)} for k, v in cls.items()}},
    }

    def batch_line(b, images_per_s, step_ms):
        """Throughput of one batch size against its own layer-wise roofline (weights are read once per step whatever
        the batch, so small batches are weight-bound)."""
        fl = sum(2.0 * layers[i].macs_per_sample * b for i in conv)
        roof = sum(max(2.0 * l.macs_per_sample * b / (MFMA_F16_PEAK_TFLOPS * 1e12),
                       (float(l.bytes_per_sample) * b + l.weight_bytes) / (HBM_PEAK_GBS * 1e9)) for l in layers)
        return {"images_per_s": round(images_per_s, 1), "ms_per_step": round(step_ms, 4),
                "tflops": round(fl / (step_ms * 1e-3) / 1e12, 1), "frac_of_mfma_peak": round(fl / (step_ms * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS, 4),
                "layerwise_roofline_ms": round(roof * 1e3, 4), "frac_of_layerwise_roofline": round(roof * 1e3 / step_ms, 4)}

    if not args.no_by_batch:
        by = {str(B): batch_line(B, value, dev_ms / K)}
        for b in (32, 8, 1):
            if b >= B:
                continue
            xb = synth.default_image_batch(md, b, seed + b)
            model.copy_in(0, prio, xb)
            model.sync(0, prio)
            kb = max(20, K)
            d, dms = timed(model, b, kb, max(5, W))
            by[str(b)] = batch_line(b, kb * b / d, dms / kb)
        out["by_batch"] = by

    model.free()

    if not args.no_by_batch:
        # the same K steps, alternately on two instances (high- and low-priority stream): what one GPU serves
        # when two batches are in flight, as in the paper's instance pools
        pair = ctx.load(blob, max_batch=B, n_instances=2)
        for inst, pr in ((0, strait.PRIO_HIGH), (1, strait.PRIO_LOW)):
            pair.copy_in(inst, pr, x)
            pair.sync(inst, pr)
        for _ in range(W):
            pair.run(0, strait.PRIO_HIGH, B)
            pair.run(1, strait.PRIO_LOW, B)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(K):
            pair.run(k & 1, strait.PRIO_HIGH if (k & 1) == 0 else strait.PRIO_LOW, B)
        torch.cuda.synchronize()
        out["two_instances"] = {"images_per_s": round(K * B / (time.perf_counter() - t0), 1), "steps": K,
                                "note": "K steps alternating between two instances on two streams"}
        by2 = {}
        for b in (32, 8, 1):                       # the smaller batch sizes the same way: small batches gain most
            if b >= B:
                continue
            xb = synth.default_image_batch(md, b, seed + b)
            for inst, pr in ((0, strait.PRIO_HIGH), (1, strait.PRIO_LOW)):
                pair.copy_in(inst, pr, xb)
                pair.sync(inst, pr)
            kb = 2 * max(K, 100)
            for phase_steps in (20, kb):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for k in range(phase_steps):
                    pair.run(k & 1, strait.PRIO_HIGH if (k & 1) == 0 else strait.PRIO_LOW, b)
                torch.cuda.synchronize()
            by2[str(b)] = round(kb * b / (time.perf_counter() - t0), 1)
        out["two_instances"]["by_batch"] = by2
        for inst, pr in ((0, strait.PRIO_HIGH), (1, strait.PRIO_LOW)):
            pair.copy_in(inst, pr, x)
            pair.sync(inst, pr)
        # end to end: the batch waits in pinned host memory; submit -> H2D on a copy stream -> kernels -> D2H, two
        # instances double-buffering (the copy of one batch runs beside the kernels of the other)
        pipe = ctx.load(blob, max_batch=B, n_instances=4)
        stage = [pipe.staging(i, B) for i in range(4)]
        outs = [pipe.new_output(B) for _ in range(4)]
        for i in range(4):
            stage[i][:] = x
        tickets = [None] * 4
        def submit_e2e(k):
            i = k & 3
            if tickets[i] is not None:
                pipe.wait(tickets[i])
            tickets[i] = pipe.submit(strait.PRIO_HIGH if (k & 1) == 0 else strait.PRIO_LOW, stage[i], None, outs[i])
        def drain():
            for i in range(4):
                if tickets[i] is not None:
                    pipe.wait(tickets[i])
                    tickets[i] = None
        for k in range(8):
            submit_e2e(k)
        drain()
        t0 = time.perf_counter()
        for k in range(K):
            submit_e2e(k)
        drain()
        out["end_to_end"] = {"images_per_s": round(K * B / (time.perf_counter() - t0), 1), "steps": K,
                             "note": "pinned host input -> H2D -> kernels -> D2H through strait_submit, four instances in rotation on the two compute streams (a batch is resubmitted when its instance's previous batch has completed)"}
        pipe.free()
        pair.free()

    if not args.no_other_models:
        # the paper's other image classifiers by shape (Table 1): VGG-19 (all 3x3 convolutions, MFMA-bound) and
        # ViT-B/16 (197 tokens), batch 64, input resident, same timing as the headline value
        out["other_models"] = {name: other_model(arch) for name, arch in others.items()}
        out["hbm_kernels"] = {"mobilenet_v2_b64": out["other_models"]["mobilenet_v2"].pop("hbm_kernels"),
                              "encoder_b64": out["other_models"]["encoder"].pop("hbm_kernels"),
                              "peak_gbs": HBM_PEAK_GBS,
                              "note": "algorithmic bytes (input + output + parameters once) over per-layer event time"}

    if args.colocation_seconds > 0:
        out["colocation"] = colocation(ctx, md, blob, args.colocation_seconds)
    if args.serving_seconds > 0:
        out["serving"] = serving(ctx, md, blob, args.serving_seconds, args.serving_hp_rate, args.serving_lp_rate)
    ctx.close()
    if args.serving_seconds > 0 and not args.no_other_models:
        out["serving_mixed"] = serving_mixed(models_data, args.serving_seconds, args.serving_mixed_scale)

    if not args.no_cpu_baseline:
        from oracle import models as omodels
        from oracle import ops as oops
        threads = oops.num_threads()
        n = args.cpu_sample or 12 * threads
        chunk = min(n, 2 * threads)
        xs = synth.default_image_batch(md, chunk, seed + 1000)
        done, t0 = 0, time.perf_counter()
        while done < n:
            omodels.resnet50_forward(md.tensors, xs)
            done += chunk
        cdt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(done / cdt, 3), "unit": "images/s", "cores": threads, "kind": "oracle",
                               "sample": f"{done} images of the same workload through the fp64 oracle in forwards of {chunk} ({cdt:.1f} s)"}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
