"""GPU parity, end to end: every served architecture through the C ABI (submit at a priority ->
pinned H2D -> kernel sequence -> D2H -> record) against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest

import synth
from oracle import models as omodels
from parity import check_kernel, check_logits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    import paper_2604_28175_amd as strait
    c = strait.Context(device=0, n_hp=1, n_lp=1, n_copy=2)
    c.S = strait
    yield c
    c.close()


def run_cnn(ctx, md, x, fwd, prio, what):
    S = ctx.S
    m = ctx.load(synth.pack(md), max_batch=x.shape[0], n_instances=1)
    try:
        out, rec = m.infer(x, prio=prio)
        ref = fwd(md.tensors, x)
        err, scale, ties = check_logits(out["logits"], ref.logits, out["top1"], what)
        assert np.abs(out["probs"] - ref.probs).max() <= 2e-2
        assert np.abs(out["probs"].sum(-1) - 1).max() < 1e-4
        assert rec.batch == x.shape[0] and rec.priority == prio
        assert rec.h2d_ms > 0 and rec.kernel_ms > 0 and rec.total_ms >= rec.kernel_ms
        assert rec.t_enqueue_ns <= rec.t_issued_ns <= rec.t_done_ns
        print(f"{what}: max|err| {err:.3e} of scale {scale:.3e} ({err / scale:.2e}), ties {ties}, kernels {rec.kernel_ms:.3f} ms")
        return m, out, ref
    except Exception:
        m.free()
        raise


def test_tiny_cnn_config(ctx):
    md = synth.tiny_cnn(synth.SEEDS[synth.ARCH_TINY_CNN])
    x = synth.default_image_batch(md, 4, synth.SEEDS[synth.ARCH_TINY_CNN] + 4)
    m, out, ref = run_cnn(ctx, md, x, omodels.tiny_cnn_forward, ctx.S.PRIO_HIGH, "tiny CNN b4")
    # zero input: zero biases -> logits exactly 0, uniform probabilities
    z, _ = m.infer(np.zeros_like(x))
    assert not z["logits"].any() and np.allclose(z["probs"], 0.1, atol=1e-6) and not z["top1"].any()
    m.free()


@pytest.mark.parametrize("hw,batch", [(64, 5), (224, 2)])
def test_resnet50(ctx, hw, batch):
    md = synth.resnet50(synth.SEEDS[synth.ARCH_RESNET50], hw=hw)
    x = synth.default_image_batch(md, batch, synth.SEEDS[synth.ARCH_RESNET50] + batch)
    m, out, ref = run_cnn(ctx, md, x, omodels.resnet50_forward, ctx.S.PRIO_HIGH, f"ResNet-50 {hw}px b{batch}")
    m.free()


def test_resnet50_layers_and_batch_independence(ctx):
    """Every layer's activation against the oracle's (catches wiring errors that cancel in the
    logits), and sample i of a batch equals the same image run alone."""
    md = synth.resnet50(3, hw=64)
    x = synth.default_image_batch(md, 3, 8)
    m = ctx.load(synth.pack(md), max_batch=3, n_instances=1)
    ref = omodels.resnet50_forward(md.tensors, x, keep=True)
    m.copy_in(0, ctx.S.PRIO_LOW, x)
    names = {}
    for i, li in enumerate(m.layers()):
        names[li.name.decode()] = i
    checked = 0
    for lname, act in ref.trace.acts.items():
        key = lname.replace(".out", ".c3")       # the fused epilogue of c3 produces the block output
        if lname.endswith(".c3") or key not in names or lname in ("fc",):
            continue
        got = m.read_activation(0, names[key], 3).astype(np.float64).reshape(act.shape)
        check_kernel(got, act, f"layer {lname}", rel=2.0 ** -8, abs_rel=1e-2)
        checked += 1
    assert checked >= 40
    full, _ = m.infer(x, prio=ctx.S.PRIO_LOW)
    for i in range(3):
        one, _ = m.infer(x[i:i + 1], prio=ctx.S.PRIO_LOW)
        assert np.abs(one["logits"][0] - full["logits"][i]).max() <= 1e-3 * np.abs(full["logits"]).max()
        assert one["top1"][0] == full["top1"][i]
    m.free()


def test_resnet50_fused_block_seams_equal_separate_launches(ctx):
    """The closing 1x1 of a bottleneck and the opening 1x1 of the next one as one launch (forced at every size here,
    ragged tiles included) give the logits of the layer-by-layer plan bit for bit, and the oracle's within tolerance."""
    md = synth.resnet50(5)            # full size, six images: no layer of a fused pair is small enough to split its reduction
    x = synth.default_image_batch(md, 6, 9)
    m = ctx.load(synth.pack(md), max_batch=6, n_instances=1)
    try:
        ctx.set_proj_fusion(1 << 40)  # the first block's pair with its projection shortcut is not bit-identical: below
        ctx.set_pair_fusion(0)
        sep, _ = m.infer(x, prio=ctx.S.PRIO_HIGH)
        ctx.set_pair_fusion(1)
        fused, _ = m.infer(x, prio=ctx.S.PRIO_HIGH)
        names = [l.name.decode() for l in m.layers()]
        assert np.array_equal(sep["logits"], fused["logits"]) and np.array_equal(sep["top1"], fused["top1"])
        ref = omodels.resnet50_forward(md.tensors, x)
        check_logits(fused["logits"], ref.logits, fused["top1"], "ResNet-50 b6, fused seams")
        # intermediate activations read back through the fused path
        ref = omodels.resnet50_forward(md.tensors, x, keep=True)
        # (s1b0.c1 is computed inside the fused stem + pooling launch)
        for lname, key in (("s1b0.c1", "s1b0.c1"), ("s1b1.c1", "s1b1.c1"), ("s1b1.out", "s1b1.c3"), ("s1b2.out", "s1b2.c3"), ("s2b0.c1", "s2b0.c1")):
            got = m.read_activation(0, names.index(key), 6).astype(np.float64).reshape(ref.trace.acts[lname].shape)
            check_kernel(got, ref.trace.acts[lname], f"layer {lname}", rel=2.0 ** -8, abs_rel=1e-2)
        # the first block's closing 1x1, its projection shortcut and the next block's opening 1x1 as one launch: one
        # rounding fewer than the separate launches, so against the oracle only
        ctx.set_proj_fusion(1)
        proj, _ = m.infer(x, prio=ctx.S.PRIO_HIGH)
        check_logits(proj["logits"], ref.logits, proj["top1"], "ResNet-50 b6, projection in the fused seam")
        assert not np.array_equal(proj["logits"], fused["logits"])          # (the other path did run)
        for lname, key in (("s1b0.out", "s1b0.c3"), ("s1b1.c1", "s1b1.c1"), ("s1b1.out", "s1b1.c3")):
            got = m.read_activation(0, names.index(key), 6).astype(np.float64).reshape(ref.trace.acts[lname].shape)
            check_kernel(got, ref.trace.acts[lname], f"layer {lname} (projection fused)", rel=2.0 ** -8, abs_rel=1e-2)
    finally:
        ctx.set_pair_fusion(40000)
        ctx.set_proj_fusion(1)
        m.free()


@pytest.mark.parametrize("hw,batch", [(64, 5), (224, 2)])
def test_mobilenet_v2(ctx, hw, batch):
    md = synth.mobilenet_v2(synth.SEEDS[synth.ARCH_MOBILENETV2], hw=hw)
    x = synth.default_image_batch(md, batch, synth.SEEDS[synth.ARCH_MOBILENETV2] + batch)
    m, out, ref = run_cnn(ctx, md, x, omodels.mobilenet_v2_forward, ctx.S.PRIO_LOW, f"MobileNetV2 {hw}px b{batch}")
    m.free()


def test_mobilenet_v2_fused_expansions_equal_separate_launches(ctx):
    """Up to batch 8 every inverted residual block runs its expansion and its depthwise layer as one launch (and the
    112 x 112 one at any batch large enough); the kernel takes the same arithmetic steps, so the whole network's output
    must be bit-identical with the fusion switched off, and the oracle's within tolerance."""
    md = synth.mobilenet_v2(synth.SEEDS[synth.ARCH_MOBILENETV2])
    x = synth.default_image_batch(md, 6, 99)
    m = ctx.load(synth.pack(md), max_batch=6, n_instances=1)
    try:
        ctx.set_pair_fusion(0)
        sep, _ = m.infer(x, prio=ctx.S.PRIO_LOW)
        ctx.set_pair_fusion(40000)
        fused, _ = m.infer(x, prio=ctx.S.PRIO_LOW)
        assert np.array_equal(sep["logits"], fused["logits"]) and np.array_equal(sep["top1"], fused["top1"])
        ref = omodels.mobilenet_v2_forward(md.tensors, x)
        check_logits(fused["logits"], ref.logits, fused["top1"], "MobileNetV2 b6, fused expansions")
    finally:
        ctx.set_pair_fusion(40000)
        m.free()


def test_run_timed_gives_zero_for_layers_inside_another_launch(ctx):
    """Per-layer times: a layer that runs inside its predecessor's launch reads exactly 0, every launch a positive time."""
    md = synth.mobilenet_v2(synth.SEEDS[synth.ARCH_MOBILENETV2], hw=64)
    m = ctx.load(synth.pack(md), max_batch=4, n_instances=1)
    try:
        m.copy_in(0, ctx.S.PRIO_LOW, synth.default_image_batch(md, 4, 3))
        names = [l.name.decode() for l in m.layers()]
        ms = m.run_timed(0, ctx.S.PRIO_LOW, 4)
        inside = [n for n, t in zip(names, ms) if t == 0.0]
        assert inside == [f"b{i}.dw" for i in range(17)], inside   # behind its expansion; the first block's behind the stem
        assert all(t > 0.0 for n, t in zip(names, ms) if n not in inside)
        ctx.set_pair_fusion(0)
        assert all(t > 0.0 for t in m.run_timed(0, ctx.S.PRIO_LOW, 4))
    finally:
        ctx.set_pair_fusion(40000)
        m.free()


@pytest.mark.parametrize("kw,batch", [(dict(layers=2, hidden=128, heads=2, ffn=256, seq=64), 3),
                                      (dict(layers=2, hidden=128, heads=2, ffn=256, seq=48), 3),      # no multiple of the 32-row blocks
                                      (dict(layers=1, hidden=64, heads=1, ffn=128, seq=200), 2),      # more than 128 keys
                                      (dict(), 2)])
def test_encoder(ctx, kw, batch):
    md = synth.encoder(synth.SEEDS[synth.ARCH_ENCODER], **kw)
    x, vl = synth.token_batch(md, batch, synth.SEEDS[synth.ARCH_ENCODER] + batch, min_len=32)
    m = ctx.load(synth.pack(md), max_batch=batch, n_instances=1)
    out, rec = m.infer(x, vl, prio=ctx.S.PRIO_LOW)
    ref = omodels.encoder_forward(md.tensors, x, vl, md.hyper)
    scale = max(float(np.abs(ref.logits[b, :vl[b]]).max()) for b in range(batch))
    worst = 0.0
    for b in range(batch):
        L = int(vl[b])
        got = out["hidden"][b, :L].astype(np.float64)
        assert np.isfinite(got).all()
        worst = max(worst, float(np.abs(got - ref.logits[b, :L]).max()))
    assert worst <= 2e-2 * scale, f"encoder: max|err| {worst:.3e} > 2e-2 * {scale:.3e}"
    # top-1 of token 0 (same tie rule as the classifiers)
    check_logits(out["hidden"][:, 0, :], ref.logits[:, 0, :], out["top1"], "encoder token 0")
    print(f"encoder {md.hyper} b{batch}: max|err| {worst:.3e} of {scale:.3e}, kernels {rec.kernel_ms:.3f} ms")
    m.free()


@pytest.mark.parametrize("hw,batch,fc", [(32, 5, 64), (64, 3, 256)])
def test_vgg19(ctx, hw, batch, fc):
    md = synth.vgg19(synth.SEEDS[synth.ARCH_VGG19], hw=hw, classes=100, fc=fc)
    x = synth.default_image_batch(md, batch, synth.SEEDS[synth.ARCH_VGG19] + batch)
    m, out, ref = run_cnn(ctx, md, x, omodels.vgg19_forward, ctx.S.PRIO_LOW, f"VGG-19 {hw}px b{batch}")
    m.free()


def test_vgg19_layers(ctx):
    """Every layer's activation against the oracle's: pooling positions, the flattening order into fc1."""
    md = synth.vgg19(4, hw=64, classes=10, fc=64)
    x = synth.default_image_batch(md, 2, 9)
    m = ctx.load(synth.pack(md), max_batch=2, n_instances=1)
    ref = omodels.vgg19_forward(md.tensors, x, keep=True)
    m.copy_in(0, ctx.S.PRIO_LOW, x)
    m.run(0, ctx.S.PRIO_LOW, 2)
    m.sync(0, ctx.S.PRIO_LOW)
    names = {li.name.decode(): i for i, li in enumerate(m.layers())}
    checked = 0
    for lname, act in ref.trace.acts.items():
        if lname not in names or lname == "fc":
            continue
        got = m.read_activation(0, names[lname], 2).astype(np.float64).reshape(act.shape)
        check_kernel(got, act, f"layer {lname}", rel=2.0 ** -8, abs_rel=1e-2)
        checked += 1
    assert checked == 16 + 5 + 2
    m.free()


def run_vit(ctx, md, x, what):
    m = ctx.load(synth.pack(md), max_batch=x.shape[0], n_instances=1)
    out, rec = m.infer(x, prio=ctx.S.PRIO_HIGH)
    ref = omodels.vit_forward(md.tensors, x, md.hyper, keep=True)
    err, scale, ties = check_logits(out["logits"], ref.logits, out["top1"], what)
    assert np.abs(out["probs"] - ref.probs).max() <= 2e-2
    print(f"{what}: max|err| {err:.3e} of scale {scale:.3e} ({err / scale:.2e}), ties {ties}, kernels {rec.kernel_ms:.3f} ms")
    return m, out, ref


@pytest.mark.parametrize("hw,batch,kw", [(48, 3, dict(layers=2, hidden=128, heads=2, ffn=256)),     # 10 tokens
                                         (96, 2, dict(layers=2, hidden=128, heads=2, ffn=256)),     # 37 tokens
                                         (224, 2, dict(layers=2, hidden=192, heads=3, ffn=384))])   # 197 tokens
def test_vit(ctx, hw, batch, kw):
    md = synth.vit(synth.SEEDS[synth.ARCH_VIT], hw=hw, classes=100, **kw)
    x = synth.default_image_batch(md, batch, synth.SEEDS[synth.ARCH_VIT] + batch)
    m, out, ref = run_vit(ctx, md, x, f"ViT {hw}px b{batch}")
    # every block's output (the residual stream) against the oracle's
    names = {li.name.decode(): i for i, li in enumerate(m.layers())}
    m.copy_in(0, ctx.S.PRIO_LOW, x)
    m.run(0, ctx.S.PRIO_LOW, batch)
    m.sync(0, ctx.S.PRIO_LOW)
    checked = 0
    for lname in ("patch", "tokens", "l0.qkv", "l0.attn", "l0.o", "l0.ffn1", "l0.ffn2", "l1.o", "l1.ffn2", "ln"):
        act = ref.trace.acts[lname]
        got = m.read_activation(0, names[lname], batch).astype(np.float64).reshape(act.shape)
        check_kernel(got, act, f"layer {lname}", rel=2.0 ** -8, abs_rel=1e-2)
        checked += 1
    assert checked == 10
    m.free()


def test_submit_errors_and_pool(ctx):
    S = ctx.S
    md = synth.tiny_cnn(1)
    m = ctx.load(synth.pack(md), max_batch=2, n_instances=2)
    x = synth.default_image_batch(md, 2, 1)
    outs = [m.new_output(2) for _ in range(3)]
    t0 = m.submit(S.PRIO_HIGH, x, None, outs[0])
    t1 = m.submit(S.PRIO_LOW, x, None, outs[1])
    assert m.try_submit(S.PRIO_LOW, x, None, outs[2]) is None            # both instances taken: E_BUSY, never blocks
    with pytest.raises(S.StraitError) as e:
        m.free()
    assert e.value.status == S.E_BUSY
    r0, r1 = m.wait(t0), m.wait(t1)
    assert {r0.instance, r1.instance} == {0, 1} and r0.priority == S.PRIO_HIGH and r1.priority == S.PRIO_LOW
    assert np.array_equal(outs[0], outs[1])                              # same input, either priority: same bits
    with pytest.raises(S.StraitError) as e:
        m.submit(S.PRIO_HIGH, synth.default_image_batch(md, 3, 1), None, m.new_output(2))
    assert e.value.status == S.E_BATCH
    m.free()
    with pytest.raises(S.StraitError) as e:
        ctx.load(b"STRX" + bytes(100), 1, 1)
    assert e.value.status == S.E_FORMAT


@pytest.mark.parametrize("arch,batch", [("resnet50", 3), ("mobilenet_v2", 4), ("encoder", 2)])
def test_graph_replay_equals_kernel_by_kernel(ctx, arch, batch):
    """The captured-graph path replays the very same launches: every replay, on fresh inputs and with
    kernel-by-kernel passes and synchronisations in between, must equal the eager result bit for bit."""
    S = ctx.S
    if arch == "encoder":
        md = synth.encoder(5, layers=2, hidden=128, heads=2, ffn=256, seq=64)
    else:
        md = getattr(synth, arch)(5, hw=64)
    m = ctx.load(synth.pack(md), max_batch=batch, n_instances=2)
    try:
        for rep in range(5):                      # first use of a key runs eagerly, the second captures, later ones replay
            if arch == "encoder":
                x, vl = synth.token_batch(md, batch, 50 + rep)
            else:
                x, vl = synth.default_image_batch(md, batch, 50 + rep), None
            for prio in (S.PRIO_HIGH, S.PRIO_LOW):
                ctx.set_graphs(False)
                eager = m.new_output(batch)
                m.wait(m.submit(prio, x, vl, eager))
                ctx.set_graphs(True)
                replay = m.new_output(batch)
                rec = m.wait(m.submit(prio, x, vl, replay))
                assert np.array_equal(eager.view(np.uint8), replay.view(np.uint8)), (arch, rep, prio)
                assert rec.kernel_ms > 0
    finally:
        ctx.set_graphs(False)
        m.free()


def test_small_batch_split_reduction_is_reproducible(ctx):
    """Small batches split long reductions over several workgroups per tile; the partial results are summed
    in a fixed order, so repeated runs must agree bit for bit, at either priority."""
    S = ctx.S
    md = synth.resnet50(9, hw=64)
    x = synth.default_image_batch(md, 2, 3)
    m = ctx.load(synth.pack(md), max_batch=2, n_instances=2)
    try:
        outs = []
        for rep in range(6):
            out = m.new_output(2)
            m.wait(m.submit(S.PRIO_HIGH if rep % 2 else S.PRIO_LOW, x, None, out))
            outs.append(out.copy())
        for o in outs[1:]:
            assert np.array_equal(o.view(np.uint8), outs[0].view(np.uint8))
        ref = omodels.resnet50_forward(md.tensors, x)
        check_logits(m.decode(outs[0], 2)["logits"], ref.logits, m.decode(outs[0], 2)["top1"], "ResNet-50 64px b2 (split reductions)")
    finally:
        m.free()


def test_input_copy_by_kernel_and_by_copy_engine_give_the_same_result(ctx):
    """Inputs up to a settable size go in by a copy kernel, larger ones by hipMemcpyAsync: same bytes on the device
    either way, so outputs are identical bit for bit."""
    md = synth.resnet50(4, hw=64)
    m = ctx.load(synth.pack(md), max_batch=4, n_instances=1)
    try:
        x = synth.default_image_batch(md, 4, 3)
        outs = []
        for limit in (0, 8 << 20):
            ctx.set_h2d_kernel_limit(limit)
            out, rec = m.infer(x)
            assert rec.h2d_ms > 0
            outs.append(out)
        assert np.array_equal(outs[0]["logits"], outs[1]["logits"]) and np.array_equal(outs[0]["top1"], outs[1]["top1"])
    finally:
        ctx.set_h2d_kernel_limit(8 << 20)
        m.free()


def test_submit_from_the_staging_buffer_makes_no_host_copy_and_gives_the_same_result(ctx):
    S = ctx.S
    md = synth.resnet50(4, hw=64)
    x = synth.default_image_batch(md, 3, 5)
    m = ctx.load(synth.pack(md), max_batch=4, n_instances=2)
    try:
        ref = m.new_output(3)
        m.wait(m.submit(S.PRIO_LOW, x, None, ref))
        st = m.staging(1, 3)                        # instance 1's pinned input buffer
        st[:] = x
        out = m.new_output(3)
        rec = m.wait(m.submit(S.PRIO_HIGH, st, None, out))
        assert rec.instance == 1 and np.array_equal(out, ref)
        t = m.submit(S.PRIO_HIGH, st, None, out)    # the same buffer again while its batch is in flight: refused, not queued
        with pytest.raises(S.StraitError) as e:
            m.submit(S.PRIO_HIGH, st, None, m.new_output(3))
        assert e.value.status == S.E_BUSY
        m.wait(t)
    finally:
        m.free()
