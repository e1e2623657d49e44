"""GPU parity at the full sizes of the workloads, in the launch configuration bench.py times
(sub-steps on instance 0: copy_in once, run, copy_out), every sample checked against the CPU
oracle.  The oracle is run in chunks to bound host memory."""
import numpy as np
import pytest

import synth
from oracle import models as omodels
from parity import check_logits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    import paper_2604_28175_amd as strait
    c = strait.Context(device=0)
    c.S = strait
    yield c
    c.close()


def oracle_logits(fwd, tensors, x, chunk=16):
    outs = [fwd(tensors, x[i:i + chunk]) for i in range(0, x.shape[0], chunk)]
    return (np.concatenate([o.logits for o in outs]), np.concatenate([o.probs for o in outs]))


def cnn_case(ctx, arch, fwd, batches):
    S = ctx.S
    seed = synth.SEEDS[arch]
    md = synth.make_model(arch, seed)
    m = ctx.load(synth.pack(md), max_batch=max(batches), n_instances=1)
    try:
        for b in batches:
            x = synth.default_image_batch(md, b, seed + b)
            m.copy_in(0, S.PRIO_HIGH, x)
            m.run(0, S.PRIO_HIGH, b)
            out = m.decode(m.copy_out(0, S.PRIO_HIGH, b), b)
            logits, probs = oracle_logits(fwd, md.tensors, x)
            err, scale, ties = check_logits(out["logits"], logits, out["top1"], f"{synth.ARCH_NAMES[arch]} b{b}")
            assert np.abs(out["probs"] - probs).max() <= 2e-2
            print(f"{synth.ARCH_NAMES[arch]} b{b}: max|err| {err:.3e} = {err / scale:.2e} of max|logit| {scale:.2f}; tie-ambiguous samples {ties}")
    finally:
        m.free()


def test_resnet50_all_batches(ctx):
    cnn_case(ctx, synth.ARCH_RESNET50, omodels.resnet50_forward, (1, 8, 32, 128))


def test_mobilenet_v2_all_batches(ctx):
    cnn_case(ctx, synth.ARCH_MOBILENETV2, omodels.mobilenet_v2_forward, (1, 16, 64))


def test_encoder_all_batches(ctx):
    S = ctx.S
    seed = synth.SEEDS[synth.ARCH_ENCODER]
    md = synth.encoder(seed)
    m = ctx.load(synth.pack(md), max_batch=64, n_instances=1)
    try:
        for b in (1, 16, 64):
            x, vl = synth.token_batch(md, b, seed + b, min_len=32)
            m.copy_in(0, S.PRIO_LOW, x, vl)
            m.run(0, S.PRIO_LOW, b)
            out = m.decode(m.copy_out(0, S.PRIO_LOW, b), b)
            worst, scale = 0.0, 0.0
            ref0 = np.zeros((b, md.hyper[1]))
            for i in range(0, b, 16):
                ref = omodels.encoder_forward(md.tensors, x[i:i + 16], vl[i:i + 16], md.hyper)
                for j in range(ref.logits.shape[0]):
                    L = int(vl[i + j])
                    got = out["hidden"][i + j, :L].astype(np.float64)
                    assert np.isfinite(got).all()
                    worst = max(worst, float(np.abs(got - ref.logits[j, :L]).max()))
                    scale = max(scale, float(np.abs(ref.logits[j, :L]).max()))
                    ref0[i + j] = ref.logits[j, 0]
            assert worst <= 2e-2 * scale, f"encoder b{b}: {worst:.3e} > 2e-2 * {scale:.3e}"
            _, _, ties = check_logits(out["hidden"][:, 0, :], ref0, out["top1"], f"encoder b{b} token 0")
            print(f"encoder b{b}: max|err| {worst:.3e} = {worst / scale:.2e} of {scale:.2f}; ties {ties}")
    finally:
        m.free()


def test_vgg19_full_size(ctx):
    cnn_case(ctx, synth.ARCH_VGG19, omodels.vgg19_forward, (1, 6, 64))      # 64: the batch the benchmark times


def test_vit_b16_full_size(ctx):
    md_hyper = (224, 224, 3, 1000, 12, 768, 12, 3072)                 # what synth.vit() draws by default
    cnn_case(ctx, synth.ARCH_VIT, lambda t, x: omodels.vit_forward(t, x, md_hyper), (1, 8, 19, 64))
