"""Pins of the oracle's model forwards: topology against the paper's Table 1 and closed-form
operation counts, wiring against short independent compositions, invariants."""
import os

import numpy as np
import pytest

import synth
from oracle import models, ops
from test_oracle_ops import conv_by_windows

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _table1():
    out = {}
    for line in open(os.path.join(GOLDEN, "table1_models.txt")):
        if line[0] != "#" and line.strip():
            k, v = line.split()
            out[k] = float(v)
    return out


@pytest.fixture(scope="module")
def resnet_full():
    md = synth.resnet50(synth.SEEDS[synth.ARCH_RESNET50])
    x = synth.default_image_batch(md, 1, 11)
    return md, x, models.resnet50_forward(md.tensors, x)


def test_resnet50_topology_matches_table1(resnet_full):
    md, x, r = resnet_full
    tr = r.trace
    assert tr.total_macs == 4_089_184_256
    assert round(tr.total_macs / 1e9, 2) == _table1()["resnet50"]          # Table 1: 4.09
    assert tr.n_kind("conv") == 53 and tr.n_kind("add") == 16
    shapes = {l.name: l.out_shape for l in tr.layers}
    assert shapes["stem"] == (1, 112, 112, 64) and shapes["maxpool"] == (1, 56, 56, 64)
    assert shapes["s1b2.out"] == (1, 56, 56, 256) and shapes["s2b3.out"] == (1, 28, 28, 512)
    assert shapes["s3b5.out"] == (1, 14, 14, 1024) and shapes["s4b2.out"] == (1, 7, 7, 2048)
    # v1.5: the stride sits on the 3x3, so the first 1x1 of a down-sampling block still runs at full size
    assert shapes["s2b0.c1"] == (1, 56, 56, 128) and shapes["s2b0.c2"] == (1, 28, 28, 128)
    conv_fc_params = sum(t.size for k, t in md.tensors.items() if k.endswith(".w"))
    assert conv_fc_params == 25_502_912
    assert r.logits.shape == (1, 1000) and r.top1.dtype == np.int32
    # no activation leaves the fp16 range, so an fp16 GPU path cannot overflow on these inputs
    assert max(l.max_abs for l in tr.layers) < 6e4


def test_mobilenet_v2_topology():
    md = synth.mobilenet_v2(synth.SEEDS[synth.ARCH_MOBILENETV2])
    x = synth.default_image_batch(md, 1, 11)
    r = models.mobilenet_v2_forward(md.tensors, x)
    tr = r.trace
    assert tr.total_macs == 300_774_272                                  # the published ~300 M
    assert tr.n_kind("dwconv") == 17 and tr.n_kind("conv") == 35 and tr.n_kind("add") == 10
    shapes = {l.name: l.out_shape for l in tr.layers}
    assert shapes["head"] == (1, 7, 7, 1280) and shapes["b0.dw"] == (1, 112, 112, 32)
    assert shapes["b1.dw"] == (1, 56, 56, 96) and shapes["b16.dw"] == (1, 7, 7, 960)
    dw_macs = sum(l.macs for l in tr.layers if l.kind == "dwconv")
    assert abs(dw_macs / 1e6 - 20.7) < 0.1
    assert max(l.max_abs for l in tr.layers) < 6e4


def test_encoder_macs_closed_form():
    md = synth.encoder(3, layers=2, hidden=64, heads=4, ffn=256, seq=16)
    x, vl = synth.token_batch(md, 3, 4, min_len=16)           # all full length
    r = models.encoder_forward(md.tensors, x, vl, md.hyper)
    L, H, F, S, B = 2, 64, 256, 16, 3
    assert r.trace.total_macs == L * B * (S * (4 * H * H + 2 * H * F) + 2 * S * S * H)
    # BERT-base shape, closed form per 128-token sequence: 11.17 G
    S, H, F = 128, 768, 3072
    assert round(12 * (S * (4 * H * H + 2 * H * F) + 2 * S * S * H) / 1e9, 2) == 11.17
    assert r.logits.shape == (3, 16, 64) and r.top1.shape == (3,)


def test_tiny_cnn_zero_input_and_homogeneity():
    md = synth.tiny_cnn(synth.SEEDS[synth.ARCH_TINY_CNN])
    z = models.tiny_cnn_forward(md.tensors, np.zeros((2, 32, 32, 3), np.float16))
    assert not z.logits.any() and np.allclose(z.probs, 0.1)
    x = synth.default_image_batch(md, 4, 5)
    r1 = models.tiny_cnn_forward(md.tensors, x)
    r2 = models.tiny_cnn_forward(md.tensors, x.astype(np.float64) * 2.0)
    assert np.allclose(r2.logits, 2.0 * r1.logits, rtol=1e-13, atol=0)        # ReLU net with zero biases is positively homogeneous
    assert abs(r1.trace.total_macs / 4 / 1e6 - 2.80) < 0.01
    assert np.abs(r1.probs.sum(-1) - 1).max() < 1e-12
    assert np.array_equal(r1.top1, r1.probs.argmax(-1))


def test_tiny_cnn_against_independent_composition():
    md = synth.tiny_cnn(7)
    t = md.tensors
    x = synth.default_image_batch(md, 2, 5)
    y = x.astype(np.float64)
    for i, s in enumerate((1, 2, 2)):
        y = np.maximum(conv_by_windows(y, t[f"conv{i}.w"].astype(np.float64), None, s, 1), 0)
    assert y.shape == (2, 8, 8, 64)
    logits = y.mean(axis=(1, 2)) @ t["fc.w"].astype(np.float64).T
    r = models.tiny_cnn_forward(t, x)
    assert np.allclose(r.logits, logits, rtol=1e-11, atol=1e-11)


def test_resnet50_batch_independence_and_homogeneity():
    md = synth.resnet50(5, hw=32)
    t = dict(md.tensors)
    x = synth.default_image_batch(md, 3, 2)
    r = models.resnet50_forward(t, x)
    for i in range(3):
        ri = models.resnet50_forward(t, x[i:i + 1])
        assert np.allclose(ri.logits[0], r.logits[i], rtol=1e-12, atol=1e-12)   # BLAS blocking differs with batch
    for k in t:
        if k.endswith(".beta") or k.endswith(".mean"):
            t[k] = np.zeros_like(t[k])
    a = models.resnet50_forward(t, x)
    b = models.resnet50_forward(t, x.astype(np.float64) * 2.0)
    assert np.allclose(b.logits, 2.0 * a.logits, rtol=1e-13, atol=0)


def test_resnet50_shortcut_wiring():
    """With the last BatchNorm of every bottleneck zeroed (gamma = beta = 0) each residual branch
    contributes nothing: identity blocks pass their input through and the first block of a stage
    reduces to its strided 1x1 projection.  The net becomes a short chain computable independently."""
    md = synth.resnet50(9, hw=32)
    t = dict(md.tensors)
    for k in t:
        if k.endswith(".c3.gamma") or k.endswith(".c3.beta"):
            t[k] = np.zeros_like(t[k])
    x = synth.default_image_batch(md, 2, 3)
    r = models.resnet50_forward(t, x)

    def unit(name, y, stride, pad):
        w, b = ops.fold_bn(t[name + ".w"], t[name + ".gamma"], t[name + ".beta"], t[name + ".mean"], t[name + ".var"])
        return conv_by_windows(y, w.astype(np.float64), b.astype(np.float64), stride, pad)

    y = np.maximum(unit("stem", x.astype(np.float64), 2, 3), 0)
    yp = np.pad(y, ((0, 0), (1, 1), (1, 1), (0, 0)), constant_values=-np.inf)
    from numpy.lib.stride_tricks import sliding_window_view
    y = sliding_window_view(yp, (3, 3), axis=(1, 2))[:, ::2, ::2].max(axis=(-1, -2))
    for si in (1, 2, 3, 4):
        y = np.maximum(unit(f"s{si}b0.down", y, 1 if si == 1 else 2, 0), 0)
    logits = y.mean(axis=(1, 2)) @ t["fc.w"].astype(np.float64).T
    assert np.allclose(r.logits, logits, rtol=1e-10, atol=1e-10)


def test_mobilenet_v2_block_wiring():
    """Zero every projection's BatchNorm gamma and beta: every block then outputs 0 (+ its input where it
    has a residual connection), so the features entering `head` are exactly zero and the logits
    depend on the head's folded bias alone."""
    md = synth.mobilenet_v2(4, hw=32)
    t = dict(md.tensors)
    for k in t:
        if k.endswith(".project.gamma") or k.endswith(".project.beta"):
            t[k] = np.zeros_like(t[k])
    x = synth.default_image_batch(md, 2, 3)
    r = models.mobilenet_v2_forward(t, x, keep=True)
    assert not r.trace.acts["b16.project"].any()
    _, hb = ops.fold_bn(t["head.w"], t["head.gamma"], t["head.beta"], t["head.mean"], t["head.var"])
    feat = np.clip(hb.astype(np.float64), 0, 6)
    want = feat @ t["fc.w"].astype(np.float64).T
    assert np.allclose(r.logits, np.broadcast_to(want, r.logits.shape), atol=1e-12)


def test_mobilenet_v2_batch_independence():
    md = synth.mobilenet_v2(4, hw=32)
    x = synth.default_image_batch(md, 2, 3)
    r = models.mobilenet_v2_forward(md.tensors, x)
    r0 = models.mobilenet_v2_forward(md.tensors, x[1:2])
    assert np.allclose(r0.logits[0], r.logits[1], rtol=1e-12, atol=1e-12)


def test_encoder_mask_invariance_and_single_layer_composition():
    md = synth.encoder(6, layers=2, hidden=32, heads=2, ffn=64, seq=12)
    x, vl = synth.token_batch(md, 3, 8, min_len=4)
    r = models.encoder_forward(md.tensors, x, vl, md.hyper)
    x2 = x.copy()
    for b in range(3):
        x2[b, vl[b]:] = 7.0                                   # change the padded tokens' values
    r2 = models.encoder_forward(md.tensors, x2, vl, md.hyper)
    for b in range(3):
        assert np.array_equal(r.logits[b, :vl[b]], r2.logits[b, :vl[b]])
    # row statistics after the closing LayerNorm: (y - beta)/gamma has mean 0 and variance 1
    t = md.tensors
    g, be = t["l1.ln2.g"].astype(np.float64), t["l1.ln2.b"].astype(np.float64)
    z = (r.logits - be) / g
    assert np.abs(z.mean(-1)).max() < 1e-9 and np.abs(z.var(-1) - 1).max() < 1e-6


# ------------------------------------------------------------------ VGG-19
def test_vgg19_topology_matches_table1():
    md = synth.vgg19(synth.SEEDS[synth.ARCH_VGG19])
    x = synth.default_image_batch(md, 1, 11)
    r = models.vgg19_forward(md.tensors, x)
    tr = r.trace
    assert round(tr.total_macs / 1e9, 2) == _table1()["vgg19"]              # Table 1: 19.63
    assert tr.n_kind("conv") == 16 and tr.n_kind("pool") == 5 and tr.n_kind("fc") == 3
    assert md.n_params() == 143_667_240                                      # the published parameter count
    shapes = {l.name: l.out_shape for l in tr.layers}
    assert shapes["conv1"] == (1, 224, 224, 64) and shapes["pool2"] == (1, 112, 112, 64)
    assert shapes["conv15"] == (1, 14, 14, 512) and shapes["pool16"] == (1, 7, 7, 512) and shapes["fc1"] == (1, 4096)
    assert max(l.max_abs for l in tr.layers) < 6e4


def test_vgg19_against_independent_composition():
    """The whole small network again from windows, reshape-max pooling and matrix products."""
    md = synth.vgg19(5, hw=64, classes=10, fc=24)
    x = synth.default_image_batch(md, 2, 6)
    r = models.vgg19_forward(md.tensors, x, keep=True)
    t = md.tensors
    y = np.asarray(x, np.float64)
    i = 0
    for c in synth.models.VGG19_CFG:
        if c == "M":
            n, h, w, ch = y.shape
            y = y.reshape(n, h // 2, 2, w // 2, 2, ch).max(axis=(2, 4))
        else:
            y = np.maximum(conv_by_windows(y, t[f"conv{i}.w"], t[f"conv{i}.b"].astype(np.float64), 1, 1), 0)
            i += 1
    assert y.shape == (2, 2, 2, 512) and np.allclose(y, r.trace.acts["pool16"], rtol=1e-9, atol=1e-9)
    # channel-major flattening: feature (c, h, w) meets fc1.w[:, c, h, w]
    f = np.maximum(np.einsum("nhwc,ochw->no", y, t["fc1.w"].astype(np.float64)) + t["fc1.b"].astype(np.float64), 0)
    g = np.maximum(f @ t["fc2.w"].astype(np.float64).T + t["fc2.b"].astype(np.float64), 0)
    logits = g @ t["fc.w"].astype(np.float64).T + t["fc.b"].astype(np.float64)
    assert np.allclose(logits, r.logits, rtol=1e-9, atol=1e-9)


def test_vgg19_flatten_order_is_channel_row_column():
    md = synth.vgg19(5, hw=64, classes=4, fc=8)
    t = dict(md.tensors)
    pick = [(0, 0, 0), (3, 0, 1), (7, 1, 0), (500, 1, 1), (511, 0, 1), (100, 1, 0), (1, 1, 1), (256, 0, 0)]
    w1 = np.zeros_like(t["fc1.w"])
    for j, (c, h, w) in enumerate(pick):
        w1[j, c, h, w] = 1
    t["fc1.w"], t["fc1.b"] = w1, np.zeros_like(t["fc1.b"])
    x = synth.default_image_batch(md, 1, 2)
    r = models.vgg19_forward(t, x, keep=True)
    feat = r.trace.acts["pool16"]
    assert np.array_equal(r.trace.acts["fc1"][0], [max(feat[0, h, w, c], 0.0) for c, h, w in pick])


# ------------------------------------------------------------------ ViT
def test_vit_topology_matches_table1():
    md = synth.vit(synth.SEEDS[synth.ARCH_VIT])
    x = synth.default_image_batch(md, 1, 11)
    r = models.vit_forward(md.tensors, x, md.hyper)
    tr = r.trace
    attn = sum(l.macs for l in tr.layers if l.kind == "attention")
    assert round((tr.total_macs - attn) / 1e9, 2) == _table1()["vit_b16"]   # Table 1: 16.85
    assert round(tr.total_macs / 1e9, 2) == _table1()["vit_b16_with_attention_products"]
    assert md.n_params() == 86_567_656                                      # the published parameter count
    shapes = {l.name: l.out_shape for l in tr.layers}
    assert shapes["patch"] == (1, 14, 14, 768) and shapes["tokens"] == (1, 197, 768) and shapes["l11.ffn2"] == (1, 197, 768)
    assert r.logits.shape == (1, 1000) and max(l.max_abs for l in tr.layers) < 6e4


def small_vit():
    md = synth.vit(9, hw=48, classes=7, layers=2, hidden=32, heads=2, ffn=64)
    return md, synth.default_image_batch(md, 3, 4)


def test_vit_patches_and_tokens():
    md, x = small_vit()
    t = md.tensors
    r = models.vit_forward(t, x, md.hyper, keep=True)
    n, g = 3, 3
    patches = np.asarray(x, np.float64).reshape(n, g, 16, g, 16, 3).transpose(0, 1, 3, 5, 2, 4).reshape(n, g * g, 3 * 256)
    emb = patches @ t["patch.w"].astype(np.float64).reshape(32, -1).T + t["patch.b"].astype(np.float64)
    z = r.trace.acts["tokens"]
    pos = t["pos"].astype(np.float64)
    assert z.shape == (n, 10, 32)
    assert np.allclose(z[:, 1:], emb + pos[1:], rtol=1e-10, atol=1e-12)
    assert np.allclose(z[:, 0], t["cls"].astype(np.float64) + pos[0], rtol=0, atol=0)


def test_vit_block_matches_the_library_pre_norm_layer():
    """torch.nn.TransformerEncoderLayer(norm_first=True, activation='gelu') is the same block."""
    import torch
    md, x = small_vit()
    t = md.tensors
    r = models.vit_forward(t, x, md.hyper, keep=True)
    layer = torch.nn.TransformerEncoderLayer(32, 2, 64, dropout=0.0, activation="gelu", layer_norm_eps=1e-6,
                                             batch_first=True, norm_first=True).double().eval()
    z = torch.from_numpy(r.trace.acts["tokens"])
    for i in range(2):
        p = f"l{i}"
        f64 = lambda k: torch.from_numpy(t[k].astype(np.float64))
        sd = {"self_attn.in_proj_weight": torch.cat([f64(p + ".q.w"), f64(p + ".k.w"), f64(p + ".v.w")]),
              "self_attn.in_proj_bias": torch.cat([f64(p + ".q.b"), f64(p + ".k.b"), f64(p + ".v.b")]),
              "self_attn.out_proj.weight": f64(p + ".o.w"), "self_attn.out_proj.bias": f64(p + ".o.b"),
              "linear1.weight": f64(p + ".ffn1.w"), "linear1.bias": f64(p + ".ffn1.b"),
              "linear2.weight": f64(p + ".ffn2.w"), "linear2.bias": f64(p + ".ffn2.b"),
              "norm1.weight": f64(p + ".ln1.g"), "norm1.bias": f64(p + ".ln1.b"),
              "norm2.weight": f64(p + ".ln2.g"), "norm2.bias": f64(p + ".ln2.b")}
        layer.load_state_dict(sd)
        with torch.no_grad():
            z = layer(z)
        assert np.allclose(z.numpy(), r.trace.acts[p + ".ffn2"], rtol=1e-9, atol=1e-11)


def test_vit_head_reads_the_class_token_after_the_final_norm():
    md, x = small_vit()
    t = dict(md.tensors)
    for i in range(2):                                                 # blocks that add nothing: tokens pass through
        for k in (f"l{i}.o.w", f"l{i}.o.b", f"l{i}.ffn2.w", f"l{i}.ffn2.b"):
            t[k] = np.zeros_like(t[k])
    r = models.vit_forward(t, x, md.hyper)
    c = t["cls"].astype(np.float64) + t["pos"][0].astype(np.float64)
    n = (c - c.mean()) / np.sqrt(c.var() + 1e-6) * t["ln.g"].astype(np.float64) + t["ln.b"].astype(np.float64)
    want = n @ t["fc.w"].astype(np.float64).T + t["fc.b"].astype(np.float64)
    assert np.allclose(r.logits, want[None], rtol=1e-10, atol=1e-12)    # the same for every image
    full = models.vit_forward(md.tensors, x, md.hyper)
    assert np.abs(full.logits - full.logits[0]).max() > 1e-6          # ... and not with the real blocks
    one = models.vit_forward(md.tensors, x[1:2], md.hyper)
    assert np.allclose(one.logits[0], full.logits[1], rtol=1e-12, atol=1e-12)


# ------------------------------------------------------------------ wiring of whole blocks, with every branch live
def _folded_unit(t, name, y, stride, pad):
    """One convolution + folded BatchNorm from windows and one tensordot (not the oracle's loops)."""
    w, b = ops.fold_bn(t[name + ".w"], t[name + ".gamma"], t[name + ".beta"], t[name + ".mean"], t[name + ".var"])
    return conv_by_windows(y, w.astype(np.float64), b.astype(np.float64), stride, pad)


def _depthwise_by_channels(t, name, y, stride):
    """Depthwise 3x3 (pad 1) as one single-channel convolution per channel."""
    w, b = ops.fold_bn(t[name + ".w"], t[name + ".gamma"], t[name + ".beta"], t[name + ".mean"], t[name + ".var"])
    cols = [conv_by_windows(y[..., c:c + 1], w[c:c + 1].astype(np.float64), None, stride, 1) for c in range(y.shape[-1])]
    return np.concatenate(cols, axis=-1) + b.astype(np.float64)


def test_resnet50_bottleneck_wiring_identity_and_downsampling():
    """A bottleneck with every convolution live: 1x1 -> ReLU -> 3x3 (carrying the stride) -> ReLU -> 1x1, plus the
    block input (identity block) or its strided 1x1 projection (first block of a stage), then ReLU.  Recomposed from
    the block's recorded input; a dropped ReLU, a dropped shortcut or a misplaced stride changes the result."""
    md = synth.resnet50(9, hw=32)
    t = md.tensors
    x = synth.default_image_batch(md, 2, 3)
    acts = models.resnet50_forward(t, x, keep=True).trace.acts
    for p, src, stride, proj in (("s1b1", "s1b0.out", 1, False), ("s2b0", "s1b2.out", 2, True),
                                 ("s1b0", "maxpool", 1, True), ("s4b2", "s4b1.out", 1, False)):
        y = acts[src]
        a = np.maximum(_folded_unit(t, p + ".c1", y, 1, 0), 0)
        assert (a == 0).any() and (a > 0).any()                       # the clamp is exercised
        a = np.maximum(_folded_unit(t, p + ".c2", a, stride, 1), 0)
        a = _folded_unit(t, p + ".c3", a, 1, 0)
        sc = _folded_unit(t, p + ".down", y, stride, 0) if proj else y
        want = np.maximum(a + sc, 0)
        got = acts[p + ".out"]
        assert got.shape == want.shape and np.abs(a).max() > 1e-3     # the residual branch is not a zero
        assert np.allclose(got, want, rtol=1e-10, atol=1e-10)
        # ... and each of the mistakes named above would have been seen
        assert not np.allclose(got, np.maximum(sc, 0), rtol=1e-6, atol=1e-6)
        assert not np.allclose(got, np.maximum(a, 0), rtol=1e-6, atol=1e-6)


def test_mobilenet_v2_inverted_residual_wiring():
    """Inverted residual with every part live: 1x1 expansion -> ReLU6 -> depthwise 3x3 (stride) -> ReLU6 -> linear 1x1
    projection, plus the block input when the stride is 1 and the widths agree.  One stride-1 block with a residual
    connection, one stride-2 block, and the first block (no expansion)."""
    md = synth.mobilenet_v2(4, hw=64)
    t = md.tensors
    x = synth.default_image_batch(md, 2, 3)
    acts = models.mobilenet_v2_forward(t, x, keep=True).trace.acts
    hit0 = hit6 = False
    for p, src, stride, expand, residual in (("b2", "b1.project", 1, True, True), ("b3", "b2.out", 2, True, False),
                                             ("b0", "stem", 1, False, False), ("b5", "b4.out", 1, True, True)):
        y = acts[src]
        a = y
        if expand:
            a = np.clip(_folded_unit(t, p + ".expand", a, 1, 0), 0, 6)
            hit0 |= bool((a == 0).any()); hit6 |= bool((a == 6).any())
        a = np.clip(_depthwise_by_channels(t, p + ".dw", a, stride), 0, 6)
        hit0 |= bool((a == 0).any()); hit6 |= bool((a == 6).any())
        a = _folded_unit(t, p + ".project", a, 1, 0)                  # linear bottleneck: no clamp here
        assert (a < 0).any()
        want = a + y if residual else a
        got = acts[p + ".out"] if residual else acts[p + ".project"]
        assert got.shape == want.shape
        assert np.allclose(got, want, rtol=1e-10, atol=1e-10)
        if residual:
            assert not np.allclose(got, a, rtol=1e-6, atol=1e-6)
    assert hit0 and hit6                                              # both clamps of ReLU6 were exercised


def test_encoder_layer_matches_the_library_post_norm_layer():
    """torch.nn.TransformerEncoderLayer(norm_first=False, activation='gelu') with a key-padding mask is the same
    layer: x -> LN(x + Attn(x)) -> LN(h + FFN(h)).  Rows at valid positions are compared, layer by layer."""
    import torch
    md = synth.encoder(6, layers=2, hidden=32, heads=2, ffn=64, seq=12)
    x, vl = synth.token_batch(md, 3, 8, min_len=4)
    assert vl.min() < 12                                              # some keys are masked
    t = md.tensors
    r = models.encoder_forward(t, x, vl, md.hyper, keep=True)
    layer = torch.nn.TransformerEncoderLayer(32, 2, 64, dropout=0.0, activation="gelu", layer_norm_eps=1e-12,
                                             batch_first=True, norm_first=False).double().train()
    pad = torch.from_numpy(np.arange(12)[None, :] >= vl[:, None])
    z = torch.from_numpy(np.asarray(x, np.float64))
    f64 = lambda k: torch.from_numpy(t[k].astype(np.float64))
    for i in range(2):
        p = f"l{i}"
        layer.load_state_dict({
            "self_attn.in_proj_weight": torch.cat([f64(p + ".q.w"), f64(p + ".k.w"), f64(p + ".v.w")]),
            "self_attn.in_proj_bias": torch.cat([f64(p + ".q.b"), f64(p + ".k.b"), f64(p + ".v.b")]),
            "self_attn.out_proj.weight": f64(p + ".o.w"), "self_attn.out_proj.bias": f64(p + ".o.b"),
            "linear1.weight": f64(p + ".ffn1.w"), "linear1.bias": f64(p + ".ffn1.b"),
            "linear2.weight": f64(p + ".ffn2.w"), "linear2.bias": f64(p + ".ffn2.b"),
            "norm1.weight": f64(p + ".ln1.g"), "norm1.bias": f64(p + ".ln1.b"),
            "norm2.weight": f64(p + ".ln2.g"), "norm2.bias": f64(p + ".ln2.b")})
        with torch.no_grad():
            z = layer(z, src_key_padding_mask=pad)
        got = r.trace.acts[p + ".ln2"]
        for b in range(3):
            assert np.allclose(z.numpy()[b, :vl[b]], got[b, :vl[b]], rtol=1e-9, atol=1e-10)
    assert np.array_equal(r.logits, r.trace.acts["l1.ln2"])
