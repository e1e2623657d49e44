"""CPU oracle: forward passes of the served architectures in fp64.

TEST INFRASTRUCTURE ONLY (see ops.py).  Written from the public definitions of the
architectures; the paper fixes the workload only as "a sequence of dependent kernels"
(Section 3.2) and lists ResNet-50 at 4.09 G multiply-accumulates (Table 1), which
`Trace.total_macs` reproduces for the topology below.

Every forward takes the seeded tensors (fp16 values) as a dict and returns a `Result` with the
pre-softmax logits, probabilities and top-1 indices, plus a `Trace` of per-layer multiply-
accumulate counts and (optionally) every layer's input and output for per-kernel checks.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

from . import ops

ARCH_TINY_CNN, ARCH_RESNET50, ARCH_MOBILENETV2, ARCH_ENCODER, ARCH_VGG19, ARCH_VIT = 0, 1, 2, 3, 4, 5
FP16_MAX = 65504.0


@dataclass
class Layer:
    name: str
    kind: str
    macs: int
    out_shape: tuple
    max_abs: float


@dataclass
class Trace:
    layers: List[Layer] = field(default_factory=list)
    keep: bool = False
    acts: Dict[str, np.ndarray] = field(default_factory=dict)

    def add(self, name, kind, macs, y):
        self.layers.append(Layer(name, kind, int(macs), tuple(y.shape), float(np.abs(y).max())))
        if self.keep:
            self.acts[name] = y

    @property
    def total_macs(self) -> int:
        return sum(l.macs for l in self.layers)

    def n_kind(self, kind) -> int:
        return sum(1 for l in self.layers if l.kind == kind)


@dataclass
class Result:
    logits: np.ndarray            # CNN: [N, classes]; encoder: hidden states [B, S, hidden]
    probs: Optional[np.ndarray]
    top1: np.ndarray              # int32
    trace: Trace


def _conv_unit(t, tr, name, x, stride, pad, act, bn=True, depthwise=False):
    w = t[name + ".w"]
    if bn:
        w, b = ops.fold_bn(w, t[name + ".gamma"], t[name + ".beta"], t[name + ".mean"], t[name + ".var"])
    else:
        b = t[name + ".b"].astype(np.float32)
    if depthwise:
        y = ops.dwconv2d(x, w, b, stride, pad)
        macs = y.size * w.shape[2] * w.shape[3]
    else:
        y = ops.conv2d(x, w, b, stride, pad)
        macs = y.size * w.shape[1] * w.shape[2] * w.shape[3]
    if act == "relu":
        y = ops.relu(y)
    elif act == "relu6":
        y = ops.relu6(y)
    tr.add(name, "dwconv" if depthwise else "conv", macs, y)
    return y


def _head(t, tr, feat):
    logits = ops.linear(feat, t["fc.w"], t["fc.b"])
    tr.add("fc", "fc", logits.size * feat.shape[-1], logits)
    return Result(logits, ops.softmax(logits), ops.argmax_first(logits), tr)


def tiny_cnn_forward(t, x, keep=False) -> Result:
    """conv3x3(16,s1,p1)+ReLU -> conv3x3(32,s2,p1)+ReLU -> conv3x3(64,s2,p1)+ReLU -> GAP -> FC -> softmax."""
    tr = Trace(keep=keep)
    y = np.asarray(x, np.float64)
    for i, stride in enumerate((1, 2, 2)):
        y = _conv_unit(t, tr, f"conv{i}", y, stride, 1, "relu", bn=False)
    feat = ops.global_avg_pool(y)
    tr.add("gap", "pool", 0, feat)
    return _head(t, tr, feat)


def resnet50_forward(t, x, keep=False) -> Result:
    """ResNet-50 v1.5: the stride of a down-sampling bottleneck sits on its 3x3 convolution."""
    tr = Trace(keep=keep)
    y = _conv_unit(t, tr, "stem", np.asarray(x, np.float64), 2, 3, "relu")
    y = ops.maxpool2d(y, 3, 2, 1)
    tr.add("maxpool", "pool", 0, y)
    for si, nb in enumerate((3, 4, 6, 3), start=1):
        for bi in range(nb):
            p = f"s{si}b{bi}"
            stride = 2 if (bi == 0 and si > 1) else 1
            a = _conv_unit(t, tr, p + ".c1", y, 1, 0, "relu")
            a = _conv_unit(t, tr, p + ".c2", a, stride, 1, "relu")
            a = _conv_unit(t, tr, p + ".c3", a, 1, 0, None)
            sc = _conv_unit(t, tr, p + ".down", y, stride, 0, None) if bi == 0 else y
            y = ops.relu(a + sc)
            tr.add(p + ".out", "add", 0, y)
    feat = ops.global_avg_pool(y)
    tr.add("gap", "pool", 0, feat)
    return _head(t, tr, feat)


MOBILENETV2_CFG = [(1, 16, 1, 1), (6, 24, 2, 2), (6, 32, 3, 2), (6, 64, 4, 2),
                   (6, 96, 3, 1), (6, 160, 3, 2), (6, 320, 1, 1)]


def mobilenet_v2_forward(t, x, keep=False) -> Result:
    """MobileNetV2 1.0: inverted residuals, ReLU6, linear bottlenecks; a block has a residual
    connection iff its stride is 1 and its input and output widths agree."""
    tr = Trace(keep=keep)
    y = _conv_unit(t, tr, "stem", np.asarray(x, np.float64), 2, 1, "relu6")
    cin, idx = 32, 0
    for tt, c, n, s in MOBILENETV2_CFG:
        for i in range(n):
            stride = s if i == 0 else 1
            p = f"b{idx}"
            a = y
            if tt != 1:
                a = _conv_unit(t, tr, p + ".expand", a, 1, 0, "relu6")
            a = _conv_unit(t, tr, p + ".dw", a, stride, 1, "relu6", depthwise=True)
            a = _conv_unit(t, tr, p + ".project", a, 1, 0, None)
            if stride == 1 and cin == c:
                a = a + y
                tr.add(p + ".out", "add", 0, a)
            y, cin, idx = a, c, idx + 1
    y = _conv_unit(t, tr, "head", y, 1, 0, "relu6")
    feat = ops.global_avg_pool(y)
    tr.add("gap", "pool", 0, feat)
    return _head(t, tr, feat)


def encoder_forward(t, x, valid_len, hyper, keep=False) -> Result:
    """Post-LayerNorm Transformer encoder stack:
         h = LN(x + Attn(x) W_o + b_o);  y = LN(h + GELU(h W_1 + b_1) W_2 + b_2)."""
    layers, hidden, heads, ffn, seq = hyper
    tr = Trace(keep=keep)
    y = np.asarray(x, np.float64)
    bsz = y.shape[0]
    ntok = bsz * seq
    attn_macs = int(sum(2 * seq * int(L) * hidden for L in valid_len))
    for i in range(layers):
        p = f"l{i}"
        q = ops.linear(y, t[p + ".q.w"], t[p + ".q.b"])
        k = ops.linear(y, t[p + ".k.w"], t[p + ".k.b"])
        v = ops.linear(y, t[p + ".v.w"], t[p + ".v.b"])
        tr.add(p + ".qkv", "gemm", 3 * ntok * hidden * hidden, np.concatenate([q, k, v], axis=-1))
        a = ops.attention(q, k, v, valid_len, heads)
        tr.add(p + ".attn", "attention", attn_macs, a)
        o = ops.linear(a, t[p + ".o.w"], t[p + ".o.b"])
        h = ops.layernorm(y + o, t[p + ".ln1.g"], t[p + ".ln1.b"])
        tr.add(p + ".ln1", "gemm", ntok * hidden * hidden, h)
        f = ops.gelu(ops.linear(h, t[p + ".ffn1.w"], t[p + ".ffn1.b"]))
        tr.add(p + ".ffn1", "gemm", ntok * hidden * ffn, f)
        f = ops.linear(f, t[p + ".ffn2.w"], t[p + ".ffn2.b"])
        y = ops.layernorm(h + f, t[p + ".ln2.g"], t[p + ".ln2.b"])
        tr.add(p + ".ln2", "gemm", ntok * hidden * ffn, y)
    return Result(y, None, ops.argmax_first(y[:, 0, :]), tr)


VGG19_CFG = [64, 64, "M", 128, 128, "M", 256, 256, 256, 256, "M", 512, 512, 512, 512, "M", 512, 512, 512, 512, "M"]


def vgg19_forward(t, x, keep=False) -> Result:
    """VGG-19 (configuration E of the VGG paper, no normalisation; Table 1 of the served-model list gives
    19.63 G multiply-accumulates): sixteen 3x3 convolutions with bias and ReLU, 2x2 max pooling of stride 2
    after the 2nd, 4th, 8th, 12th and 16th, the feature map flattened channel-major (channel, row, column),
    then FC-ReLU-FC-ReLU-FC and softmax."""
    tr = Trace(keep=keep)
    y = np.asarray(x, np.float64)
    i = 0
    for c in VGG19_CFG:
        if c == "M":
            y = ops.maxpool2d(y, 2, 2, 0)
            tr.add(f"pool{i}", "pool", 0, y)
        else:
            y = _conv_unit(t, tr, f"conv{i}", y, 1, 1, "relu", bn=False)
            i += 1
    n = y.shape[0]
    w1 = np.asarray(t["fc1.w"], np.float64)
    flat = np.transpose(y, (0, 3, 1, 2)).reshape(n, -1)                 # [N, C*H*W]
    f = ops.relu(ops.linear(flat, w1.reshape(w1.shape[0], -1), t["fc1.b"]))
    tr.add("fc1", "fc", f.size * flat.shape[1], f)
    g = ops.relu(ops.linear(f, t["fc2.w"], t["fc2.b"]))
    tr.add("fc2", "fc", g.size * f.shape[1], g)
    return _head(t, tr, g)


def vit_forward(t, x, hyper, keep=False) -> Result:
    """Vision Transformer ("An image is worth 16x16 words"), pre-LayerNorm blocks:
         tokens = [cls ; patches W_p + b_p] + pos
         z <- z + Attn(LN1(z)) W_o + b_o ;  z <- z + GELU(LN2(z) W_1 + b_1) W_2 + b_2      (per block)
         logits = LN(z)[token 0] W_h + b_h.
    A patch is a 16x16 window taken with stride 16, its values ordered as the weight tensor's (channel, row,
    column); LayerNorm eps 1e-6; every key takes part in attention."""
    layers, hidden, heads, ffn = hyper[4:8]
    tr = Trace(keep=keep)
    pw = t["patch.w"]
    y = ops.conv2d(np.asarray(x, np.float64), pw, t["patch.b"].astype(np.float64), pw.shape[2], 0)
    n, gh, gw, _ = y.shape
    tr.add("patch", "conv", y.size * pw.shape[1] * pw.shape[2] * pw.shape[3], y)
    tok = y.reshape(n, gh * gw, hidden)
    cls = np.broadcast_to(np.asarray(t["cls"], np.float64), (n, 1, hidden))
    z = np.concatenate([cls, tok], axis=1) + np.asarray(t["pos"], np.float64)[None]
    tr.add("tokens", "add", 0, z)
    seq = z.shape[1]
    ntok = n * seq
    full = np.full(n, seq, dtype=np.int32)
    for i in range(layers):
        p = f"l{i}"
        h = ops.layernorm(z, t[p + ".ln1.g"], t[p + ".ln1.b"], eps=1e-6)
        q = ops.linear(h, t[p + ".q.w"], t[p + ".q.b"])
        k = ops.linear(h, t[p + ".k.w"], t[p + ".k.b"])
        v = ops.linear(h, t[p + ".v.w"], t[p + ".v.b"])
        tr.add(p + ".qkv", "gemm", 3 * ntok * hidden * hidden, np.concatenate([q, k, v], axis=-1))
        a = ops.attention(q, k, v, full, heads)
        tr.add(p + ".attn", "attention", 2 * n * seq * seq * hidden, a)
        z = z + ops.linear(a, t[p + ".o.w"], t[p + ".o.b"])
        tr.add(p + ".o", "gemm", ntok * hidden * hidden, z)
        h = ops.layernorm(z, t[p + ".ln2.g"], t[p + ".ln2.b"], eps=1e-6)
        f = ops.gelu(ops.linear(h, t[p + ".ffn1.w"], t[p + ".ffn1.b"]))
        tr.add(p + ".ffn1", "gemm", ntok * hidden * ffn, f)
        z = z + ops.linear(f, t[p + ".ffn2.w"], t[p + ".ffn2.b"])
        tr.add(p + ".ffn2", "gemm", ntok * hidden * ffn, z)
    feat = ops.layernorm(z[:, 0, :], t["ln.g"], t["ln.b"], eps=1e-6)
    tr.add("ln", "norm", 0, feat)
    return _head(t, tr, feat)


def forward(arch, tensors, x, valid_len=None, hyper=None, keep=False) -> Result:
    if arch == ARCH_TINY_CNN:
        return tiny_cnn_forward(tensors, x, keep)
    if arch == ARCH_RESNET50:
        return resnet50_forward(tensors, x, keep)
    if arch == ARCH_MOBILENETV2:
        return mobilenet_v2_forward(tensors, x, keep)
    if arch == ARCH_ENCODER:
        return encoder_forward(tensors, x, valid_len, hyper, keep)
    if arch == ARCH_VGG19:
        return vgg19_forward(tensors, x, keep)
    if arch == ARCH_VIT:
        return vit_forward(tensors, x, hyper, keep)
    raise ValueError(arch)
