"""Seeded synthetic weights and inputs for the four served architectures.

This module only *draws numbers* and names them; it contains none of the
forward-pass arithmetic (no convolution, no BatchNorm fold, no layout change).
The CPU oracle and the GPU library each read the tensors produced here and do
everything else on their own.

All values are drawn in fp64, rounded once to fp16 (round-to-nearest-even) and
kept as fp16, so that weight/input quantisation is common to both sides.

Weight recipe
-------------
* conv / linear weights of the CNNs: He-normal, std = sqrt(2 / fan_in),
  fan_in = k*k*Cin/groups; stored OIHW (linear: [out, in]).
* BatchNorm (ResNet-50, MobileNetV2), eps = 1e-5: gamma ~ U[0.8,1.2],
  beta ~ N(0,0.05), running mean ~ N(0,0.05), running var ~ U[0.8,1.2].
  The BatchNorm that closes a ResNet bottleneck (`c3`) draws gamma from
  U[0.2,0.4] instead, which keeps the activations of the random residual net
  inside a healthy fp16 range.  (MobileNetV2 needs no such device: ReLU6
  bounds its activations, and both clamps are exercised.)
* tiny CNN: no BatchNorm, explicit zero biases; FC biases are zero everywhere.
* encoder: all matrices and biases N(0,0.02); LayerNorm gamma ~ U[0.8,1.2],
  beta ~ N(0,0.02).
* VGG-19 (no BatchNorm): He-normal weights, biases N(0,0.02); the first fully connected layer is
  stored [out, 512, h, w] so that the order in which the feature map is flattened (channel, row,
  column) is part of the data.
* ViT: every matrix, bias, the class token and the position embeddings N(0,0.02); LayerNorm as the
  encoder's; hyper = (H, W, 3, classes, layers, hidden, heads, ffn), patches of 16 x 16.
"""
from __future__ import annotations

from collections import OrderedDict
from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np

from . import rng

ARCH_TINY_CNN = 0
ARCH_RESNET50 = 1
ARCH_MOBILENETV2 = 2
ARCH_ENCODER = 3
ARCH_VGG19 = 4
ARCH_VIT = 5

ARCH_NAMES = {ARCH_TINY_CNN: "tiny_cnn", ARCH_RESNET50: "resnet50_v1.5",
              ARCH_MOBILENETV2: "mobilenet_v2", ARCH_ENCODER: "encoder",
              ARCH_VGG19: "vgg19", ARCH_VIT: "vit_b16"}

BN_EPS = 1e-5

# MobileNetV2 width 1.0: (expansion t, output channels c, repeats n, first stride s)
MOBILENETV2_CFG = [(1, 16, 1, 1), (6, 24, 2, 2), (6, 32, 3, 2), (6, 64, 4, 2),
                   (6, 96, 3, 1), (6, 160, 3, 2), (6, 320, 1, 1)]
# VGG-19: output channels of the 3x3 convolutions, "M" = 2x2 max pooling with stride 2
VGG19_CFG = [64, 64, "M", 128, 128, "M", 256, 256, 256, 256, "M", 512, 512, 512, 512, "M", 512, 512, 512, 512, "M"]
VIT_PATCH = 16
RESNET50_BLOCKS = [3, 4, 6, 3]
RESNET50_PLANES = [64, 128, 256, 512]


@dataclass
class ModelData:
    arch: int
    hyper: Tuple[int, ...]            # CNN: (H, W, C_in, classes); encoder: (layers, hidden, heads, ffn, seq)
    tensors: "OrderedDict[str, np.ndarray]" = field(default_factory=OrderedDict)

    def n_params(self) -> int:
        return int(sum(t.size for t in self.tensors.values()))


def _f16(x: np.ndarray, shape) -> np.ndarray:
    return np.ascontiguousarray(x.reshape(shape).astype(np.float16))


class _Gen:
    def __init__(self, seed: int, md: ModelData):
        self.seed, self.md = seed, md

    def he(self, name, shape):
        fan_in = int(np.prod(shape[1:]))
        n = int(np.prod(shape))
        self.md.tensors[name] = _f16(rng.normal(self.seed, name, n, 0.0, (2.0 / fan_in) ** 0.5), shape)

    def normal(self, name, shape, std, mean=0.0):
        n = int(np.prod(shape))
        self.md.tensors[name] = _f16(rng.normal(self.seed, name, n, mean, std), shape)

    def uniform(self, name, shape, lo, hi):
        n = int(np.prod(shape))
        self.md.tensors[name] = _f16(rng.uniform(self.seed, name, n, lo, hi), shape)

    def zeros(self, name, shape):
        self.md.tensors[name] = np.zeros(shape, dtype=np.float16)

    def conv_bn(self, name, cout, cin_g, k, small_gamma=False):
        self.he(name + ".w", (cout, cin_g, k, k))
        if small_gamma:
            self.uniform(name + ".gamma", (cout,), 0.2, 0.4)
        else:
            self.uniform(name + ".gamma", (cout,), 0.8, 1.2)
        self.normal(name + ".beta", (cout,), 0.05)
        self.normal(name + ".mean", (cout,), 0.05)
        self.uniform(name + ".var", (cout,), 0.8, 1.2)


def tiny_cnn(seed: int, hw: int = 32, classes: int = 10) -> ModelData:
    md = ModelData(ARCH_TINY_CNN, (hw, hw, 3, classes))
    g = _Gen(seed, md)
    cin = 3
    for i, cout in enumerate((16, 32, 64)):
        g.he(f"conv{i}.w", (cout, cin, 3, 3))
        g.zeros(f"conv{i}.b", (cout,))
        cin = cout
    g.he("fc.w", (classes, 64))
    g.zeros("fc.b", (classes,))
    return md


def resnet50(seed: int, hw: int = 224, classes: int = 1000) -> ModelData:
    md = ModelData(ARCH_RESNET50, (hw, hw, 3, classes))
    g = _Gen(seed, md)
    g.conv_bn("stem", 64, 3, 7)
    cin = 64
    for si, (nb, planes) in enumerate(zip(RESNET50_BLOCKS, RESNET50_PLANES), start=1):
        for bi in range(nb):
            p = f"s{si}b{bi}"
            g.conv_bn(p + ".c1", planes, cin, 1)
            g.conv_bn(p + ".c2", planes, planes, 3)
            g.conv_bn(p + ".c3", 4 * planes, planes, 1, small_gamma=True)
            if bi == 0:
                g.conv_bn(p + ".down", 4 * planes, cin, 1)
            cin = 4 * planes
    g.he("fc.w", (classes, cin))
    g.zeros("fc.b", (classes,))
    return md


def mobilenet_v2(seed: int, hw: int = 224, classes: int = 1000) -> ModelData:
    md = ModelData(ARCH_MOBILENETV2, (hw, hw, 3, classes))
    g = _Gen(seed, md)
    g.conv_bn("stem", 32, 3, 3)
    cin, idx = 32, 0
    for t, c, n, s in MOBILENETV2_CFG:
        for i in range(n):
            hid = cin * t
            p = f"b{idx}"
            if t != 1:
                g.conv_bn(p + ".expand", hid, cin, 1)
            g.conv_bn(p + ".dw", hid, 1, 3)
            g.conv_bn(p + ".project", c, hid, 1)
            cin = c
            idx += 1
    g.conv_bn("head", 1280, cin, 1)
    g.he("fc.w", (classes, 1280))
    g.zeros("fc.b", (classes,))
    return md


def encoder(seed: int, layers: int = 12, hidden: int = 768, heads: int = 12, ffn: int = 3072,
            seq: int = 128) -> ModelData:
    md = ModelData(ARCH_ENCODER, (layers, hidden, heads, ffn, seq))
    g = _Gen(seed, md)
    for i in range(layers):
        p = f"l{i}"
        for nm in ("q", "k", "v", "o"):
            g.normal(f"{p}.{nm}.w", (hidden, hidden), 0.02)
            g.normal(f"{p}.{nm}.b", (hidden,), 0.02)
        g.uniform(f"{p}.ln1.g", (hidden,), 0.8, 1.2)
        g.normal(f"{p}.ln1.b", (hidden,), 0.02)
        g.normal(f"{p}.ffn1.w", (ffn, hidden), 0.02)
        g.normal(f"{p}.ffn1.b", (ffn,), 0.02)
        g.normal(f"{p}.ffn2.w", (hidden, ffn), 0.02)
        g.normal(f"{p}.ffn2.b", (hidden,), 0.02)
        g.uniform(f"{p}.ln2.g", (hidden,), 0.8, 1.2)
        g.normal(f"{p}.ln2.b", (hidden,), 0.02)
    return md


def vgg19(seed: int, hw: int = 224, classes: int = 1000, fc: int = 4096) -> ModelData:
    assert hw % 32 == 0
    md = ModelData(ARCH_VGG19, (hw, hw, 3, classes, fc))
    g = _Gen(seed, md)
    cin, i = 3, 0
    for c in VGG19_CFG:
        if c == "M":
            continue
        g.he(f"conv{i}.w", (c, cin, 3, 3))
        g.normal(f"conv{i}.b", (c,), 0.02)
        cin, i = c, i + 1
    f = hw // 32
    g.he("fc1.w", (fc, cin, f, f))
    g.normal("fc1.b", (fc,), 0.02)
    g.he("fc2.w", (fc, fc))
    g.normal("fc2.b", (fc,), 0.02)
    g.he("fc.w", (classes, fc))
    g.normal("fc.b", (classes,), 0.02)
    return md


def vit(seed: int, hw: int = 224, classes: int = 1000, layers: int = 12, hidden: int = 768, heads: int = 12,
        ffn: int = 3072) -> ModelData:
    assert hw % VIT_PATCH == 0
    md = ModelData(ARCH_VIT, (hw, hw, 3, classes, layers, hidden, heads, ffn))
    g = _Gen(seed, md)
    n_tok = (hw // VIT_PATCH) ** 2 + 1
    g.normal("patch.w", (hidden, 3, VIT_PATCH, VIT_PATCH), 0.02)
    g.normal("patch.b", (hidden,), 0.02)
    g.normal("cls", (hidden,), 0.02)
    g.normal("pos", (n_tok, hidden), 0.02)
    for i in range(layers):
        p = f"l{i}"
        g.uniform(f"{p}.ln1.g", (hidden,), 0.8, 1.2)
        g.normal(f"{p}.ln1.b", (hidden,), 0.02)
        for nm in ("q", "k", "v", "o"):
            g.normal(f"{p}.{nm}.w", (hidden, hidden), 0.02)
            g.normal(f"{p}.{nm}.b", (hidden,), 0.02)
        g.uniform(f"{p}.ln2.g", (hidden,), 0.8, 1.2)
        g.normal(f"{p}.ln2.b", (hidden,), 0.02)
        g.normal(f"{p}.ffn1.w", (ffn, hidden), 0.02)
        g.normal(f"{p}.ffn1.b", (ffn,), 0.02)
        g.normal(f"{p}.ffn2.w", (hidden, ffn), 0.02)
        g.normal(f"{p}.ffn2.b", (hidden,), 0.02)
    g.uniform("ln.g", (hidden,), 0.8, 1.2)
    g.normal("ln.b", (hidden,), 0.02)
    g.normal("fc.w", (classes, hidden), 0.02)
    g.normal("fc.b", (classes,), 0.02)
    return md


def make_model(arch: int, seed: int, **kw) -> ModelData:
    return {ARCH_TINY_CNN: tiny_cnn, ARCH_RESNET50: resnet50, ARCH_MOBILENETV2: mobilenet_v2,
            ARCH_ENCODER: encoder, ARCH_VGG19: vgg19, ARCH_VIT: vit}[arch](seed, **kw)


# ----------------------------------------------------------------------------
# inputs
# ----------------------------------------------------------------------------

def image_batch(md: ModelData, batch: int, seed: int, dist: str = "normal") -> np.ndarray:
    """fp16 NHWC batch: N(0,1) (ResNet-50, MobileNetV2) or U[0,1) (tiny CNN)."""
    h, w, c = md.hyper[:3]
    n = batch * h * w * c
    name = f"input.b{batch}"
    x = rng.normal(seed, name, n) if dist == "normal" else rng.uniform(seed, name, n)
    return _f16(x, (batch, h, w, c))


def default_image_batch(md: ModelData, batch: int, seed: int) -> np.ndarray:
    return image_batch(md, batch, seed, "uniform" if md.arch == ARCH_TINY_CNN else "normal")


def token_batch(md: ModelData, batch: int, seed: int, min_len: int = 32):
    """Encoder input: fp16 [batch, seq, hidden] ~ N(0,1) and int32 valid lengths
    uniform on {min_len..seq} inclusive."""
    _, hidden, _, _, seq = md.hyper
    x = _f16(rng.normal(seed, f"tokens.b{batch}", batch * seq * hidden), (batch, seq, hidden))
    vl = rng.integers(seed, f"valid_len.b{batch}", batch, min(min_len, seq), seq).astype(np.int32)
    return x, vl


def poisson_arrivals_ns(seed: int, rate_per_s: float, duration_s: float) -> np.ndarray:
    """Integer-nanosecond arrival times of a Poisson process on [0, duration)."""
    n = int(rate_per_s * duration_s * 1.5) + 64
    gaps = rng.exponential(seed, "poisson", n, rate_per_s)
    t = np.cumsum(gaps)
    t = t[t < duration_s]
    return np.floor(t * 1e9).astype(np.int64)
