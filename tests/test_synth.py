"""The seeded generator: known-answer test, reproducibility, distribution moments."""
import os

import numpy as np

import synth
from synth import rng

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_splitmix64_known_answer():
    want = [int(l) for l in open(os.path.join(GOLDEN, "splitmix64_kat.txt")) if l[0] != "#"]
    with np.errstate(over="ignore"):
        idx = np.arange(1, 6, dtype=np.uint64)
        got = rng._mix(np.uint64(1234567) + idx * rng._GOLDEN)
    assert [int(g) for g in got] == want


def test_streams_reproducible_and_distinct():
    a = rng.normal(5, "a", 1000)
    assert np.array_equal(a, rng.normal(5, "a", 1000))
    assert not np.array_equal(a, rng.normal(6, "a", 1000))
    assert not np.array_equal(a, rng.normal(5, "b", 1000))
    # counter-based: a prefix of a longer draw is the shorter draw
    assert np.array_equal(rng.uniform(5, "a", 10), rng.uniform(5, "a", 100)[:10])


def test_moments():
    u = rng.uniform(1, "u", 200000, 2.0, 4.0)
    assert 2.0 <= u.min() and u.max() < 4.0 and abs(u.mean() - 3.0) < 0.01
    z = rng.normal(1, "z", 200000, 1.0, 2.0)
    assert abs(z.mean() - 1.0) < 0.02 and abs(z.std() - 2.0) < 0.02
    k = rng.integers(1, "k", 200000, 32, 128)
    assert k.min() == 32 and k.max() == 128 and abs(k.mean() - 80.0) < 0.5


def test_poisson_schedule():
    t = synth.poisson_arrivals_ns(synth.SEEDS["colocation"], 200.0, 10.0)
    assert t.dtype == np.int64 and np.all(np.diff(t) >= 0) and t[-1] < 10_000_000_000
    assert abs(len(t) - 2000) <= 3 * np.sqrt(2000)
    assert abs(np.diff(t).mean() - 5e6) < 0.4e6
    assert np.array_equal(t, synth.poisson_arrivals_ns(synth.SEEDS["colocation"], 200.0, 10.0))


def test_he_normal_and_container():
    md = synth.tiny_cnn(3)
    w = md.tensors["conv2.w"].astype(np.float64)
    assert w.shape == (64, 32, 3, 3) and abs(w.std() - (2.0 / 288) ** 0.5) < 0.003
    assert not md.tensors["conv0.b"].any()
    blob = synth.pack(md)
    assert blob[:4] == b"STRW" and len(blob) % 64 == 0
    # the fp16 payload of the last tensor sits at the end of the blob
    last = list(md.tensors.values())[-1].tobytes()
    assert last in blob[-128:] or blob.rstrip(b"\0").endswith(last.rstrip(b"\0"))


def test_input_shapes():
    md = synth.resnet50(1, hw=32)
    x = synth.default_image_batch(md, 2, 9)
    assert x.shape == (2, 32, 32, 3) and x.dtype == np.float16
    enc = synth.encoder(1, layers=1, hidden=64, heads=2, ffn=128, seq=16)
    tok, vl = synth.token_batch(enc, 5, 2, min_len=4)
    assert tok.shape == (5, 16, 64) and vl.dtype == np.int32 and vl.min() >= 4 and vl.max() <= 16
