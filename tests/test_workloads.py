"""The synthetic workload generator: determinism, shapes, lattice exactness of the
router inputs (checked with the oracle's fp64 logits), realised load shape."""

import numpy as np
import pytest

from oracle import moqe_oracle as O
from paper_2310_02410_amd import workloads as W


def test_deterministic_and_shapes():
    wl = W.CONFIGS["c0"]
    a, b = W.make_layer(wl), W.make_layer(wl)
    for k in a:
        assert np.array_equal(a[k], b[k])
    assert a["w1"].shape == (4, 64, 256) and a["w1"].dtype == np.float32
    assert a["w2"].shape == (4, 256, 64) and a["b1"].dtype == np.float16
    assert a["w_gate"].shape == (64, 4) and a["w_gate"].dtype == np.float16
    x = W.make_tokens(wl)
    assert x.shape == (32, 64) and x.dtype == np.float16
    assert not np.array_equal(W.make_layer(wl, 1)["w1"], a["w1"])


def test_weight_distribution():
    wl = W.small(E=2, d=256, f=512)
    w = W.make_layer(wl)["w1"]
    out = np.abs(w) == np.float32(0.16)
    assert 0.0003 < out.mean() < 0.003
    body = w[~out]
    assert abs(body.std() - 0.02) < 0.001 and abs(body.mean()) < 0.001


@pytest.mark.parametrize("name", ("c0", "c1", "c3"))
def test_router_inputs_are_exact_in_fp32(name):
    wl = W.CONFIGS[name]
    if name != "c0":
        wl = W.small(name, E=wl.E, d=wl.d, f=32, T=min(wl.T, 256), routing=wl.routing, n_empty=wl.n_empty)
    layer, x = W.make_layer(wl), W.make_tokens(wl)
    x64, g64 = x.astype(np.float64), layer["w_gate"].astype(np.float64)
    assert np.all(x64 * 16 == np.rint(x64 * 16)) and np.all(g64 * 512 == np.rint(g64 * 512))
    # worst-case partial sum stays inside fp32's 24-bit significand on the 2^-13 lattice
    assert (np.abs(x64) @ np.abs(g64)).max() < 2048.0
    l = O.route_logits(x, layer["w_gate"])
    assert np.array_equal(l.astype(np.float32).astype(np.float64), l)
    # fp32 accumulation in a different order gives the same numbers
    l32 = np.zeros(l.shape, np.float32)
    for k in reversed(range(wl.d)):
        l32 += x[:, k:k + 1].astype(np.float32) * layer["w_gate"][k:k + 1, :].astype(np.float32)
    assert np.array_equal(l32.astype(np.float64), l)
    m = O.top2_margin(l)
    assert np.all((m == 0) | (m >= 2.0 ** -13))


def test_uniform_load_is_spread():
    wl = W.small(E=32, d=1024, f=32, T=512)
    idx, _, offs, _ = O.route(W.make_tokens(wl), W.make_layer(wl)["w_gate"])
    counts = np.diff(offs)
    assert counts.min() >= 1 and counts.max() < 48


def test_zipf_load_shape():
    wl = W.small(E=32, d=1024, f=32, T=1536, routing="zipf", n_empty=4)
    layer = W.make_layer(wl)
    _, _, offs, _ = O.route(W.make_tokens(wl), layer["w_gate"])
    counts = np.sort(np.diff(offs))[::-1]
    assert (counts == 0).sum() >= 4
    target = np.arange(1, 29) ** -1.1
    target = 1536 * target / target.sum()
    assert abs(counts[0] - target[0]) < 0.25 * target[0]      # ~436 tokens in the largest segment
    assert abs(counts[1] - target[1]) < 0.35 * target[1]
    assert counts[:8].sum() > 0.6 * 1536


def test_c4_variants():
    v = W.c4_variants()
    assert [(w.T, w.routing) for w in v] == [(24, "uniform"), (24, "zipf"), (4096, "uniform"), (4096, "zipf")]
    assert all(w.layers == 12 and w.bits == (2,) for w in v)
