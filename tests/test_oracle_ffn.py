"""Pins for the oracle's expert FFN (Sec. 2.1 two-layer Transformer FFN) and the
MoE layer / stack built from it."""

import numpy as np
import pytest

from oracle import brute
from oracle import moqe_oracle as O
from paper_2310_02410_amd import workloads as W


def _layer(E=3, d=16, f=32, T=7, seed=0):
    wl = W.Workload("t", E=E, d=d, f=f, T=T, bits=(4,), seed=seed)
    return wl, W.make_layer(wl), W.make_tokens(wl)


def test_fp16_single_expert_equals_dense_ffn():
    wl, layer, x = _layer(E=1, d=32, f=64, T=9)
    ql = O.quantize_layer(layer, 16)
    y, (idx, gate, _, _) = O.moe_layer(x, ql)
    assert np.all(idx == 0) and np.all(gate == 1.0)
    w1 = layer["w1"][0].astype(np.float16).astype(np.float64)
    w2 = layer["w2"][0].astype(np.float16).astype(np.float64)
    # the textbook FFN written with einsum rather than the oracle's call chain
    h = np.maximum(0, np.einsum("tk,kn->tn", x.astype(np.float64), w1) + layer["b1"][0].astype(np.float64))
    ref = np.einsum("tk,kn->tn", h, w2) + layer["b2"][0].astype(np.float64)
    assert np.allclose(y, ref, rtol=1e-12, atol=1e-15)
    assert np.allclose(O.dense_ffn(x, w1, layer["b1"][0], w2, layer["b2"][0]), ref, rtol=1e-12, atol=1e-15)


@pytest.mark.parametrize("bits", (2, 3, 4, 8))
def test_every_expert_then_select(bits):
    wl, layer, x = _layer(E=3, d=32 if bits != 3 else 128, f=64 if bits != 3 else 128, T=5, seed=bits)
    ql = O.quantize_layer(layer, bits)
    y, (idx, gate, _, _) = O.moe_layer(x, ql)
    w1, w2 = O.layer_weights(ql)
    by = brute.expert_ffn_every_expert(
        x.astype(np.float64).tolist(), idx.tolist(), gate.tolist(), w1.tolist(),
        layer["b1"].astype(np.float64).tolist(), w2.tolist(), layer["b2"].astype(np.float64).tolist())
    assert np.allclose(y, np.array(by), rtol=1e-11, atol=1e-14)


def test_token_independence():
    wl, layer, x = _layer(E=4, d=32, f=64, T=11, seed=3)
    ql = O.quantize_layer(layer, 4)
    y, _ = O.moe_layer(x, ql)
    for t in (0, 5, 10):
        yt, _ = O.moe_layer(x[t:t + 1], ql)
        assert np.array_equal(yt[0], y[t])


def test_linear_in_gate_and_zero_input():
    wl, layer, x = _layer(E=2, d=32, f=64, T=6, seed=4)
    ql = O.quantize_layer(layer, 4)
    w1, w2 = O.layer_weights(ql)
    idx = np.array([0, 1, 0, 1, 1, 0])
    g = np.linspace(0.3, 0.9, 6)
    y1 = O.expert_ffn(x, idx, g, w1, layer["b1"], w2, layer["b2"])
    y2 = O.expert_ffn(x, idx, 2 * g, w1, layer["b1"], w2, layer["b2"])
    assert np.allclose(y2, 2 * y1, rtol=1e-15)
    z = np.zeros_like(x)
    y0 = O.expert_ffn(z, idx, g, w1, layer["b1"], w2, layer["b2"])
    for t in range(6):
        e = idx[t]
        ref = g[t] * (np.maximum(0, layer["b1"][e].astype(np.float64)) @ w2[e] + layer["b2"][e].astype(np.float64))
        assert np.allclose(y0[t], ref, rtol=1e-13, atol=1e-18)


def test_relu_and_bias_are_there():
    # one expert, identity-like weights: y = relu(x + b1) + b2
    d = 32
    eye = np.eye(d)[None]
    x = np.linspace(-2, 2, d)[None, :].astype(np.float16)
    b1 = np.full((1, d), 0.5, np.float16)
    b2 = np.full((1, d), -0.25, np.float16)
    y = O.expert_ffn(x, np.array([0]), np.array([1.0]), eye, b1, eye, b2)
    assert np.array_equal(y[0], np.maximum(0, x[0].astype(np.float64) + 0.5) - 0.25)


def test_weight_orientation():
    # w1 is [d, f]: a non-square layer only type-checks one way, and a planted
    # single weight must move exactly one hidden unit
    E, d, f = 1, 32, 64
    w1 = np.zeros((E, d, f)); w2 = np.zeros((E, f, d))
    w1[0, 3, 10] = 2.0
    w2[0, 10, 7] = 5.0
    x = np.zeros((1, d), np.float16); x[0, 3] = 1.5
    y = O.expert_ffn(x, np.array([0]), np.array([1.0]), w1, np.zeros((E, f)), w2, np.zeros((E, d)))
    ref = np.zeros(d); ref[7] = 1.5 * 2.0 * 5.0
    assert np.array_equal(y[0], ref)


def test_bits_converge_to_fp16():
    wl, layer, x = _layer(E=2, d=128, f=256, T=12, seed=5)
    ref, _ = O.moe_layer(x, O.quantize_layer(layer, 16))
    errs = []
    for b in (2, 3, 4):
        y, _ = O.moe_layer(x, O.quantize_layer(layer, b))
        errs.append(np.abs(y - ref).mean())
    assert errs[0] > errs[1] > errs[2]


def test_residual_and_stack():
    wl = W.Workload("s", E=2, d=32, f=64, T=5, bits=(4,), seed=6, layers=3)
    x = W.make_tokens(wl)
    qls = [O.quantize_layer(W.make_layer(wl, l), 4) for l in range(3)]
    xs = O.stack(x, qls)
    assert len(xs) == 4 and all(a.dtype == np.float16 for a in xs)
    cur = x
    for l in range(3):
        y, _ = O.moe_layer(cur, qls[l])
        nxt = (cur.astype(np.float64) + y).astype(np.float16)
        assert np.array_equal(nxt, xs[l + 1])
        cur = nxt


def test_route_override():
    wl, layer, x = _layer(E=3, d=32, f=64, T=4, seed=7)
    ql = O.quantize_layer(layer, 4)
    idx = np.array([2, 2, 0, 1]); g = np.array([1.0, 0.5, 0.25, 1.0])
    y, _ = O.moe_layer(x, ql, route_override=(idx, g))
    w1, w2 = O.layer_weights(ql)
    for t in range(4):
        ref = g[t] * O.dense_ffn(x[t:t + 1], w1[idx[t]], layer["b1"][idx[t]], w2[idx[t]], layer["b2"][idx[t]])[0]
        assert np.allclose(y[t], ref, rtol=1e-14)
