"""Config 4: a stack of 12 int2 MoE layers with an fp16 residual stream,
x_{l+1} = fp16(x_l + MoE_l(x_l)), at T = 24 and T = 4096 with uniform and Zipf(1.1) routing.

Parity is checked layer by layer with teacher forcing: the oracle is given the residual
stream the GPU produced for layer l (so differences cannot compound or flip routes further
down) and must reproduce layer l's routing exactly and its output within the FFN tolerance.
From layer 1 on the router's inputs are no longer on the generator's lattice, so a token whose
two best logits are closer than 2^-12 in the oracle may legitimately go to either of them; such
tokens are counted, their FFN is evaluated under the GPU's choice, and there must be few.
Every token of every layer is compared, at T = 4096 too (the oracle takes a few seconds per
layer at that size), so every 64-token tile of the tiled kernel, ragged ones and segment ends
included, is checked and not sampled.
One test per layer keeps every test well under a minute; they run in order and share the
residual streams through a module-level store."""

import numpy as np
import pytest
import torch

from oracle import moqe_oracle as O
from paper_2310_02410_amd import moqe, workloads as W
from tests.helpers import FFN_TOL, GATE_RTOL, dev, ffn_error, gpu_quantize_layer, route_to_numpy

pytestmark = pytest.mark.gpu

BITS = 2
NEAR_TIE = 2.0 ** -12
VARIANTS = {v.name: v for v in W.c4_variants()}   # c4_T24_uniform, c4_T24_zipf, c4_T4096_uniform, c4_T4096_zipf
STATE = {}                                        # variant -> device fp16 residual stream entering the next layer


class LazyWeights:
    """Oracle weights of one matrix stack, dequantized per expert on first use."""

    def __init__(self, q, s):
        self.q, self.s, self.cache = q, s, {}

    def __getitem__(self, e):
        e = int(e)
        if e not in self.cache:
            self.cache[e] = O.dequantize(self.q[e], self.s[e])
        return self.cache[e]


def _check_variant(name, layer, oq, w1, w2, ql_gpu, lidx):
    wl = VARIANTS[name]
    gate_key = "w_gate_zipf" if wl.routing == "zipf" else "w_gate"
    if lidx == 0:
        STATE[name] = dev(W.make_tokens(wl))
    assert name in STATE, "layers must run in order"
    xd = STATE[name]
    x = xd.cpu().numpy()
    qg = moqe.QuantLayer(BITS, ql_gpu.E, ql_gpu.d, ql_gpu.f, ql_gpu.codes1, ql_gpu.scales1, ql_gpu.bias1,
                         ql_gpu.codes2, ql_gpu.scales2, ql_gpu.bias2, dev(layer[gate_key]))
    y, r = moqe.moqe_moe_layer(qg, xd, residual=xd)
    torch.cuda.synchronize()
    idx, gate, offs, perm = route_to_numpy(r)

    # ---- routing: exact, except near-ties from layer 1 on ----
    logits = O.route_logits(x, layer[gate_key])
    ridx, rgate, _, _ = O.route_from_logits(logits)
    differ = np.flatnonzero(idx != ridx)
    if differ.size:
        assert lidx > 0, "layer 0 inputs are on the lattice: routing must be exact"
        srt = np.sort(logits[differ], axis=1)
        assert np.all(srt[:, -1] - srt[:, -2] < NEAR_TIE), "a token with a clear margin went elsewhere"
        second = np.argsort(logits[differ], axis=1)[:, -2]
        assert np.array_equal(idx[differ], second), "a near-tie token went to neither of its two best experts"
        assert differ.size <= max(2, wl.T // 500), f"{differ.size} near-ties in {wl.T} tokens"
    same = idx == ridx
    assert np.allclose(gate[same], rgate[same], rtol=4 * GATE_RTOL, atol=0)
    counts = np.bincount(idx, minlength=wl.E)
    assert np.array_equal(offs, np.concatenate([[0], np.cumsum(counts)]))
    assert np.array_equal(perm, np.argsort(idx, kind="stable"))

    # ---- output under the GPU's route, every token ----
    sel = np.arange(wl.T)
    ref = O.expert_ffn(x[sel], idx[sel], gate[sel].astype(np.float64), w1, layer["b1"], w2, layer["b2"],
                       residual=x[sel])
    got = y.cpu().numpy()[sel]
    err = ffn_error(got, ref)
    assert err <= FFN_TOL, f"{name} layer {lidx}: {err:.3e}"
    # the MoE contribution on its own (the residual dominates the output's magnitude)
    inc_ref = ref - x[sel].astype(np.float64)
    inc_err = np.abs(got.astype(np.float64) - x[sel].astype(np.float64) - inc_ref).max()
    assert inc_err <= 2.0 ** -8 * max(1.0, np.abs(ref).max()), f"{name} layer {lidx}: increment off by {inc_err:.3e}"
    STATE[name] = y
    return counts


@pytest.mark.parametrize("lidx", range(12))
def test_stack_layer(lidx):
    base = W.CONFIGS["c4"]
    layer = W.make_layer(base, layer=lidx, zipf_gate=True)
    ql_gpu = gpu_quantize_layer(layer, BITS)
    oq = O.quantize_layer(layer, BITS)
    w1, w2 = LazyWeights(oq["q1"], oq["s1"]), LazyWeights(oq["q2"], oq["s2"])
    for name in VARIANTS:
        counts = _check_variant(name, layer, oq, w1, w2, ql_gpu, lidx)
        if lidx == 0 and name == "c4_T4096_zipf":
            assert counts.max() > 800 and (counts == 0).sum() >= 4
        if lidx == 0 and name == "c4_T4096_uniform":
            assert counts.min() > 60


def test_stack_finished():
    assert set(STATE) == set(VARIANTS)
    for name, y in STATE.items():
        assert torch.isfinite(y).all(), name
    STATE.clear()
