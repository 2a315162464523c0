"""GPU parity of the tiled kernel that keeps a pair's token rows resident in LDS (pairs of 64 tokens
for K <= 1024, of 16 tokens up to K = 4096) against the oracle, next to the kernel that stages K in
blocks: every shape the work split, the staging and the unit hand-out distinguish."""

import numpy as np
import pytest
import torch

from oracle import moqe_oracle as O
from paper_2310_02410_amd import moqe, workloads as W
from tests.helpers import FFN_TOL, dev, ffn_error, gpu_quantize_layer, make_route, oracle_layer_output

pytestmark = pytest.mark.gpu


@pytest.fixture
def all_tiled():
    """Every segment, however small, takes the tiled kernel; defaults restored afterwards."""
    moqe.moqe_set_prefill_policy(1, 1, moqe.PREFILL_NEVER)
    yield
    moqe.moqe_set_prefill_policy()
    moqe.moqe_set_tiled_kernel(moqe.TILED_AUTO)


def _run(wl, bits, idx, gate, residual=False, codec="linear"):
    layer, x = W.make_layer(wl), W.make_tokens(wl)
    xd = dev(x)
    r = make_route(idx, gate, wl.E)
    g64 = np.asarray(gate, dtype=np.float64)
    if codec == "log":
        ql = moqe.quantize_layer(dev(layer["w1"]), dev(layer["b1"]), dev(layer["w2"]), dev(layer["b2"]), bits,
                                 dev(layer["w_gate"]), codec=moqe.CODEC_LOG)
        q1, s1 = O.quantize_log(layer["w1"], bits)
        q2, s2 = O.quantize_log(layer["w2"], bits)
        ref = O.expert_ffn(x, idx, g64, O.dequantize_log(q1, s1, bits), layer["b1"], O.dequantize_log(q2, s2, bits),
                           layer["b2"], residual=x if residual else None)
    else:
        ql = gpu_quantize_layer(layer, bits)
        ref = oracle_layer_output(x, layer, bits, idx, g64, residual=residual)
    out = {}
    for name, which in (("resident", moqe.TILED_RESIDENT), ("streamed", moqe.TILED_STREAMED)):
        moqe.moqe_set_tiled_kernel(which)
        y = moqe.moqe_expert_ffn(ql, xd, r, residual=xd if residual else None)
        torch.cuda.synchronize()
        out[name] = y.cpu().numpy()
        err = ffn_error(out[name], ref)
        assert err <= FFN_TOL, f"{wl.name} {codec} {bits} bits, {name}: max|err|/max|ref| = {err:.3e}"
    return out, ref


def _forced(sizes, seed):
    idx = np.concatenate([np.full(n, e) for e, n in enumerate(sizes)]).astype(np.int32)
    rng = np.random.default_rng(seed)
    rng.shuffle(idx)
    return idx, rng.uniform(0.2, 1.0, size=idx.size).astype(np.float32)


@pytest.mark.parametrize("bits", (4, 3, 2))
def test_ragged_pairs_of_every_height(all_tiled, bits):
    """Segments that end in a pair of 1, 2, 3 and 4 token tiles (1, 17, 33, 49 and 64 rows), full
    pairs in front of some of them, an empty expert; d = 1024 (the largest K that stays resident,
    four or eight chunks per column tile) and d_ff = 512 (FFN2 resident too, K = 512)."""
    sizes = (1, 17, 33, 49, 64, 65, 0, 64 + 64 + 3)
    idx, gate = _forced(sizes, 91)
    _run(W.small(E=8, d=1024, f=512, T=int(sum(sizes)), seed=91), bits, idx, gate, residual=True)


@pytest.mark.parametrize("bits", (4, 2))
def test_more_pairs_than_workgroups(all_tiled, bits):
    """A narrow FFN1 (128 channels at int4: four units per pair, half a round; 256 at int2) and
    20,000 tokens: 300-odd pairs for 256 workgroups, so every workgroup takes up several pairs,
    some of them ragged."""
    wl = W.small(E=24, d=512, f=128 if bits == 4 else 256, T=20000, seed=92)
    rng = np.random.default_rng(92)
    idx = rng.integers(0, 24, size=wl.T).astype(np.int32)
    idx[idx == 5] = 6  # an empty expert in the middle
    gate = rng.uniform(0.2, 1.0, size=wl.T).astype(np.float32)
    layer, x = W.make_layer(wl), W.make_tokens(wl)
    xd = dev(x)
    r = make_route(idx, gate, wl.E)
    ql = gpu_quantize_layer(layer, bits)
    moqe.moqe_set_tiled_kernel(moqe.TILED_AUTO)
    y = moqe.moqe_expert_ffn(ql, xd, r).cpu().numpy()
    rows = np.random.default_rng(93).choice(wl.T, size=1500, replace=False)
    perm = np.argsort(idx, kind="stable")
    offs = np.concatenate([[0], np.cumsum(np.bincount(idx, minlength=wl.E))])
    ne = np.diff(offs) > 0
    rows = np.unique(np.concatenate([rows, perm[offs[:-1][ne]], perm[offs[1:][ne] - 1]]))
    ref = oracle_layer_output(x[rows], layer, bits, idx[rows], gate[rows].astype(np.float64))
    assert ffn_error(y[rows], ref) <= FFN_TOL
    moqe.moqe_set_tiled_kernel(moqe.TILED_STREAMED)
    y2 = moqe.moqe_expert_ffn(ql, xd, r).cpu().numpy().astype(np.float64)
    assert np.abs(y2 - y).max() <= 2 * FFN_TOL * np.abs(y2).max()


@pytest.mark.parametrize("bits", (4, 3, 2))
def test_window_of_two_chunks_and_partial_rounds(all_tiled, bits):
    """Column tiles with six chunks (d = 768 at int4) or two (d_ff = 256 at int4, 512 at int3 / int2):
    a window of two chunks instead of four; and, at int4, d = 128: FFN2 has four units per pair,
    half a round (FFN1, K = 128, stays with the decode kernel)."""
    sizes = (40, 130, 7, 64)
    idx, gate = _forced(sizes, 94)
    T = int(sum(sizes))
    if bits == 4:
        _run(W.small(E=4, d=768, f=256, T=T, seed=94), bits, idx, gate)
        _run(W.small(E=4, d=128, f=512, T=T, seed=97), bits, idx, gate, residual=True)
    else:
        _run(W.small(E=4, d=512, f=512, T=T, seed=94), bits, idx, gate)


@pytest.mark.parametrize("bits", (4, 3, 2))
def test_log_scale_codes_resident(all_tiled, bits):
    sizes = (70, 3, 50, 0)
    idx, gate = _forced(sizes, 95)
    _run(W.small(E=4, d=512, f=1024, T=int(sum(sizes)), seed=95), bits, idx, gate, residual=True, codec="log")


@pytest.mark.parametrize("bits", (4, 3, 2))
def test_offsets_left_in_the_sum_cost_no_accuracy(all_tiled, bits):
    """The resident kernel leaves a constant per code position in the unpacked weights and takes
    sum_k a_k c_k out once per pair.  Worst case for that: long K (1024), activations that are all
    positive and far from zero mean (FFN2 reads h after ReLU; here x itself is shifted to mean 3),
    so that the constants' sum is thousands of times the signal.  Same bound as everywhere."""
    wl = W.small(E=4, d=1024, f=1024, T=200, seed=96)
    layer, x = W.make_layer(wl), W.make_tokens(wl)
    x = (np.abs(x.astype(np.float32)) + 3.0).astype(np.float16)
    sizes = (64, 100, 33, 3)
    idx, gate = _forced(sizes, 96)
    xd = dev(x)
    r = make_route(idx, gate, wl.E)
    ql = gpu_quantize_layer(layer, bits)
    ref = oracle_layer_output(x, layer, bits, idx, gate.astype(np.float64))
    moqe.moqe_set_tiled_kernel(moqe.TILED_AUTO)
    err = ffn_error(moqe.moqe_expert_ffn(ql, xd, r).cpu().numpy(), ref)
    assert err <= FFN_TOL, f"int{bits}: {err:.3e}"


def test_resident_and_streamed_agree_at_the_benchmarked_size(all_tiled):
    """One layer of the 12-layer int2 stack at 4096 tokens (E = 32, d = 1024, d_ff = 4096): FFN1
    through both tiled kernels, every element of h within two fp16 units of the other kernel's
    (they add the same products in different groupings)."""
    wl = [v for v in W.c4_variants() if v.name == "c4_T4096_uniform"][0]
    layer, x = W.make_layer(wl), W.make_tokens(wl)
    ql = gpu_quantize_layer(layer, 2)
    xd = dev(x)
    r = moqe.moqe_route(xd, ql.w_gate)
    hs = []
    for which in (moqe.TILED_AUTO, moqe.TILED_STREAMED):
        moqe.moqe_set_tiled_kernel(which)
        h = torch.empty((wl.T, wl.f), dtype=torch.float16, device="cuda")
        moqe.moqe_expert_ffn1(ql, xd, r, h)
        hs.append(h.float().cpu().numpy())
    scale = np.abs(hs[1]).max()
    assert np.abs(hs[0] - hs[1]).max() <= 2e-3 * scale


@pytest.mark.parametrize("bits", (4, 3, 2))
def test_pairs_of_16_tokens_for_long_k(all_tiled, bits):
    """K = 4096, 2048 and 1536 (FFN2 of d_ff that size): pairs of 16 tokens, ragged ones of 1, 15
    and 5 rows, several pairs per expert, an empty expert; few pairs, so units of one column tile.
    K = 1536 has 12 chunks per column tile at int4 (window of four) and 6 at int2 (of two); int3
    needs K to be a multiple of 512 there and stays with the staged kernel."""
    sizes = (1, 15, 16, 17, 33, 0, 70, 5)
    idx, gate = _forced(sizes, 98)
    T = int(sum(sizes))
    E, d, f = 8, 512, 4096
    assert moqe.moqe_contraction_path(bits, T, E, f, d) == moqe.PATH_TILED_STAGED
    moqe.moqe_set_tiled_kernel(moqe.TILED_RESIDENT)
    assert moqe.moqe_contraction_path(bits, T, E, f, d) == moqe.PATH_TILED_RESIDENT
    _run(W.small(E=E, d=d, f=f, T=T, seed=98), bits, idx, gate, residual=True)
    _run(W.small(E=E, d=d, f=2048, T=T, seed=99), bits, idx, gate)
    _run(W.small(E=E, d=256, f=1536, T=T, seed=100), bits, idx, gate, residual=True)


@pytest.mark.parametrize("bits", (4, 2))
def test_pairs_of_16_tokens_many_per_workgroup(all_tiled, bits):
    """6000 tokens on 24 experts with K = 4096: 380-odd pairs of 16 for 256 workgroups, units of
    two column tiles; sampled rows against the oracle, everything against the staged kernel."""
    wl = W.small(E=24, d=256, f=4096, T=6000, seed=101)
    rng = np.random.default_rng(101)
    idx = rng.integers(0, 24, size=wl.T).astype(np.int32)
    idx[idx == 5] = 6
    gate = rng.uniform(0.2, 1.0, size=wl.T).astype(np.float32)
    out, _ = _run(wl, bits, idx, gate)
    assert np.abs(out["resident"].astype(np.float64) - out["streamed"]).max() <= 2 * FFN_TOL * np.abs(out["streamed"]).max()


@pytest.mark.parametrize("bits", (4, 3, 2))
def test_pairs_of_16_tokens_log_codes_and_offsets(all_tiled, bits):
    """Log-scale codes through the pairs of 16 (no offsets to take out), and the worst case for the
    offsets that linear codes leave in the sum: K = 4096 with all-positive rows far from zero
    mean (FFN1 of a layer with d_model 4096, rows shifted to mean 3)."""
    sizes = (20, 3, 50, 0)
    idx, gate = _forced(sizes, 102)
    _run(W.small(E=4, d=512, f=4096, T=int(sum(sizes)), seed=102), bits, idx, gate, residual=True, codec="log")
    wl = W.small(E=4, d=4096, f=256, T=200, seed=103)
    layer, x = W.make_layer(wl), W.make_tokens(wl)
    x = (np.abs(x.astype(np.float32)) + 3.0).astype(np.float16)
    idx, gate = _forced((64, 100, 33, 3), 103)
    xd = dev(x)
    r = make_route(idx, gate, wl.E)
    ql = gpu_quantize_layer(layer, bits)
    ref = oracle_layer_output(x, layer, bits, idx, gate.astype(np.float64))
    moqe.moqe_set_tiled_kernel(moqe.TILED_RESIDENT)
    assert moqe.moqe_contraction_path(bits, wl.T, wl.E, wl.d, wl.f) == moqe.PATH_TILED_RESIDENT
    err = ffn_error(moqe.moqe_expert_ffn(ql, xd, r).cpu().numpy(), ref)
    assert err <= FFN_TOL, f"int{bits}: {err:.3e}"


def test_default_path_at_mid_sized_batches():
    """What the library picks by itself between 65 and 1024 tokens on the benchmark layer - the
    decode-sized kernel up to 128 tokens, then both contractions on the resident kernel up to 16
    tokens per expert, FFN2 staged beyond - against the oracle."""
    moqe.moqe_set_prefill_policy()
    moqe.moqe_set_tiled_kernel(moqe.TILED_AUTO)
    base = W.CONFIGS["c1"]
    layer = W.make_layer(base)
    for bits in (4, 2):
        ql = gpu_quantize_layer(layer, bits)
        w1, w2 = O.layer_weights(O.quantize_layer(layer, bits))
        for T in (128, 129, 512, 600):
            wl = W.small(E=base.E, d=base.d, f=base.f, T=T, seed=104 + T, outlier_prob=base.outlier_prob)
            x = W.make_tokens(wl)
            xd = dev(x)
            r = moqe.moqe_route(xd, ql.w_gate)
            want1 = moqe.PATH_DECODE_SMALL if T <= 128 else moqe.PATH_TILED_RESIDENT
            want2 = want1 if T <= 16 * base.E else moqe.PATH_TILED_STAGED
            assert moqe.moqe_contraction_path(bits, T, base.E, base.d, base.f) == want1
            assert moqe.moqe_contraction_path(bits, T, base.E, base.f, base.d) == want2
            y = moqe.moqe_expert_ffn(ql, xd, r).cpu().numpy()
            idx, gate = r.expert_idx.cpu().numpy(), r.gate.cpu().numpy().astype(np.float64)
            ref = O.expert_ffn(x, idx, gate, w1, layer["b1"], w2, layer["b2"], residual=None)
            err = ffn_error(y, ref)
            assert err <= FFN_TOL, f"int{bits} T={T}: {err:.3e}"
        del w1, w2


def test_offset_sums_go_out_slab_by_slab():
    """FFN2 reads h after ReLU: all-positive rows over K = 4096, so the constants the unpack leaves
    in the sum add up to thousands of times the signal, and taken out in one piece their fp32
    rounding showed (2.3e-3 of the largest output on this case, int2, against the bound's 2e-3).
    The pairs of 16 tokens take them out per 512 of K: the error is back at the exact unpack's."""
    from tests.test_gpu_random_sweep import run_mid_case
    case = (2, 0, 4, 1024, 4096, 128, False, False, moqe.TILED_RESIDENT, (5, 65, moqe.PREFILL_NEVER), 209828)
    assert moqe.moqe_contraction_path(2, 128, 4, 4096, 1024) == moqe.PATH_DECODE_SMALL  # (default thresholds)
    err = run_mid_case(case)
    assert err <= 1e-3, f"{err:.3e}"
