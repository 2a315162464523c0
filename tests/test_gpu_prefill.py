"""GPU parity of the many-token path of moqe_expert_ffn (tiled MFMA kernel, token rows staged
in LDS) against the oracle, alone and beside the decode kernel (per-segment path choice)."""

import numpy as np
import pytest
import torch

from oracle import moqe_oracle as O
from paper_2310_02410_amd import moqe, workloads as W
from tests.helpers import (FFN_TOL, assert_route_equal, dev, ffn_error, gpu_quantize_layer, make_route,
                           oracle_layer_output, route_to_numpy)

pytestmark = pytest.mark.gpu


@pytest.fixture
def prefill_min():
    """Sets the path-choice thresholds for one test (any batch size may use the tiled kernel,
    segments below n tokens always take the decode kernel) and restores the defaults afterwards."""

    def set_min(n):
        moqe.moqe_set_prefill_policy(n, 1, moqe.PREFILL_NEVER)

    yield set_min
    moqe.moqe_set_prefill_policy()


@pytest.fixture(params=("resident", "streamed"))
def tiled(request):
    """Runs a test once per tiled kernel: token rows resident in LDS where a pair's fit (the
    library's choice), and K staged in blocks throughout."""
    moqe.moqe_set_tiled_kernel(moqe.TILED_AUTO if request.param == "resident" else moqe.TILED_STREAMED)
    yield request.param
    moqe.moqe_set_tiled_kernel(moqe.TILED_AUTO)


def _parity(wl, bits, residual=False, forced=None, layer=None):
    layer = W.make_layer(wl) if layer is None else layer
    x = W.make_tokens(wl)
    ql = gpu_quantize_layer(layer, bits)
    xd = dev(x)
    if forced is None:
        r = moqe.moqe_route(xd, ql.w_gate)
        idx, gate, offs, perm = route_to_numpy(r)
        assert_route_equal((idx, gate, offs, perm), O.route(x, layer["w_gate"]), wl.T, wl.E)
    else:
        idx, gate = forced
        r = make_route(idx, gate, wl.E)
    y = moqe.moqe_expert_ffn(ql, xd, r, residual=xd if residual else None)
    torch.cuda.synchronize()
    ref = oracle_layer_output(x, layer, bits, idx, np.asarray(gate, dtype=np.float64), residual=residual)
    err = ffn_error(y.cpu().numpy(), ref)
    assert err <= FFN_TOL, f"{wl.name} int{bits}: max|err|/max|ref| = {err:.3e}"
    return np.bincount(idx, minlength=wl.E)


@pytest.mark.parametrize("bits", (8, 4, 3, 2))
@pytest.mark.parametrize("T", (1, 37, 150, 700))
def test_every_segment_through_the_tiled_kernel(prefill_min, tiled, bits, T):
    # threshold 1: also one-token segments take 64-token tiles (ragged in every way);
    # d=256, f=512: one and two K blocks for int2/int3, two and four for int4
    prefill_min(1)
    _parity(W.small(E=8, d=256, f=512, T=T, seed=70 + T), bits)


@pytest.mark.parametrize("bits", (8, 4, 3, 2))
def test_tiled_kernel_residual_and_odd_widths(prefill_min, tiled, bits):
    prefill_min(1)
    _parity(W.small(E=4, d=512, f=1024, T=90, seed=81), bits, residual=True)
    _parity(W.small(E=3, d=768, f=256, T=33, seed=83), bits)
    if bits != 3:
        # FFN2 with N = 64 channels: half a column block, two waves have nothing to load
        # (FFN1 has K = 64, too short for the tiled kernel: decode kernel)
        _parity(W.small(E=3, d=64, f=256, T=70, seed=82), bits)


@pytest.mark.parametrize("all_tiled", (False, True))
@pytest.mark.parametrize("bits", (4, 2))
def test_forced_segment_sizes(bits, all_tiled, prefill_min, tiled):
    """Segments of exactly 4, 5, 63, 64, 65 and 200 tokens, with full and ragged tiles.  With
    the decode kernel kept for segments below 5 tokens (thresholds 5, 65, never) the first goes
    there and the others to the tiled kernel; at the defaults this batch has 50 tokens per expert,
    so all of them, the 4-token one included, take the tiled kernel and no decode kernel is
    launched."""
    if all_tiled:
        moqe.moqe_set_prefill_policy()
    else:
        moqe.moqe_set_prefill_policy(5, 65, moqe.PREFILL_NEVER)
    wl = W.small(E=8, d=256, f=512, T=4 + 5 + 63 + 64 + 65 + 200, seed=84)
    sizes = (4, 5, 63, 64, 65, 200, 0, 0)
    idx = np.concatenate([np.full(n, e) for e, n in enumerate(sizes)])
    rng = np.random.default_rng(84)
    rng.shuffle(idx)
    gate = rng.uniform(0.2, 1.0, size=idx.size).astype(np.float32)
    counts = _parity(wl, bits, forced=(idx, gate))
    assert tuple(counts) == sizes


@pytest.mark.parametrize("bits", (4, 2))
def test_more_experts_than_the_kernel_keeps_segment_starts_for(prefill_min, bits):
    """160 experts: above 128 the tiled kernel reads the segment starts from memory instead of
    its LDS copy; threshold 1, so every non-empty segment (most of them a few tokens) is a tile."""
    prefill_min(1)
    counts = _parity(W.small(E=160, d=256, f=256, T=900, seed=87), bits)
    assert (counts > 0).sum() > 128


def test_wide_tile_shape_takes_large_launches():
    """Enough tiles for three full rounds of 64 x 256 tiles (T = 8192 over 4 experts, N = 4096):
    FFN1 runs the wide shape, FFN2 (N = 256) the narrow one; sampled rows against the oracle."""
    wl = W.small(E=4, d=256, f=4096, T=8192, seed=88)
    layer, x = W.make_layer(wl), W.make_tokens(wl)
    ql = gpu_quantize_layer(layer, 4)
    xd = dev(x)
    r = moqe.moqe_route(xd, ql.w_gate)
    idx, gate, offs, perm = route_to_numpy(r)
    y = moqe.moqe_expert_ffn(ql, xd, r).cpu().numpy()
    rows = np.random.default_rng(88).choice(wl.T, size=256, replace=False)
    rows = np.concatenate([rows, perm[offs[:-1][np.diff(offs) > 0]], perm[offs[1:][np.diff(offs) > 0] - 1]])
    ref = oracle_layer_output(x[rows], layer, 4, idx[rows], gate[rows].astype(np.float64))
    assert ffn_error(y[rows], ref) <= FFN_TOL


def test_largest_batch_the_tiled_kernel_addresses():
    """520,000 tokens with d_ff 4096: h holds 4.26e9 bytes and 2.13e9 elements, just inside the
    32-bit offsets of the tiled kernel (byte offsets below 2^32, element offsets below 2^31).
    Routing tables for every token, the FFN on sampled rows - the last rows of h and y, the
    highest addresses, among them."""
    T = 520_000
    wl = W.small(E=4, d=256, f=4096, T=T, seed=89)
    layer, x = W.make_layer(wl), W.make_tokens(wl)
    ql = gpu_quantize_layer(layer, 4)
    xd = dev(x)
    r = moqe.moqe_route(xd, ql.w_gate)
    idx, gate, offs, perm = route_to_numpy(r)
    assert_route_equal((idx, gate, offs, perm), O.route(x, layer["w_gate"]), T, wl.E)
    y = moqe.moqe_expert_ffn(ql, xd, r)
    torch.cuda.synchronize()
    rows = np.random.default_rng(89).choice(T, size=192, replace=False)
    rows = np.concatenate([rows, np.arange(T - 64, T), perm[offs[1:] - 1], perm[offs[:-1]]])
    ref = oracle_layer_output(x[rows], layer, 4, idx[rows], gate[rows].astype(np.float64))
    assert ffn_error(y[torch.from_numpy(rows).cuda()].cpu().numpy(), ref) <= FFN_TOL


def test_batch_beyond_the_tiled_kernels_offsets():
    """530,000 tokens with d_ff 4096: h has more than 2^31 elements and 2^32 bytes, which the
    tiled kernel does not address; both contractions stay with the decode kernel (64-bit
    offsets, token tables read from memory).  Sampled rows, the last ones among them."""
    T = 530_000
    wl = W.small(E=4, d=256, f=4096, T=T, seed=90)
    layer, x = W.make_layer(wl), W.make_tokens(wl)
    ql = gpu_quantize_layer(layer, 2)
    xd = dev(x)
    r = moqe.moqe_route(xd, ql.w_gate)
    idx, gate, offs, perm = route_to_numpy(r)
    assert_route_equal((idx, gate, offs, perm), O.route(x, layer["w_gate"]), T, wl.E)
    y = moqe.moqe_expert_ffn(ql, xd, r)
    torch.cuda.synchronize()
    rows = np.random.default_rng(90).choice(T, size=192, replace=False)
    rows = np.concatenate([rows, np.arange(T - 64, T), perm[offs[1:] - 1], perm[offs[:-1]]])
    ref = oracle_layer_output(x[rows], layer, 2, idx[rows], gate[rows].astype(np.float64))
    assert ffn_error(y[torch.from_numpy(rows).cuda()].cpu().numpy(), ref) <= FFN_TOL


def test_mixed_paths_under_zipf_load(prefill_min):
    """Zipf load with both kernels side by side (segments from 5 tokens on tiled, the rest by the
    decode kernel; the defaults would tile everything here): some experts stay empty; both
    kernels write disjoint rows of h and y."""
    moqe.moqe_set_prefill_policy(5, 65, moqe.PREFILL_NEVER)
    wl = W.small(E=16, d=256, f=512, T=200, routing="zipf", n_empty=3, seed=85)
    for bits in (8, 4, 3, 2):
        counts = _parity(wl, bits, residual=True)
    assert (counts >= 5).any() and ((counts > 0) & (counts < 5)).any() and (counts == 0).sum() >= 3


def test_threshold_does_not_change_results_beyond_tolerance(prefill_min):
    wl = W.small(E=8, d=256, f=512, T=300, seed=86)
    layer, x = W.make_layer(wl), W.make_tokens(wl)
    ql = gpu_quantize_layer(layer, 4)
    xd = dev(x)
    r = moqe.moqe_route(xd, ql.w_gate)
    outs = []
    for n in (1, 5, 1 << 20):
        prefill_min(n)
        outs.append(moqe.moqe_expert_ffn(ql, xd, r).cpu().numpy().astype(np.float64))
    scale = np.abs(outs[2]).max()
    assert np.abs(outs[0] - outs[2]).max() <= 2 * FFN_TOL * scale
    assert np.abs(outs[1] - outs[2]).max() <= 2 * FFN_TOL * scale


def test_config3_full_size(tiled):
    """Config 3: T=1536, Zipf(1.1) load over 32 experts (largest segment several hundred
    tokens, four experts empty), int4; every output compared."""
    wl = W.CONFIGS["c3"]
    counts = _parity(wl, 4)
    assert counts.max() > 300 and (counts == 0).sum() >= 4
