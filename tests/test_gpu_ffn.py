"""GPU parity of moqe_expert_ffn against the oracle (Sec. 2.1 expert FFN with
App. A dequantization): max|err| <= 2e-3 max|ref| on the [T,d] output."""

import numpy as np
import pytest
import torch

from oracle import moqe_oracle as O
from paper_2310_02410_amd import moqe, workloads as W
from tests.helpers import (FFN_TOL, assert_route_equal, dev, ffn_error, gpu_quantize_layer, make_route,
                           oracle_layer_output, route_to_numpy)

pytestmark = pytest.mark.gpu


def _layer_parity(wl, bits, residual=False, forced=None):
    layer, x = W.make_layer(wl), W.make_tokens(wl)
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
    ref = oracle_layer_output(x, layer, bits, idx, gate.astype(np.float64), residual=residual)
    err = ffn_error(y.cpu().numpy(), ref)
    assert err <= FFN_TOL, f"{wl.name} int{bits}: max|err|/max|ref| = {err:.3e}"
    return err


def test_config0():
    _layer_parity(W.CONFIGS["c0"], 4)


@pytest.mark.parametrize("bits", (8, 4, 3, 2))
@pytest.mark.parametrize("T", (1, 37, 150))
def test_small_layer(bits, T):
    # d=128 (one wave slice of 4 steps), f=256 (8 steps); T=150 over 8 experts gives
    # segments longer than one 16-token tile with ragged tails
    _layer_parity(W.small(T=T), bits)


@pytest.mark.parametrize("bits", (8, 4, 3, 2))
def test_split_k_shapes(bits):
    # d=512 -> 16 steps, f=2048 -> 16 steps x 4 waves; d=768/f=3072 -> 24 steps (x4)
    _layer_parity(W.small(E=4, d=512, f=2048, T=40, seed=21), bits)
    _layer_parity(W.small(E=3, d=768, f=3072, T=21, seed=22), bits)


@pytest.mark.parametrize("bits", (8, 4, 3, 2))
def test_residual_fused(bits):
    _layer_parity(W.small(T=50, seed=23), bits, residual=True)


@pytest.mark.parametrize("bits", (4, 2))
def test_forced_routes(bits):
    wl = W.small(E=8, d=128, f=256, T=40, seed=24)
    rng = np.random.default_rng(1)
    # everything to one expert (others empty), gate values arbitrary
    _layer_parity(wl, bits, forced=(np.full(40, 5, np.int32), rng.uniform(0.1, 1.0, 40).astype(np.float32)))
    # last expert only gets the last token
    idx = np.zeros(40, np.int32)
    idx[-1] = 7
    _layer_parity(wl, bits, forced=(idx, np.ones(40, np.float32)))


def test_zero_input_closed_form():
    # x = 0 => y = g (max(0, b1) W2' + b2): FFN2 and the biases alone
    wl = W.small(E=4, d=128, f=256, T=9, seed=25)
    layer = W.make_layer(wl)
    ql = gpu_quantize_layer(layer, 4)
    x = np.zeros((9, 128), np.float16)
    idx = np.arange(9, dtype=np.int32) % 4
    g = np.linspace(0.2, 1.0, 9).astype(np.float32)
    y = moqe.moqe_expert_ffn(ql, dev(x), make_route(idx, g, 4)).cpu().numpy()
    ref = oracle_layer_output(x, layer, 4, idx, g.astype(np.float64))
    assert ffn_error(y, ref) <= FFN_TOL


@pytest.mark.parametrize("name,bits", (("c1", 8), ("c1", 4), ("c2", 3), ("c2", 2)))
def test_decode_configs_full_size(name, bits):
    """Benchmark decode layers at full size: E=32, d=1024, f=4096, T=24 (int8: Table 2's 8-bit
    row on C1's layer)."""
    _layer_parity(W.CONFIGS[name], bits)


def test_deterministic_output():
    wl = W.small(E=8, d=512, f=2048, T=33, seed=26)
    layer, x = W.make_layer(wl), W.make_tokens(wl)
    ql = gpu_quantize_layer(layer, 2)
    xd = dev(x)
    r = moqe.moqe_route(xd, ql.w_gate)
    a = moqe.moqe_expert_ffn(ql, xd, r).cpu().numpy()
    b = moqe.moqe_expert_ffn(ql, xd, r).cpu().numpy()
    assert np.array_equal(a.view(np.uint16), b.view(np.uint16))


@pytest.mark.parametrize("T", (1, 24, 150))
def test_fp16_experts_small(T):
    """Unquantized fp16 experts (bits = 16) against the oracle's 16-bit path; they run on the
    tiled kernel at every batch size."""
    _layer_parity(W.small(E=4, d=256, f=512, T=T, seed=60 + T), 16)
    _layer_parity(W.small(E=3, d=384, f=256, T=T, seed=61 + T), 16, residual=True)


def test_fp16_experts_decode_config():
    """C1's layer with fp16 experts: the baseline row of the bit-width comparison."""
    _layer_parity(W.CONFIGS["c1"], 16)


def _log_layer_parity(wl, bits=4, residual=False, launch_mode=None, sample=None):
    """A layer of log-scale codes (App. A: A' = P s 2^Q) through the FFN calls, against the
    oracle's expert FFN on the oracle's log-dequantized weights."""
    layer, x = W.make_layer(wl), W.make_tokens(wl)
    ql = moqe.quantize_layer(dev(layer["w1"]), dev(layer["b1"]), dev(layer["w2"]), dev(layer["b2"]), bits,
                             dev(layer["w_gate"]), codec=moqe.CODEC_LOG)
    q1, s1 = O.quantize_log(layer["w1"], bits)
    q2, s2 = O.quantize_log(layer["w2"], bits)
    assert np.array_equal(ql.codes1.cpu().numpy(), O.pack(q1, bits))
    assert np.array_equal(ql.codes2.cpu().numpy(), O.pack(q2, bits))
    xd = dev(x)
    saved = moqe.moqe_set_launch_mode(launch_mode) if launch_mode is not None else None
    try:
        ws = moqe.alloc_workspace(moqe.moqe_layer_workspace_bytes(wl.T, wl.E, wl.d, wl.f), xd.device)
        y, r = moqe.moqe_moe_layer(ql, xd, residual=xd if residual else None, workspace=ws)
        torch.cuda.synchronize()
        assert not moqe.workspace_error(ws)
        r2 = moqe.moqe_route(xd, ql.w_gate)
        y2 = moqe.moqe_expert_ffn(ql, xd, r2, residual=xd if residual else None)
    finally:
        if saved is not None:
            moqe.moqe_set_launch_mode(saved)
    idx, gate, offs, perm = route_to_numpy(r)
    assert_route_equal((idx, gate, offs, perm), O.route(x, layer["w_gate"]), wl.T, wl.E)
    assert np.array_equal(y.cpu().numpy().view(np.uint16), y2.cpu().numpy().view(np.uint16))
    yh = y.cpu().numpy()
    if sample is not None:  # a seeded sample of the rows plus every segment's first and last
        rows = np.random.default_rng(wl.seed).choice(wl.T, size=sample, replace=False)
        has = np.diff(offs) > 0
        rows = np.concatenate([rows, perm[offs[:-1][has]], perm[offs[1:][has] - 1]])
        x, idx, gate, yh = x[rows], idx[rows], gate[rows], yh[rows]
    ref = O.expert_ffn(x, idx, gate.astype(np.float64), O.dequantize_log(q1, s1, bits), layer["b1"],
                       O.dequantize_log(q2, s2, bits), layer["b2"], residual=x if residual else None)
    err = ffn_error(yh, ref)
    assert err <= FFN_TOL, f"{wl.name} log{bits}: max|err|/max|ref| = {err:.3e}"


@pytest.mark.parametrize("bits", (4, 3, 2))
@pytest.mark.parametrize("T", (1, 24, 37, 150))
def test_log_scale_layer_small(bits, T):
    _log_layer_parity(W.small(T=T, seed=91 + T), bits)


@pytest.mark.parametrize("bits", (4, 3, 2))
def test_log_scale_layer_shapes_and_modes(bits):
    _log_layer_parity(W.small(E=4, d=512, f=2048, T=40, seed=95), bits, residual=True)
    _log_layer_parity(W.small(E=3, d=768, f=3072, T=21, seed=96), bits)
    _log_layer_parity(W.small(E=8, d=512, f=2048, T=24, seed=97), bits, launch_mode=moqe.LAUNCH_FUSED)
    # many tokens per expert: the tiled kernel (all three tile shapes over the two calls), then a
    # Zipf load where the decode kernel takes the small segments beside it
    _log_layer_parity(W.small(E=4, d=256, f=512, T=700, seed=98), bits)
    _log_layer_parity(W.small(E=4, d=256, f=4096, T=8192, seed=99), bits, sample=256)
    _log_layer_parity(W.small(E=16, d=256, f=512, T=200, routing="zipf", n_empty=3, seed=85), bits, residual=True)


@pytest.mark.parametrize("bits", (4, 3, 2))
def test_log_scale_layer_benchmark_shape(bits):
    _log_layer_parity(W.CONFIGS["c1"], bits)


@pytest.mark.parametrize("bits", (4, 3, 2))
def test_decode_kernels_agree(bits):
    """The kernel built for batches of at most 64 tokens and the general decode kernel run the same
    arithmetic in the same order (same unpack, same K order, same K-split sums): FFN1's output is
    identical bit for bit, and the layer output differs at most by how gate x output is rounded to
    fp16 (one unit in the last place, in a few outputs of ten thousand), as the header says for
    moqe_set_decode_kernel.  C1 at full size, shapes with other slice lengths and K splits, a
    residual, 128 experts, and log-scale codes."""
    cases = [(W.CONFIGS["c1"], False, moqe.CODEC_LINEAR), (W.small(E=4, d=512, f=2048, T=40, seed=21), True, moqe.CODEC_LINEAR),
             (W.small(E=3, d=768, f=3072, T=21, seed=22), False, moqe.CODEC_LINEAR),
             (W.small(E=128, d=256, f=512, T=64, seed=23), True, moqe.CODEC_LINEAR),
             (W.small(E=8, d=128, f=256, T=37, seed=24), False, moqe.CODEC_LOG),
             (W.small(E=8, d=1024, f=4096, T=64, routing="zipf", n_empty=2, seed=25), True, moqe.CODEC_LINEAR),
             (W.small(E=2, d=1024, f=1024, T=23, seed=26), True, moqe.CODEC_LOG),
             # more than 64 experts (the tables' second half) with slices of 32 steps: pairs of 8 rows apply
             (W.small(E=72, d=1024, f=1024, T=64, seed=27), False, moqe.CODEC_LINEAR)]
    for wl, residual, codec in cases:
        layer, x = W.make_layer(wl), W.make_tokens(wl)
        ql = moqe.quantize_layer(dev(layer["w1"]), dev(layer["b1"]), dev(layer["w2"]), dev(layer["b2"]), bits,
                                 dev(layer["w_gate"]), codec=codec)
        xd = dev(x)
        r = moqe.moqe_route(xd, ql.w_gate)
        h_small = torch.zeros((wl.T, wl.f), dtype=torch.float16, device="cuda")
        h_general = torch.zeros_like(h_small)
        old = moqe.moqe_set_decode_kernel(moqe.DECODE_AUTO)
        try:
            moqe.moqe_expert_ffn1(ql, xd, r, h_small)
            y_small = moqe.moqe_expert_ffn(ql, xd, r, residual=xd if residual else None)
            moqe.moqe_set_decode_kernel(moqe.DECODE_GENERAL)
            moqe.moqe_expert_ffn1(ql, xd, r, h_general)
            y_general = moqe.moqe_expert_ffn(ql, xd, r, residual=xd if residual else None)
            # pairs of 8 token rows instead of 4: the same sums per token, so the same bits
            moqe.moqe_set_decode_kernel(moqe.DECODE_ROWS8)
            h_rows8 = torch.zeros_like(h_small)
            moqe.moqe_expert_ffn1(ql, xd, r, h_rows8)
            y_rows8 = moqe.moqe_expert_ffn(ql, xd, r, residual=xd if residual else None)
        finally:
            moqe.moqe_set_decode_kernel(old)
        torch.cuda.synchronize()
        assert torch.equal(h_small.view(torch.int16), h_general.view(torch.int16)), wl.name
        assert torch.equal(h_small.view(torch.int16), h_rows8.view(torch.int16)), wl.name
        assert torch.equal(y_small.view(torch.int16), y_rows8.view(torch.int16)), wl.name
        a, b = y_small.cpu().numpy(), y_general.cpu().numpy()
        differ = a.view(np.uint16) != b.view(np.uint16)
        assert differ.mean() <= 2e-3, f"{wl.name}: {differ.sum()} outputs differ"
        # neighbours in fp16: the bit patterns of two finite halves of one sign differ by one
        assert np.all(np.abs(a.view(np.int16).astype(np.int32)[differ] - b.view(np.int16).astype(np.int32)[differ]) == 1), wl.name


@pytest.mark.parametrize("bits", (4, 3, 2))
def test_decode_sized_kernel_from_65_to_128_tokens(bits):
    """Batches of 65 to 128 tokens stay with the decode-sized kernel where its pairs of 8 rows
    apply (K = 1024 or 4096): the routing tables then take two registers per lane.  Same
    arithmetic as the general decode kernel (FFN1 bit for bit, the layer output up to the last
    rounding), and the oracle's result: the first size, the last, a skewed load, more than 64
    experts, and one expert with every token but one (16 pairs, tokens from both halves of the
    tables in one pair's rows)."""
    cases = [(W.small(E=8, d=1024, f=4096, T=65, seed=31), False, False),
             (W.small(E=8, d=1024, f=4096, T=128, seed=32), True, False),
             (W.small(E=8, d=1024, f=4096, T=100, routing="zipf", n_empty=2, seed=33), True, False),
             (W.small(E=72, d=1024, f=1024, T=128, seed=34), False, False),
             (W.small(E=4, d=1024, f=1024, T=127, seed=35), True, True)]
    for wl, residual, one_expert in cases:
        layer, x = W.make_layer(wl), W.make_tokens(wl)
        ql = gpu_quantize_layer(layer, bits)
        xd = dev(x)
        if one_expert:
            idx = np.full(wl.T, 2, np.int32)
            idx[-1] = 0
            r = make_route(idx, np.random.default_rng(5).uniform(0.2, 1.0, wl.T).astype(np.float32), wl.E)
        else:
            r = moqe.moqe_route(xd, ql.w_gate)
        outs = {}
        old = moqe.moqe_set_decode_kernel(moqe.DECODE_AUTO)
        moqe.moqe_set_prefill_policy(moqe.PREFILL_NEVER, moqe.PREFILL_NEVER, moqe.PREFILL_NEVER)  # no tiled kernel
        try:
            for name, which, want in (("small", moqe.DECODE_AUTO, moqe.PATH_DECODE_SMALL),
                                      ("general", moqe.DECODE_GENERAL, moqe.PATH_DECODE)):
                moqe.moqe_set_decode_kernel(which)
                assert moqe.moqe_contraction_path(bits, wl.T, wl.E, wl.d, wl.f) == want
                assert moqe.moqe_contraction_path(bits, wl.T, wl.E, wl.f, wl.d) == want
                h = torch.zeros((wl.T, wl.f), dtype=torch.float16, device="cuda")
                moqe.moqe_expert_ffn1(ql, xd, r, h)
                outs[name] = (h, moqe.moqe_expert_ffn(ql, xd, r, residual=xd if residual else None))
        finally:
            moqe.moqe_set_decode_kernel(old)
            moqe.moqe_set_prefill_policy()
        torch.cuda.synchronize()
        assert torch.equal(outs["small"][0].view(torch.int16), outs["general"][0].view(torch.int16)), wl.name
        a, b = outs["small"][1].cpu().numpy(), outs["general"][1].cpu().numpy()
        differ = a.view(np.uint16) != b.view(np.uint16)
        assert differ.mean() <= 2e-3, f"{wl.name}: {differ.sum()} outputs differ"
        assert np.all(np.abs(a.view(np.int16).astype(np.int32)[differ] - b.view(np.int16).astype(np.int32)[differ]) == 1), wl.name
        if wl.E <= 8:
            idx, gate = r.expert_idx.cpu().numpy(), r.gate.cpu().numpy().astype(np.float64)
            ref = oracle_layer_output(x, layer, bits, idx, gate, residual=residual)
            assert ffn_error(a, ref) <= FFN_TOL, wl.name


def test_stream_read_leaves_its_input_alone():
    """The plain read that bench.py times as the ceiling: runs, writes nothing but (at most) its
    sink word, rejects sizes that are not whole KiB."""
    src = torch.arange(0, 3 << 20, dtype=torch.int32, device="cuda")
    keep = src.clone()
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    L = moqe.lib()
    for nbytes in (1024, 37 * 1024, src.numel() * 4):
        assert L.moqe_stream_read(src.data_ptr(), nbytes, sink.data_ptr(), torch.cuda.current_stream().cuda_stream) == 0
    torch.cuda.synchronize()
    assert torch.equal(src, keep)
    assert L.moqe_stream_read(src.data_ptr(), 1000, sink.data_ptr(), None) == 3
