"""A seeded sweep of whole layer steps over random combinations of what the other GPU tests
vary one at a time: layer shape, token count, load shape, weight width and codec, residual,
launch mode and path-choice thresholds.  Every case: routing tables bit-exact against the
oracle, the FFN output within the bound, and a second call bit-identical to the first."""

import numpy as np
import pytest
import torch

from oracle import moqe_oracle as O
from paper_2310_02410_amd import moqe, workloads as W
from tests.helpers import FFN_TOL, assert_route_equal, dev, ffn_error, route_to_numpy

pytestmark = pytest.mark.gpu

DIMS = (64, 128, 256, 384, 512, 768, 1024, 1536, 2048)
POLICIES = ((5, 65, 16), (1, 1, moqe.PREFILL_NEVER), (5, 1, moqe.PREFILL_NEVER), (1 << 20, 1, moqe.PREFILL_NEVER),
            (3, 20, 4))


def _cases(seed, n):
    rng = np.random.default_rng(seed)
    L = moqe.lib()
    out = []
    while len(out) < n:
        bits = int(rng.choice([2, 3, 4, 8, 16]))
        codec = int(rng.random() < 0.35) if bits in (2, 3, 4) else 0
        E = int(rng.choice([1, 2, 3, 5, 8, 16, 32, 40, 64]))
        d, f = int(rng.choice(DIMS)), int(rng.choice(DIMS))
        T = int(rng.choice([1, 2, 3, 7, 24, 33, 64, 65, 100, 257, 700, 1500]))
        zipf = bool(E >= 8 and rng.random() < 0.3)
        residual = bool(rng.random() < 0.4)
        mode = int(rng.choice([moqe.LAUNCH_AUTO, moqe.LAUNCH_SEPARATE, moqe.LAUNCH_FUSED]))
        policy = POLICIES[int(rng.integers(len(POLICIES)))]
        wseed = int(rng.integers(1 << 20))
        if L.moqe_check_layer(bits, E, d, f) != 0 or E * d * f > 1e8:
            continue
        out.append((bits, codec, E, d, f, T, zipf, residual, mode, policy, wseed))
    return out


def _weights(layer, bits, codec):
    if bits == 16:
        return O.quantize_fp16(layer["w1"]), O.quantize_fp16(layer["w2"])
    if codec:
        (q1, s1), (q2, s2) = O.quantize_log(layer["w1"], bits), O.quantize_log(layer["w2"], bits)
        return O.dequantize_log(q1, s1, bits), O.dequantize_log(q2, s2, bits)
    (q1, s1), (q2, s2) = O.quantize(layer["w1"], bits), O.quantize(layer["w2"], bits)
    return O.dequantize(q1, s1), O.dequantize(q2, s2)


@pytest.mark.parametrize("chunk", range(4))
def test_random_layer_steps(chunk):
    for case in _cases(1000 + chunk, 12):
        bits, codec, E, d, f, T, zipf, residual, mode, policy, wseed = case
        wl = W.small(E=E, d=d, f=f, T=T, seed=wseed, routing="zipf" if zipf else "uniform", n_empty=2 if zipf else 0)
        layer, x = W.make_layer(wl), W.make_tokens(wl)
        ql = moqe.quantize_layer(dev(layer["w1"]), dev(layer["b1"]), dev(layer["w2"]), dev(layer["b2"]), bits,
                                 dev(layer["w_gate"]), codec=codec)
        xd = dev(x)
        saved = moqe.moqe_set_launch_mode(mode)
        moqe.moqe_set_prefill_policy(*policy)
        try:
            ws = moqe.alloc_workspace(moqe.moqe_layer_workspace_bytes(T, E, d, f), xd.device)
            y, r = moqe.moqe_moe_layer(ql, xd, residual=xd if residual else None, workspace=ws)
            y2, _ = moqe.moqe_moe_layer(ql, xd, residual=xd if residual else None, workspace=ws)
            torch.cuda.synchronize()
            assert not moqe.workspace_error(ws), case
        finally:
            moqe.moqe_set_launch_mode(saved)
            moqe.moqe_set_prefill_policy()
        got = route_to_numpy(r)
        assert_route_equal(got, O.route(x, layer["w_gate"]), T, E)
        w1, w2 = _weights(layer, bits, codec)
        ref = O.expert_ffn(x, got[0], got[1].astype(np.float64), w1, layer["b1"], w2, layer["b2"],
                           residual=x if residual else None)
        err = ffn_error(y.cpu().numpy(), ref)
        assert err <= FFN_TOL, (case, err)
        assert np.array_equal(y.cpu().numpy().view(np.uint16), y2.cpu().numpy().view(np.uint16)), case


MID_DIMS = (512, 768, 1024, 1536, 2048, 3072, 4096)
MID_POLICIES = ((moqe.PREFILL_MIN_SEGMENT_DEFAULT, moqe.PREFILL_MIN_BATCH_DEFAULT, moqe.PREFILL_ALL_TILED_DEFAULT),
                (1, 1, moqe.PREFILL_NEVER), (5, 65, moqe.PREFILL_NEVER),
                (moqe.PREFILL_NEVER, moqe.PREFILL_NEVER, moqe.PREFILL_NEVER))


def _mid_cases(seed, n):
    """Mid-sized batches on layers with long K: the sizes where the decode-sized kernel works with
    routing tables of two registers, the resident tiled kernel with pairs of 16 tokens, and the
    path choice changes hands; under the library's default thresholds and three others, and
    under each setting of the tiled kernel."""
    rng = np.random.default_rng(seed)
    L = moqe.lib()
    out = []
    while len(out) < n:
        bits = int(rng.choice([2, 3, 4]))
        codec = int(rng.random() < 0.3)
        E = int(rng.choice([2, 4, 8, 16, 24]))
        d, f = int(rng.choice(MID_DIMS)), int(rng.choice(MID_DIMS))
        T = int(rng.choice([65, 100, 127, 128, 129, 160, 200, 256, 300, 400]))
        zipf = bool(E >= 8 and rng.random() < 0.3)
        residual = bool(rng.random() < 0.4)
        tiled = int(rng.choice([moqe.TILED_AUTO, moqe.TILED_STREAMED, moqe.TILED_RESIDENT]))
        policy = MID_POLICIES[int(rng.integers(len(MID_POLICIES)))]
        wseed = int(rng.integers(1 << 20))
        if L.moqe_check_layer(bits, E, d, f) != 0 or E * d * f > 1e8:
            continue
        out.append((bits, codec, E, d, f, T, zipf, residual, tiled, policy, wseed))
    return out


def run_mid_case(case):
    bits, codec, E, d, f, T, zipf, residual, tiled, policy, wseed = case
    wl = W.small(E=E, d=d, f=f, T=T, seed=wseed, routing="zipf" if zipf else "uniform", n_empty=2 if zipf else 0)
    layer, x = W.make_layer(wl), W.make_tokens(wl)
    ql = moqe.quantize_layer(dev(layer["w1"]), dev(layer["b1"]), dev(layer["w2"]), dev(layer["b2"]), bits,
                             dev(layer["w_gate"]), codec=codec)
    xd = dev(x)
    moqe.moqe_set_tiled_kernel(tiled)
    moqe.moqe_set_prefill_policy(*policy)
    try:
        ws = moqe.alloc_workspace(moqe.moqe_layer_workspace_bytes(T, E, d, f), xd.device)
        y, r = moqe.moqe_moe_layer(ql, xd, residual=xd if residual else None, workspace=ws)
        y2, _ = moqe.moqe_moe_layer(ql, xd, residual=xd if residual else None, workspace=ws)
        torch.cuda.synchronize()
        assert not moqe.workspace_error(ws), case
    finally:
        moqe.moqe_set_tiled_kernel(moqe.TILED_AUTO)
        moqe.moqe_set_prefill_policy()
    got = route_to_numpy(r)
    assert_route_equal(got, O.route(x, layer["w_gate"]), T, E)
    w1, w2 = _weights(layer, bits, codec)
    ref = O.expert_ffn(x, got[0], got[1].astype(np.float64), w1, layer["b1"], w2, layer["b2"],
                       residual=x if residual else None)
    err = ffn_error(y.cpu().numpy(), ref)
    assert err <= FFN_TOL, (case, err)
    assert np.array_equal(y.cpu().numpy().view(np.uint16), y2.cpu().numpy().view(np.uint16)), case
    return err


@pytest.mark.parametrize("chunk", range(2))
def test_random_mid_sized_steps(chunk):
    for case in _mid_cases(3000 + chunk, 12):
        run_mid_case(case)


def test_random_router_shapes():
    """moqe_route and moqe_route_logits over 40 seeded random (E, d, T), expert counts that no
    kernel is specialised for and token counts on both sides of every kernel's limit among them;
    the given logits are small integers, so exact ties are everywhere."""
    rng = np.random.default_rng(2000)
    done = 0
    while done < 40:
        E = int(rng.choice([1, 2, 3, 4, 7, 8, 13, 16, 24, 32, 33, 64, 100, 128, 129, 200, 256, 300, 511, 1024]))
        d = int(rng.choice([8, 16, 24, 32, 64, 96, 128, 256, 264, 512, 768, 1024, 2048]))
        T = int(rng.choice([1, 2, 15, 16, 17, 24, 32, 33, 63, 64, 65, 128, 255, 256, 257, 1000, 1536, 4096, 5000, 20000]))
        zipf = bool(E >= 8 and rng.random() < 0.3)
        wseed = int(rng.integers(1 << 20))
        if T * d > 2e7 or E * d > 2e5:
            continue
        done += 1
        wl = W.small(E=E, d=d, f=32, T=T, seed=wseed, routing="zipf" if zipf else "uniform",
                     n_empty=min(2, E - 1) if zipf else 0)
        layer, x = W.make_layer(wl), W.make_tokens(wl)
        r = moqe.moqe_route(dev(x), dev(layer["w_gate"]))
        assert_route_equal(route_to_numpy(r), O.route(x, layer["w_gate"]), T, E)
        logits = rng.integers(-3, 4, size=(T, E)).astype(np.float32)
        r2 = moqe.moqe_route_logits(dev(logits))
        assert_route_equal(route_to_numpy(r2), O.route_from_logits(logits), T, E)
