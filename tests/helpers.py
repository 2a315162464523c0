"""Shared plumbing of the GPU parity tests: move a generated layer to the device,
run the HIP path through the C ABI, run the oracle, compare."""

import numpy as np
import torch

from oracle import moqe_oracle as O
from paper_2310_02410_amd import moqe

FFN_TOL = 2e-3   # max|err| <= FFN_TOL * max|ref| on FFN outputs
GATE_RTOL = 2e-6  # fp32 softmax against the fp64 oracle


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t if dtype is None else t.to(dtype)


def gpu_quantize_layer(layer, bits):
    return moqe.quantize_layer(dev(layer["w1"]), dev(layer["b1"]), dev(layer["w2"]), dev(layer["b2"]), bits,
                               dev(layer["w_gate"]))


def route_to_numpy(r):
    return (r.expert_idx.cpu().numpy(), r.gate.cpu().numpy(), r.seg_offsets.cpu().numpy(), r.perm.cpu().numpy())


def make_route(idx, gate, E):
    """Device Route from a given assignment (numpy), dispatch built with numpy."""
    idx = np.asarray(idx, dtype=np.int32)
    counts = np.bincount(idx, minlength=E)
    offs = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    perm = np.argsort(idx, kind="stable").astype(np.int32)
    T = idx.size
    pad = lambda a: dev(np.concatenate([a, np.zeros(1, a.dtype)]))[:T]
    return moqe.Route(pad(idx), pad(np.asarray(gate, dtype=np.float32)), dev(offs), pad(perm))


def assert_route_equal(got, ref, T, E):
    gi, gg, go, gp = got
    ri, rg, ro, rp = ref
    assert np.array_equal(gi, ri), "expert_idx differs"
    assert np.array_equal(go, ro), "seg_offsets differ"
    assert np.array_equal(gp, rp), "perm differs"
    assert np.allclose(gg, rg, rtol=GATE_RTOL, atol=0), "gate differs"


def ffn_error(y_gpu, y_ref):
    y_gpu = y_gpu.astype(np.float64)
    scale = np.abs(y_ref).max()
    return np.abs(y_gpu - y_ref).max() / (scale if scale > 0 else 1.0)


def oracle_layer_output(x, layer, bits, idx, gate, residual=False, qlayer=None):
    ql = qlayer if qlayer is not None else O.quantize_layer(layer, bits)
    w1, w2 = O.layer_weights(ql)
    return O.expert_ffn(x, idx, gate, w1, layer["b1"], w2, layer["b2"], residual=x if residual else None)
