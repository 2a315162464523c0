"""GPU parity of moqe_route / moqe_route_logits against the oracle (App. B top-1
gating): expert indices, segment offsets and the permutation are bit-exact."""

import numpy as np
import pytest
import torch

from oracle import moqe_oracle as O
from paper_2310_02410_amd import moqe, workloads as W
from tests.helpers import assert_route_equal, dev, route_to_numpy

pytestmark = pytest.mark.gpu


def _route_case(wl):
    layer, x = W.make_layer(wl), W.make_tokens(wl)
    got = route_to_numpy(moqe.moqe_route(dev(x), dev(layer["w_gate"])))
    torch.cuda.synchronize()
    assert_route_equal(got, O.route(x, layer["w_gate"]), wl.T, wl.E)
    return got


@pytest.mark.parametrize("name", ("c0", "c1", "c3"))
def test_benchmark_configs(name):
    wl = W.CONFIGS[name]
    wl = W.small(name, E=wl.E, d=wl.d, f=32, T=wl.T, routing=wl.routing, n_empty=wl.n_empty, seed=wl.seed)
    got = _route_case(wl)
    if name == "c3":
        counts = np.diff(got[2])
        assert counts.max() > 300 and (counts == 0).sum() >= 4


@pytest.mark.parametrize("T,d,E", [(1, 64, 4), (37, 128, 8), (65, 64, 1), (130, 256, 128), (700, 64, 100),
                                   (4096, 1024, 32), (5000, 128, 8), (20000, 64, 256)])
def test_shapes(T, d, E):
    _route_case(W.small("r", E=E, d=d, f=32, T=T, seed=T + E))


@pytest.mark.parametrize("T,d,E", [(1, 512, 16), (24, 1024, 32), (64, 512, 32), (17, 1536, 32), (33, 1024, 16),
                                   (32, 1024, 64), (16, 1024, 128), (8, 512, 128), (5, 2048, 64),
                                   (16, 768, 128), (24, 96, 32), (3, 32, 16), (24, 768, 128), (32, 1024, 128),
                                   (17, 1024, 128), (33, 1024, 64), (64, 1024, 64)])
def test_single_launch_router_shapes(T, d, E):
    """Decode-sized batches take the one-workgroup MFMA router: up to 64 tokens, 32 with 128
    experts; (33, 1024, 128) does not fit it and takes the two-kernel path (covered below)."""
    _route_case(W.small("r1", E=E, d=d, f=32, T=T, seed=3 * T + E))


@pytest.mark.parametrize("T,d,E", [(65, 512, 16), (300, 1024, 64), (1000, 512, 128), (1536, 1024, 32),
                                   (129, 1536, 32), (4096, 768, 128), (81, 96, 16), (33, 1024, 128)])
def test_mfma_scoring_for_many_tokens(T, d, E):
    """More than 64 tokens with E in {16, 32, 64, 128} and d a multiple of 32: MFMA scoring by
    one workgroup per 16 tokens (ragged last tile), then the segment kernel."""
    _route_case(W.small("r3", E=E, d=d, f=32, T=T, seed=5 * T + E))


def test_single_launch_router_ties_and_skew():
    """Duplicate expert columns force exact ties (lowest index must win) on the one-launch path,
    Zipf routing fills some experts and leaves others empty."""
    wl = W.small("r2", E=32, d=1024, f=32, T=64, routing="zipf", n_empty=6, seed=77)
    layer, x = W.make_layer(wl), W.make_tokens(wl)
    wg = layer["w_gate"].copy()
    wg[:, 9] = wg[:, 3]
    wg[:, 30] = wg[:, 3]
    got = route_to_numpy(moqe.moqe_route(dev(x), dev(wg)))
    torch.cuda.synchronize()
    ref = O.route(x, wg)
    assert_route_equal(got, ref, wl.T, wl.E)
    assert not np.isin(got[0], (9, 30)).any()


def test_empty_batch():
    x = torch.empty((1, 64), dtype=torch.float16, device="cuda")[:0]
    wg = dev(W.make_layer(W.small("r", E=8, d=64, f=32))["w_gate"])
    r = moqe.moqe_route(x, wg)
    torch.cuda.synchronize()
    assert r.seg_offsets.cpu().tolist() == [0] * 9


def test_logits_with_exact_ties_and_forced_loads():
    rng = np.random.default_rng(5)
    T, E = 300, 32
    l = rng.integers(-4, 5, size=(T, E)).astype(np.float32) * 0.5   # many exact ties
    l[:40] = 0.0                                                     # all tied: expert 0, gate 1/E
    l[40:80, 7] = 9.0                                                # forced to expert 7
    got = route_to_numpy(moqe.moqe_route_logits(dev(l)))
    torch.cuda.synchronize()
    ref = O.route_from_logits(l)
    assert_route_equal(got, ref, T, E)
    assert np.all(got[0][:40] == 0) and np.allclose(got[1][:40], 1.0 / E, rtol=1e-6)
    assert np.all(got[0][40:80] == 7)


@pytest.mark.parametrize("T,E", [(24, 32), (200, 32), (24, 8), (5000, 100)])
def test_non_finite_logits_stay_in_the_dispatch(T, E):
    """Rows of -inf, rows of NaN, NaN or +inf among numbers: outside the method's domain, but no
    token may leave the dispatch (an index beyond E would send a kernel's row access astray).
    The oracle pins the convention: a NaN counts as the maximum, a row of -inf takes expert 0."""
    rng = np.random.default_rng(T + E)
    l = rng.standard_normal((T, E)).astype(np.float32)
    l[1] = -np.inf
    l[2] = np.nan
    l[3, E // 2] = np.nan
    l[4, [1, E - 1]] = np.inf
    l[T - 1] = -np.inf
    l[T - 2, E - 1] = np.nan
    got = route_to_numpy(moqe.moqe_route_logits(dev(l)))
    torch.cuda.synchronize()
    ri, rg, ro, rp = O.route_from_logits(l)
    assert np.array_equal(got[0], ri) and np.array_equal(got[2], ro) and np.array_equal(got[3], rp)
    assert got[0].min() >= 0 and got[0].max() < E
    assert np.allclose(got[1], rg, rtol=2e-6, atol=0, equal_nan=True)


def test_non_finite_activations_through_the_router():
    """A NaN or inf in x makes a whole row of logits non-finite on every scoring kernel: the
    index stays in range and the tables stay a partition of the tokens."""
    for T, d, E in ((24, 1024, 32), (200, 1024, 32), (24, 96, 24), (3000, 64, 10)):
        wl = W.small("nf", E=E, d=d, f=32, T=T, seed=T + d)
        x, wg = W.make_tokens(wl), W.make_layer(wl)["w_gate"]
        x[1, 5] = np.nan
        x[T - 1, 0] = np.inf
        x[T - 1, 1] = -np.inf
        idx, gate, offs, perm = route_to_numpy(moqe.moqe_route(dev(x), dev(wg)))
        torch.cuda.synchronize()
        assert idx.min() >= 0 and idx.max() < E and idx[1] == 0
        assert np.array_equal(np.diff(offs), np.bincount(idx, minlength=E)) and offs[-1] == T
        assert sorted(perm.tolist()) == list(range(T)) and np.array_equal(perm, np.argsort(idx, kind="stable"))
        keep = np.ones(T, bool)
        keep[[1, T - 1]] = False
        ri, rg, _, _ = O.route(x[keep], wg)
        assert np.array_equal(idx[keep], ri)


def test_deterministic():
    wl = W.small("r", E=32, d=1024, f=32, T=1536, routing="zipf", n_empty=4)
    layer, x = W.make_layer(wl), W.make_tokens(wl)
    xd, gd = dev(x), dev(layer["w_gate"])
    a = route_to_numpy(moqe.moqe_route(xd, gd))
    b = route_to_numpy(moqe.moqe_route(xd, gd))
    for u, v in zip(a, b):
        assert np.array_equal(u, v)
