"""Pins for the oracle's top-1 gating and dispatch (App. B "MoE architecture")."""

import numpy as np
import pytest
import scipy.special

from oracle import brute
from oracle import moqe_oracle as O


def _case(T, d, E, seed):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, d)).astype(np.float16)
    wg = (rng.standard_normal((d, E)) * 0.1).astype(np.float16)
    return x, wg


@pytest.mark.parametrize("T,d,E", ((37, 32, 8), (5, 16, 4), (200, 64, 32)))
def test_structure(T, d, E):
    x, wg = _case(T, d, E, T)
    idx, gate, offs, perm = O.route(x, wg)
    assert offs[0] == 0 and offs[-1] == T and np.all(np.diff(offs) >= 0)
    assert np.array_equal(np.diff(offs), np.bincount(idx, minlength=E))
    assert sorted(perm.tolist()) == list(range(T))
    assert np.all(np.diff(idx[perm]) >= 0)
    for e in range(E):
        seg = perm[offs[e]:offs[e + 1]]
        assert np.all(idx[seg] == e) and np.all(np.diff(seg) > 0)
    assert np.all(gate >= 1.0 / E - 1e-15) and np.all(gate <= 1.0)


def test_gate_is_library_softmax_at_argmax():
    x, wg = _case(50, 48, 16, 3)
    l = O.route_logits(x, wg)
    idx, gate, _, _ = O.route_from_logits(l)
    p = scipy.special.softmax(l, axis=1)
    assert np.array_equal(idx, p.argmax(axis=1))
    assert np.allclose(gate, p[np.arange(50), idx], rtol=1e-13, atol=0)


def test_zero_gate_weights_closed_form():
    x, _ = _case(9, 16, 8, 4)
    idx, gate, offs, perm = O.route(x, np.zeros((16, 8), np.float16))
    assert np.all(idx == 0) and np.all(gate == 1.0 / 8)
    assert offs.tolist() == [0] + [9] * 8 and perm.tolist() == list(range(9))


def test_duplicate_columns_lowest_index_wins():
    x, wg = _case(40, 16, 6, 5)
    wg[:, 4] = wg[:, 1]
    idx, _, _, _ = O.route(x, wg)
    assert not np.any(idx == 4) and np.any(idx == 1)


def test_token_permutation_equivariance():
    x, wg = _case(30, 16, 8, 6)
    idx, gate, _, _ = O.route(x, wg)
    p = np.random.default_rng(0).permutation(30)
    idx2, gate2, _, _ = O.route(x[p], wg)
    assert np.array_equal(idx2, idx[p]) and np.array_equal(gate2, gate[p])


def test_logits_against_scalar_sum_and_brute_route():
    x, wg = _case(6, 12, 5, 7)
    xl, wl = x.astype(np.float64).tolist(), wg.astype(np.float64).tolist()
    bidx, bgate, boffs, bperm = brute.route(xl, wl)
    idx, gate, offs, perm = O.route(x, wg)
    assert idx.tolist() == bidx and offs.tolist() == boffs and perm.tolist() == bperm
    assert np.allclose(gate, bgate, rtol=1e-13, atol=0)


def test_empty_batch():
    idx, gate, offs, perm = O.route_from_logits(np.zeros((0, 4)))
    assert idx.size == 0 and gate.size == 0 and perm.size == 0 and offs.tolist() == [0] * 5


def test_margin_helper():
    l = np.array([[0.0, 3.0, 1.0], [2.0, 2.0, -1.0]])
    assert O.top2_margin(l).tolist() == [2.0, 0.0]


def test_non_finite_rows_stay_in_range():
    """Outside the method's domain, pinned so that no token can fall out of the dispatch: a NaN
    counts as the row maximum (the first one wins), a row of -inf takes expert 0."""
    inf = np.inf
    l = np.array([[0.5, np.nan, 2.0, np.nan],      # first NaN
                  [-inf, -inf, -inf, -inf],        # nothing above -inf
                  [np.nan, np.nan, np.nan, np.nan],
                  [-inf, 1.0, inf, inf],           # +inf is an ordinary maximum, lowest index
                  [3.0, 1.0, 3.0, -2.0]])          # finite row, exact tie
    idx, gate, offs, perm = O.route_from_logits(l)
    assert idx.tolist() == [1, 0, 0, 2, 0]
    assert offs.tolist() == [0, 3, 4, 5, 5] and perm.tolist() == [1, 2, 4, 0, 3]
    assert np.isnan(gate[:4]).all() and np.isclose(gate[4], 1.0 / (2.0 + np.exp(-2.0) + np.exp(-5.0)))
    # by hand, independent of argmax: scan each row for the first entry no other entry ranks above
    def first_max(row):
        rank = lambda v: (2, 0.0) if np.isnan(v) else (1, v)
        best = max(rank(v) for v in row)
        return next(i for i, v in enumerate(row) if rank(v) == best)
    assert [first_max(r) for r in l] == idx.tolist()
