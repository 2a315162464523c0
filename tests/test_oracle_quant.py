"""Pins for the oracle's quantizer (paper App. A linear quantization, App. C fp16
scales): hand-worked examples, invariants the formula fixes, brute force."""

import os

import numpy as np
import pytest

from oracle import brute
from oracle import moqe_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "quant_hand_examples.txt")
BITS = (2, 3, 4, 8)


def _rows():
    rows = []
    with open(GOLDEN) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            b, col, s, q, dq = [p.strip() for p in line.split("|")]
            rows.append((int(b), [float(v) for v in col.split()], float(s),
                         [int(v) for v in q.split()], [float(v) for v in dq.split()]))
    return rows


@pytest.mark.parametrize("row", _rows())
def test_hand_examples(row):
    bits, col, s, q, dq = row
    w = np.array(col, dtype=np.float64)[:, None]
    qq, ss = O.quantize(w, bits)
    assert float(ss[0]) == s
    assert qq[:, 0].tolist() == q
    assert O.dequantize(qq, ss)[:, 0].tolist() == dq
    # the scalar brute force agrees on the same example
    bq, bs, _ = brute.quantize_column(col, bits)
    assert bq == q and bs == s


def _rand(shape, seed, outliers=True):
    rng = np.random.default_rng(seed)
    w = (rng.standard_normal(shape) * 0.02).astype(np.float32)
    if outliers:
        mask = rng.random(shape) < 0.01
        w[mask] = np.float32(0.16) * rng.choice([-1.0, 1.0], size=int(mask.sum())).astype(np.float32)
    return w


@pytest.mark.parametrize("bits", BITS)
def test_range_and_half_step_bound(bits):
    w = _rand((3, 96, 48), 5)
    q, s = O.quantize(w, bits)
    lo, hi = O.code_range(bits)
    assert q.min() >= lo and q.max() <= hi
    sd = s.astype(np.float64)[:, None, :]
    err = np.abs(w.astype(np.float64) - O.dequantize(q, s))
    assert np.all(err <= 0.5 * sd * (1 + 2.0 ** -50))
    # bound is attained at a positive channel maximum when the fp16 scale is exact
    col = np.array([[3.0], [1.0], [-2.0]])
    qq, ss = O.quantize(col, 2)
    assert abs(3.0 - float(qq[0, 0]) * float(ss[0])) == 0.5 * float(ss[0])


@pytest.mark.parametrize("bits", BITS)
def test_scale_is_smallest_fp16_not_below_formula(bits):
    w = _rand((2, 64, 32), 6)
    _, s = O.quantize(w, bits)
    m = np.abs(w.astype(np.float64)).max(axis=1)
    s64 = 2 * m / (2 ** bits - 1)
    sd = s.astype(np.float64)
    assert np.all(sd >= s64)
    below = np.nextafter(s, np.float16(-np.inf)).astype(np.float64)
    assert np.all(below < s64)


@pytest.mark.parametrize("bits", BITS)
def test_channel_maximum_gets_an_extreme_code(bits):
    w = _rand((2, 64, 32), 7)
    q, s = O.quantize(w, bits)
    lo, hi = O.code_range(bits)
    for e in range(w.shape[0]):
        k = np.argmax(np.abs(w[e]), axis=0)
        n = np.arange(w.shape[2])
        top = w[e][k, n]
        code = q[e][k, n]
        m = np.abs(top).astype(np.float64)
        exact = s[e].astype(np.float64) == 2 * m / (2 ** bits - 1)
        assert np.all(code[top > 0] == hi)
        neg = top < 0
        assert np.all(code[neg & exact] == lo)
        assert np.all(code[neg & ~exact] == -hi)


@pytest.mark.parametrize("bits", BITS)
def test_power_of_two_scaling(bits):
    w = _rand((1, 64, 32), 8)
    q0, s0 = O.quantize(w, bits)
    # (int8 scales are 17 times smaller than int4's: 2^-3 would push them into fp16's
    # subnormal range, where the stored scale has fewer bits and the codes may change)
    for j in ((-3, 2, 5) if bits < 8 else (-1, 2, 5)):
        q1, s1 = O.quantize(w * np.float32(2.0 ** j), bits)
        assert np.array_equal(q0, q1)
        assert np.array_equal(s1.astype(np.float64), s0.astype(np.float64) * 2.0 ** j)


@pytest.mark.parametrize("bits", BITS)
def test_channel_independence(bits):
    w = _rand((1, 64, 32), 9)
    q0, s0 = O.quantize(w, bits)
    w2 = w.copy()
    w2[0, :, 5] *= np.float32(3.7)
    w2[0, 3, 5] = np.float32(1.0)
    q1, s1 = O.quantize(w2, bits)
    keep = np.arange(32) != 5
    assert np.array_equal(q0[..., keep], q1[..., keep])
    assert np.array_equal(s0[..., keep], s1[..., keep])
    assert not np.array_equal(s0[..., 5], s1[..., 5])


@pytest.mark.parametrize("bits", BITS)
def test_zero_channel(bits):
    w = _rand((1, 32, 16), 10)
    w[0, :, 3] = 0
    q, s = O.quantize(w, bits)
    assert s[0, 3] == 0 and np.all(q[0, :, 3] == 0)
    assert np.all(O.dequantize(q, s)[0, :, 3] == 0)


def test_tiny_scale_becomes_smallest_subnormal():
    w = np.full((4, 1), 1e-9)
    q, s = O.quantize(w, 4)
    assert float(s[0]) == 2.0 ** -24
    assert np.all(q == 0)


def test_rejects_nonfinite_and_overflow():
    with pytest.raises(ValueError):
        O.quantize(np.array([[np.inf], [1.0]]), 4)
    with pytest.raises(ValueError):
        O.quantize(np.array([[1e6], [1.0]]), 2)


@pytest.mark.parametrize("bits", BITS)
def test_matches_scalar_brute_force(bits):
    w = _rand((1, 24, 5), 12)[0]
    # plant exact ties: a/s = +-k.5 with an exactly representable scale
    w[:, 0] = 0
    w[0, 0] = 7.5 if bits == 4 else (3.5 if bits == 3 else 1.5)
    w[1, 0] = 2.5 * (2 * w[0, 0] / (2 ** bits - 1))
    w[2, 0] = -1.5 * (2 * w[0, 0] / (2 ** bits - 1))
    q, s = O.quantize(w, bits)
    bq, bs = brute.quantize_matrix(w.astype(np.float64).tolist(), bits)
    assert q.tolist() == bq
    assert s.astype(np.float64).tolist() == bs


def test_fp16_path_is_plain_cast():
    w = _rand((1, 8, 4), 13)
    assert np.array_equal(O.quantize_fp16(w), w.astype(np.float16).astype(np.float64))


def test_more_bits_is_closer():
    w = _rand((1, 256, 64), 14, outliers=False)
    errs = [np.abs(O.dequantize(*O.quantize(w, b)) - w).mean() for b in (2, 3, 4)]
    assert errs[0] > errs[1] > errs[2]


@pytest.mark.parametrize("bits", BITS)
def test_tensor_wise_scale(bits):
    """App. A's other choice of s ("per the whole tensor"): one scale from the matrix maximum.
    Hand example: columns with maxima 3 and 1.5 share s = 2*3/(2^b - 1); invariants as for the
    channel-wise scale; a matrix of one column is the same either way; channel-wise scales never
    exceed the tensor's."""
    w = np.array([[3.0, 1.5], [-1.0, -1.5], [0.4, 0.0]])
    q, s = O.quantize(w, bits, scale_per="tensor")
    expect = float(O.fp16_round_up(np.array(6.0 / (2 ** bits - 1))))
    assert s.tolist() == [expect, expect]
    assert q[0, 0] == 2 ** (bits - 1) - 1                      # the maximum takes the top code
    assert q[0, 1] == int(np.clip(np.rint(1.5 / expect), -(2 ** (bits - 1)), 2 ** (bits - 1) - 1))
    w = _rand((2, 64, 32), 9)
    q, s = O.quantize(w, bits, scale_per="tensor")
    lo, hi = O.code_range(bits)
    assert q.min() >= lo and q.max() <= hi
    assert np.all(s == s[:, :1])                                # one value per matrix
    err = np.abs(w.astype(np.float64) - O.dequantize(q, s))
    assert np.all(err <= 0.5 * s.astype(np.float64)[:, None, :] * (1 + 2.0 ** -50))
    qc, sc = O.quantize(w, bits)
    assert np.all(sc.astype(np.float64) <= s.astype(np.float64))
    assert np.array_equal(s[:, 0].astype(np.float64), sc.astype(np.float64).max(axis=1))
    q1, s1 = O.quantize(w[:, :, :1], bits, scale_per="tensor")
    q2, s2 = O.quantize(w[:, :, :1], bits)
    assert np.array_equal(q1, q2) and np.array_equal(s1, s2)
    with pytest.raises(ValueError):
        O.quantize(w, bits, scale_per="row")
