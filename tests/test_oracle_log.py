"""Pins for the oracle's log-scale quantizer (paper App. A "Log-scale quantization"):
hand-worked examples, the printed formulas evaluated in exact rational arithmetic, the
logarithm taken literally where rounding cannot matter, and the invariants the format fixes."""

import os

import numpy as np
import pytest

from oracle import brute
from oracle import moqe_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "log_quant_hand_examples.txt")
BITS = O.LOG_BITS


def _rows():
    rows = []
    with open(GOLDEN) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            b, col, s, sg, ex, dq = [p.strip() for p in line.split("|")]
            rows.append((int(b), [float(v) for v in col.split()], float(s), [int(v) for v in sg.split()],
                         [int(v) for v in ex.split()], [float(v) for v in dq.split()]))
    return rows


@pytest.mark.parametrize("row", _rows())
def test_hand_examples(row):
    bits, col, s, signs, expos, dq = row
    q, ss = O.quantize_log(np.array(col)[:, None], bits)
    assert float(ss[0]) == s
    neg, ex = O.log_code_parts(q[:, 0], bits)
    assert neg.astype(int).tolist() == signs
    assert ex.tolist() == expos
    assert O.dequantize_log(q, ss, bits)[:, 0].tolist() == dq
    # the exact-rational evaluation of the printed formulas agrees on the same example
    bs, be, bscale = brute.log_quantize_column(col, bits)
    assert bs == signs and be == expos and bscale == s


def _rand(shape, seed):
    rng = np.random.default_rng(seed)
    w = (rng.standard_normal(shape) * 0.02).astype(np.float32)
    mask = rng.random(shape) < 0.01
    w[mask] = np.float32(0.16) * rng.choice([-1.0, 1.0], size=int(mask.sum())).astype(np.float32)
    return w


@pytest.mark.parametrize("bits", BITS)
def test_matches_exact_rational_brute_force(bits):
    w = _rand((1, 40, 6), 21)[0]
    w[3, 0] = 0.0
    w[4, 1] = -0.0
    w[:, 2] *= 1e-3                       # a channel of small numbers
    w[5, 3] = 0.75 * np.abs(w[:, 3]).max()  # near a break (the fp16 scale decides the side)
    q, s = O.quantize_log(w, bits)
    neg, ex = O.log_code_parts(q, bits)
    for n in range(w.shape[1]):
        bs, be, bscale = brute.log_quantize_column(w[:, n].astype(np.float64).tolist(), bits)
        assert float(s[n]) == bscale
        assert neg[:, n].astype(int).tolist() == bs
        assert ex[:, n].tolist() == be


@pytest.mark.parametrize("bits", BITS)
def test_matches_the_logarithm_away_from_the_breaks(bits):
    """Q = ceil(log2(2T/3)) computed with the library logarithm, wherever 2T/3 is not within
    rounding distance of a power of two (there the comparison form decides exactly)."""
    w = _rand((2, 256, 16), 22)
    q, s = O.quantize_log(w, bits)
    _, ex = O.log_code_parts(q, bits)
    lo, hi = O.log_exponent_range(bits)
    t = np.clip(np.abs(w.astype(np.float64)) / s.astype(np.float64)[:, None, :], 2.0 ** lo, 1.0)
    lg = np.log2(2.0 * t / 3.0)
    safe = np.abs(lg - np.rint(lg)) > 1e-9
    assert safe.mean() > 0.99
    assert np.array_equal(np.ceil(lg)[safe].astype(np.int64), ex[safe])
    assert ex.min() >= lo and ex.max() <= hi and ex.min() == lo and ex.max() == hi


@pytest.mark.parametrize("bits", BITS)
def test_format_invariants(bits):
    w = _rand((3, 96, 32), 23)
    q, s = O.quantize_log(w, bits)
    lo, hi = O.log_exponent_range(bits)
    assert q.min() >= -(1 << (bits - 1)) and q.max() <= (1 << (bits - 1)) - 1
    d = O.dequantize_log(q, s, bits)
    a = w.astype(np.float64)
    sd = s.astype(np.float64)[:, None, :]
    # magnitudes are s times a power of two in range; signs are kept
    ratio = np.abs(d) / sd
    assert np.array_equal(ratio, 2.0 ** np.round(np.log2(ratio)))
    assert ratio.min() >= 2.0 ** lo and ratio.max() <= 1.0
    assert np.all(np.sign(d)[a != 0] == np.sign(a)[a != 0])
    # the scale is the smallest fp16 number not below the channel maximum, whose code is exponent 0
    m = np.abs(a).max(axis=1)
    assert np.all(s.astype(np.float64) >= m)
    assert np.all(np.nextafter(s, np.float16(-np.inf)).astype(np.float64) < m)
    # inside the clip range the value is reproduced within a factor (2/3, 4/3]
    inside = np.abs(a) / sd >= 2.0 ** lo
    r = (np.abs(d) / np.where(inside, np.abs(a), 1.0))[inside]
    assert r.min() >= 2.0 / 3.0 and r.max() < 4.0 / 3.0 + 1e-12
    # below it everything becomes the smallest magnitude
    assert np.all(ratio[~inside] == 2.0 ** lo)
    # larger magnitude never gets a smaller exponent (per channel)
    _, ex = O.log_code_parts(q, bits)
    order = np.argsort(np.abs(a), axis=1, kind="stable")
    assert np.all(np.diff(np.take_along_axis(ex, order, axis=1), axis=1) >= 0)


@pytest.mark.parametrize("bits", BITS)
def test_quantizing_the_dequantized_values_changes_nothing(bits):
    """Every channel maximum decodes to s itself (its T lies in (0.75, 1]), so the dequantized
    matrix has the same scales, and every value s 2^Q has T = 2^Q, which encodes to Q again."""
    w = _rand((2, 64, 16), 24)
    q, s = O.quantize_log(w, bits)
    d = O.dequantize_log(q, s, bits)
    assert np.array_equal(np.abs(d).max(axis=1), s.astype(np.float64))
    q2, s2 = O.quantize_log(d, bits)
    assert np.array_equal(s, s2) and np.array_equal(q, q2)


@pytest.mark.parametrize("bits", BITS)
def test_power_of_two_scaling_and_channel_independence(bits):
    w = _rand((1, 64, 32), 25)
    q0, s0 = O.quantize_log(w, bits)
    for j in (-3, 4):
        q1, s1 = O.quantize_log(w * np.float32(2.0 ** j), bits)
        assert np.array_equal(q0, q1)
        assert np.array_equal(s1.astype(np.float64), s0.astype(np.float64) * 2.0 ** j)
    w2 = w.copy()
    w2[0, :, 5] *= np.float32(3.7)
    q1, s1 = O.quantize_log(w2, bits)
    keep = np.arange(32) != 5
    assert np.array_equal(q0[..., keep], q1[..., keep]) and np.array_equal(s0[..., keep], s1[..., keep])


@pytest.mark.parametrize("bits", BITS)
def test_zero_channel_tensor_scale_and_packing(bits):
    w = _rand((2, 128, 16), 26)
    w[0, :, 3] = 0
    q, s = O.quantize_log(w, bits)
    assert s[0, 3] == 0 and np.all(O.dequantize_log(q, s, bits)[0, :, 3] == 0)
    assert np.all(q[0, :, 3] == -(1 << (bits - 1)))          # field 0
    qt, st = O.quantize_log(w, bits, scale_per="tensor")
    assert np.all(st == st[:, :1])
    assert np.array_equal(st[:, 0].astype(np.float64), s.astype(np.float64).max(axis=1))
    # the codes are b-bit fields like the linear ones: the same dense packing holds them
    assert np.array_equal(O.unpack(O.pack(q, bits), bits, 128, 16), q)
    with pytest.raises(ValueError):
        O.quantize_log(w, 8)
    with pytest.raises(ValueError):
        O.quantize_log(w, bits, scale_per="row")
