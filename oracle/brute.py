"""Brute-force scalar versions of the oracle's steps, for tiny inputs only.

TEST INFRASTRUCTURE ONLY (see moqe_oracle).  Pure-Python loops over single
numbers, written as independent formulations so they can pin the numpy oracle:
the quantizer walks one scalar at a time and finds the fp16 scale by searching
the half-precision bit patterns; the packer enumerates storage positions and
asks which code lives there (the inverse of the oracle's code -> position map);
the FFN evaluates every expert for every token and then selects.
"""

from __future__ import annotations

import math
import struct


def _half_from_bits(u: int) -> float:
    return struct.unpack("<e", struct.pack("<H", u))[0]


def smallest_half_at_least(v: float) -> tuple[int, float]:
    """Smallest non-negative fp16 value >= v, by bisection over bit patterns
    0x0000..0x7BFF (monotone in value).  Returns (bits, value)."""
    if not (0.0 <= v <= 65504.0):
        raise ValueError("not representable")
    lo, hi = 0, 0x7BFF
    while lo < hi:
        mid = (lo + hi) // 2
        if _half_from_bits(mid) >= v:
            hi = mid
        else:
            lo = mid + 1
    return lo, _half_from_bits(lo)


def round_half_even(r: float) -> int:
    f = math.floor(r)
    d = r - f
    if d < 0.5:
        return int(f)
    if d > 0.5:
        return int(f) + 1
    return int(f) if int(f) % 2 == 0 else int(f) + 1


def quantize_column(col, bits: int):
    """App. A linear quantization of one channel (a Python list of floats).
    Returns (codes list[int], scale float (an fp16 value), scale_bits int)."""
    m = max(abs(float(v)) for v in col)
    s_bits, s = smallest_half_at_least(2.0 * m / ((1 << bits) - 1))
    lo, hi = -(1 << (bits - 1)), (1 << (bits - 1)) - 1
    codes = []
    for v in col:
        if s == 0.0:
            codes.append(0)
            continue
        codes.append(min(hi, max(lo, round_half_even(float(v) / s))))
    return codes, s, s_bits


def quantize_matrix(w, bits: int):
    """w: list of K rows of N floats.  Returns (q[K][N], scales[N])."""
    K, N = len(w), len(w[0])
    q = [[0] * N for _ in range(K)]
    scales = [0.0] * N
    for n in range(N):
        codes, s, _ = quantize_column([w[k][n] for k in range(K)], bits)
        scales[n] = s
        for k in range(K):
            q[k][n] = codes[k]
    return q, scales


def log_quantize_column(col, bits: int):
    """App. A log-scale quantization of one channel, in exact rational arithmetic and straight
    from the printed formulas: T = clip(|a|/s, 2^(1-2^(b-1)), 1), Q = ceil(log2(2T/3)) found as
    the smallest integer with 2^Q >= 2T/3, sign kept apart; s = smallest fp16 >= max|a|.
    Returns (signs list[int] (1 = negative), exponents list[int], scale float)."""
    from fractions import Fraction

    m = max(abs(float(v)) for v in col)
    _, s = smallest_half_at_least(m)
    low = Fraction(1, 2 ** ((1 << (bits - 1)) - 1))
    signs, expos = [], []
    for v in col:
        signs.append(1 if float(v) < 0 else 0)
        if s == 0.0:
            expos.append(None)
            continue
        t = abs(Fraction(float(v))) / Fraction(s)
        t = min(Fraction(1), max(low, t))
        target = Fraction(2, 3) * t
        expo = 0
        while Fraction(2) ** (expo - 1) >= target:   # 2^Q >= 2T/3 still holds one lower
            expo -= 1
        while Fraction(2) ** expo < target:
            expo += 1
        expos.append(expo)
    return signs, expos, s


def pack_matrix(q, bits: int) -> bytes:
    """Pack q[K][N] by enumerating the storage in order: column tile, chunk,
    (bit plane,) slot, 32-bit word, half, field -> which (k, n) sits there."""
    K, N = len(q), len(q[0])
    S = K // 32
    sc = min({4: 4, 8: 2, 16: 1}.get(bits, 8), S)
    assert K % 32 == 0 and N % 16 == 0 and S % sc == 0
    out = bytearray()
    z = 0 if bits == 16 else 1 << (bits - 1)  # 16: q holds fp16 bit patterns, stored as they are
    plane_defs = [(bits, 0, (1 << bits) - 1)] if bits in (2, 4, 8, 16) else [(2, 0, 3), (1, 2, 1)]
    for c in range(N // 16):
        for p in range(S // sc):
            for fbits, vshift, vmask in plane_defs:
                per = 32 // fbits
                codes_per_slot = 8 * sc
                assert codes_per_slot % per == 0
                for slot in range(64):
                    g, j = slot // 16, slot % 16
                    n = 16 * c + j
                    for word in range(codes_per_slot // per):
                        val = 0
                        for half in range(2):
                            for field in range(per // 2):
                                t = 2 * field + half
                                m = word * per + t
                                s1, i = m // 8, m % 8
                                k = 32 * (p * sc + s1) + 8 * g + i
                                u = q[k][n] + z
                                val |= ((u >> vshift) & vmask) << (16 * half + fbits * field)
                        out += struct.pack("<I", val)
    assert len(out) == K * N * bits // 8
    return bytes(out)


def softmax_top1(logit_row):
    """(argmax with lowest index on ties, softmax probability there)."""
    best = 0
    for e in range(1, len(logit_row)):
        if logit_row[e] > logit_row[best]:
            best = e
    mx = logit_row[best]
    den = sum(math.exp(v - mx) for v in logit_row)
    return best, 1.0 / den


def route(x, w_gate):
    """x: T rows of d floats, w_gate: d rows of E floats."""
    T, d, E = len(x), len(w_gate), len(w_gate[0])
    idx, gate = [], []
    for t in range(T):
        logits = [math.fsum(x[t][k] * w_gate[k][e] for k in range(d)) for e in range(E)]
        b, g = softmax_top1(logits)
        idx.append(b)
        gate.append(g)
    counts = [0] * E
    for b in idx:
        counts[b] += 1
    offs = [0]
    for cnt in counts:
        offs.append(offs[-1] + cnt)
    perm = [t for e in range(E) for t in range(T) if idx[t] == e]
    return idx, gate, offs, perm


def expert_ffn_every_expert(x, idx, gate, w1, b1, w2, b2):
    """y_t = sum_e [e == idx_t] g_t FFN_e(x_t): all experts evaluated, then
    selected.  Arguments are nested Python lists; weights already dequantized."""
    T, d = len(x), len(x[0])
    E, f = len(w1), len(b1[0])
    y = [[0.0] * d for _ in range(T)]
    for t in range(T):
        for e in range(E):
            h = [max(0.0, math.fsum(x[t][k] * w1[e][k][n] for k in range(d)) + b1[e][n])
                 for n in range(f)]
            o = [math.fsum(h[k] * w2[e][k][n] for k in range(f)) + b2[e][n] for n in range(d)]
            sel = 1.0 if e == idx[t] else 0.0
            for n in range(d):
                y[t][n] += sel * gate[t] * o[n]
    return y
