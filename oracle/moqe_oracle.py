"""MoQE CPU oracle: plain, slow, fp64 numpy statement of what the hot path computes.

TEST INFRASTRUCTURE ONLY.  Nothing on the product path may import this module;
only the tests, the smoke check and the benchmark's CPU-baseline leg do.  It
shares no code, tables or helpers with the HIP library and never imports it.

What it states (all arithmetic IEEE fp64 unless the paper fixes a precision):

* ``quantize`` / ``dequantize``  - channel-wise linear quantization with the
  absolute maximum, paper App. A "Linear quantization with absolute maximum"
  (s_j = 2 max|A_:,j| / (2^b - 1), Q = int(A / s), A' = Q * s), scales kept in
  half precision as App. C says.
* ``quantize_log`` / ``dequantize_log`` - the log-scale alternative of App. A
  (sign bit + (b-1)-bit exponent, A' = P * s * 2^Q), which the paper compares
  with the linear one and sets aside.
* ``pack`` / ``unpack``          - the dense b-bit storage implied by Table 2's
  size column (exactly b bits per weight); the byte/bit position of every code
  is the layout function written out in ``code_positions``.
* ``route``                      - top-1 learned gating (App. B "MoE
  architecture", Switch-style): softmax over x W_g, expert = argmax, gate = that
  probability; then the per-expert histogram, exclusive scan and stable token
  permutation the dispatch needs.
* ``expert_ffn``                 - the two-layer Transformer FFN of Sec. 2.1
  (ReLU, with biases) evaluated with the token's expert, output scaled by the
  gate; ``moe_layer`` / ``stack`` chain the pieces.

Readings taken where the paper is silent are listed next to each function.
Parity status: every function here is pinned by tests (closed forms, worked
hand examples, invariants, brute force); none is "parity unpinned".
"""

from __future__ import annotations

import numpy as np

SUPPORTED_BITS = (2, 3, 4, 8)  # Table 2's quantized rows: int8, int4, int3, int2


# --------------------------------------------------------------------------
# quantizer (App. A, linear quantization with absolute maximum; App. C scales)
# --------------------------------------------------------------------------

def code_range(bits: int) -> tuple[int, int]:
    """Two's-complement range of a b-bit code: [-(2^(b-1)), 2^(b-1)-1]."""
    if bits not in SUPPORTED_BITS:
        raise ValueError(f"unsupported bit width {bits}")
    return -(1 << (bits - 1)), (1 << (bits - 1)) - 1


def fp16_round_up(s64) -> np.ndarray:
    """Smallest half-precision number >= s64 (one rounding, toward +inf).

    App. C stores the scaling factors in fp16.  Reading: the stored fp16 scale
    is also the one used to quantize, and it is rounded upward so that
    max|A|/s never exceeds (2^b - 1)/2; this keeps |a - q s| <= s/2 for every
    entry (round-to-nearest could shrink s and break that bound at the
    channel maximum).
    """
    s64 = np.asarray(s64, dtype=np.float64)
    if not np.all(np.isfinite(s64)) or np.any(s64 < 0) or np.any(s64 > 65504.0):
        raise ValueError("scale not representable in fp16 (non-finite weight or overflow)")
    h = s64.astype(np.float16)                       # nearest-even, single rounding
    low = h.astype(np.float64) < s64
    h = np.where(low, np.nextafter(h, np.float16(np.inf)), h).astype(np.float16)
    return h


def quantize(w, bits: int, scale_per: str = "channel"):
    """Channel-wise absmax linear quantization of a stack of matrices.

    w: [E, K, N] (or [K, N]); a channel is a column A_:,j, i.e. one of the N
    outputs of y = x A, and the maximum runs over the K inputs.
    Returns (q int8 [E,K,N], s fp16 [E,N]).

    Steps, in the paper's order: s_j = 2 max|A_:,j| / (2^b - 1); store s in
    fp16 (rounded up, see fp16_round_up); Q = int(A / s) read as
    round-to-nearest, ties to even, evaluated in fp64 with the stored scale;
    clamp to the two's-complement range (A/s spans +-(2^b-1)/2, whose rounding
    has one level too many for b bits).  An all-zero channel gets s = 0 and
    codes 0.

    scale_per = "tensor" is the alternative App. A names ("per the whole tensor", the
    matrix-wise scale App. C compares against): one s = 2 max|A| / (2^b - 1) for the whole
    matrix, returned as N equal channel scales so that everything downstream is unchanged.
    """
    if scale_per not in ("channel", "tensor"):
        raise ValueError("scale_per must be 'channel' or 'tensor'")
    w = np.asarray(w)
    squeeze = w.ndim == 2
    if squeeze:
        w = w[None]
    if w.ndim != 3:
        raise ValueError("w must be [E,K,N] or [K,N]")
    lo, hi = code_range(bits)
    E, K, N = w.shape
    q = np.empty((E, K, N), dtype=np.int8)
    s = np.empty((E, N), dtype=np.float16)
    for e in range(E):
        a = w[e].astype(np.float64)
        m = np.max(np.abs(a), axis=0)
        if scale_per == "tensor":
            m = np.full_like(m, m.max())
        s64 = (2.0 * m) / float((1 << bits) - 1)
        s16 = fp16_round_up(s64)
        sd = s16.astype(np.float64)
        nz = sd > 0.0
        r = a / np.where(nz, sd, 1.0)[None, :]
        r = np.rint(r)
        r = np.where(nz[None, :], r, 0.0)
        q[e] = np.clip(r, lo, hi).astype(np.int8)
        s[e] = s16
    if squeeze:
        return q[0], s[0]
    return q, s


def dequantize(q, s) -> np.ndarray:
    """A'_:,j = Q_:,j * s_j (App. A), exact in fp64. q [...,K,N], s [...,N]."""
    q = np.asarray(q)
    s = np.asarray(s)
    return q.astype(np.float64) * s.astype(np.float64)[..., None, :]


def quantize_fp16(w) -> np.ndarray:
    """The unquantized 16-bit path: A' = fp16(A), returned as fp64."""
    return np.asarray(w).astype(np.float16).astype(np.float64)


# --------------------------------------------------------------------------
# log-scale quantizer (App. A, "log-scale quantization": the alternative the
# paper compares with the linear one and does not adopt)
# --------------------------------------------------------------------------

LOG_BITS = (2, 3, 4)


def log_exponent_range(bits: int) -> tuple[int, int]:
    """Exponents Q a b-bit log code can hold: one bit is the sign, the other b-1 bits
    count the 2^(b-1) values 1 - 2^(b-1) .. 0."""
    if bits not in LOG_BITS:
        raise ValueError(f"unsupported log-scale bit width {bits}")
    return 1 - (1 << (bits - 1)), 0


def quantize_log(w, bits: int, scale_per: str = "channel"):
    """Log-scale quantization of a stack of matrices (App. A).

    P = sign(A);  T = clip(|A| / s, 2^(1 - 2^(b-1)), 1);  Q = ceil(log2(2/3 T)).
    Returns (q int8 [E,K,N], s fp16 [E,N]).

    Readings.  The printed clip has its two bounds in the order (1, 2^(1-2^(b-1))), a lower
    bound above the upper one; it is read as the interval [2^(1-2^(b-1)), 1], the one whose
    ends give exactly the 2^(b-1) exponents 1 - 2^(b-1) .. 0 that b - 1 bits can count.
    s is the first of the two choices the paper names, the absolute maximum (the MSE-optimal
    search is another paper's algorithm), taken per output channel like the linear scale (or
    per matrix with scale_per = "tensor") and stored in fp16 rounded upward, so that T <= 1.
    Q = ceil(log2(2T/3)) is the smallest integer with 2^Q >= 2T/3, i.e. with
    |A| <= 1.5 * 2^Q * s; that comparison is exact in floating point (1.5 * 2^Q * s has few
    bits), so the exponent is decided without rounding a quotient or a logarithm.  It rounds
    |A|/s to the nearest power of two on the linear axis (the break between 2^(Q-1) and 2^Q is
    their mean 0.75 * 2^Q, which goes down).
    Stored code: u = sign_bit * 2^(b-1) + (Q - (1 - 2^(b-1))), a b-bit field; it is returned
    offset like the linear codes, q = u - 2^(b-1), so that pack() / unpack() serve both.
    A zero weight has T below the lower bound and takes the smallest magnitude with a plus
    sign (the format has no zero); an all-zero channel has s = 0 and decodes to zeros.
    """
    if scale_per not in ("channel", "tensor"):
        raise ValueError("scale_per must be 'channel' or 'tensor'")
    q_lo, q_hi = log_exponent_range(bits)
    w = np.asarray(w)
    squeeze = w.ndim == 2
    if squeeze:
        w = w[None]
    if w.ndim != 3:
        raise ValueError("w must be [E,K,N] or [K,N]")
    E, K, N = w.shape
    half = 1 << (bits - 1)
    q = np.empty((E, K, N), dtype=np.int8)
    s = np.empty((E, N), dtype=np.float16)
    for e in range(E):
        a = w[e].astype(np.float64)
        m = np.max(np.abs(a), axis=0)
        if scale_per == "tensor":
            m = np.full_like(m, m.max())
        s16 = fp16_round_up(m)
        sd = s16.astype(np.float64)
        mag = np.abs(a)
        # smallest exponent in range whose upper break 1.5 * 2^Q * s is not below |A|
        expo = np.full((K, N), q_hi, dtype=np.int64)
        for cand in range(q_hi - 1, q_lo - 1, -1):
            expo = np.where(mag <= 1.5 * 2.0 ** cand * sd[None, :], cand, expo)
        neg = (a < 0).astype(np.int64)
        u = neg * half + (expo - q_lo)
        u = np.where(sd[None, :] > 0, u, 0)
        q[e] = (u - half).astype(np.int8)
        s[e] = s16
    if squeeze:
        return q[0], s[0]
    return q, s


def log_code_parts(q, bits: int):
    """(negative flag, exponent Q) of stored log codes q = u - 2^(b-1)."""
    q_lo, _ = log_exponent_range(bits)
    half = 1 << (bits - 1)
    u = np.asarray(q).astype(np.int64) + half
    return u >= half, (u % half) + q_lo


def dequantize_log(q, s, bits: int) -> np.ndarray:
    """A' = P * s * 2^Q (App. A), exact in fp64. q [...,K,N], s [...,N]."""
    neg, expo = log_code_parts(q, bits)
    mag = np.asarray(s).astype(np.float64)[..., None, :] * 2.0 ** expo
    return np.where(neg, -mag, mag)


# --------------------------------------------------------------------------
# dense bit packing (Table 2 size column: exactly b bits per weight)
# --------------------------------------------------------------------------

def packed_bytes(bits: int, K: int, N: int) -> int:
    """Bytes of one packed [K,N] matrix: K*N*b/8, no padding."""
    return K * N * bits // 8


def model_size_ratio(expert_fraction: float, bits: int) -> float:
    """Whole-model size relative to fp16 when only the expert weights (a
    fraction f of all weights) go from 16 to b bits: 1 - f (1 - b/16)."""
    return 1.0 - expert_fraction * (1.0 - bits / 16.0)


def steps_per_chunk(bits: int, K: int) -> int:
    """SC of the layout below: 32-row steps per chunk."""
    if bits not in SUPPORTED_BITS and bits != 16:
        raise ValueError(f"unsupported bit width {bits}")
    if K <= 0 or K % 32:
        raise ValueError("K must be a positive multiple of 32")
    S = K // 32
    sc = min({4: 4, 8: 2, 16: 1}.get(bits, 8), S)  # a slot owns at most 16 bytes of a chunk's main plane
    if S % sc:
        raise ValueError("K/32 must be a multiple of the chunk length")
    if bits == 2 and sc % 2:
        raise ValueError("int2 needs K to be a multiple of 64")
    if bits == 3 and sc % 4:
        raise ValueError("int3 needs K to be a multiple of 128")
    return sc


def code_positions(bits: int, K: int, N: int):
    """Where every code of one [K,N] matrix lives in its packed byte string.

    Returns a list of planes; each plane is (value_shift, value_mask,
    byte_offset[K,N], bit_shift[K,N], field_bits): the stored field is
    ((u >> value_shift) & value_mask) with u = q + 2^(b-1) (offset binary),
    placed at bit `bit_shift` of byte `byte_offset`.

    Layout function (the storage the device reads; the paper gives none):
      n -> column tile c = n // 16, j = n % 16
      k -> step s = k // 32, row group g = (k % 32) // 8, i = k % 8
      slot l = 16 g + j (64 slots per tile), chunk p = s // SC, s' = s % SC,
      m = 8 s' + i  (index among the 8 SC codes a slot owns in a chunk)
      Q = K / (32 SC) chunks per column tile; chunks are stored tile-major.
    b in {2,4,8}: a chunk is 64 slots x (SC b) bytes, slot-major; inside a slot
      32/b codes fill one little-endian 32-bit word: word = m // (32/b),
      t = m % (32/b), half = t & 1, field = t >> 1, bit = 16 half + b field.
    b = 3: a chunk is a 2-bit plane (as b = 2, holding u & 3) followed by a
      1-bit plane (holding u >> 2): 64 slots x SC bytes, word = m // 32,
      t = m % 32, half = t & 1, field = t >> 1, bit = 16 half + field.
    b = 16 (the unquantized half-precision path, see pack_fp16): the same rule as b in {2,4,8}
      with u = the fp16 bit pattern; a field is a whole half of a word, returned here as its
      low and its high byte.
    """
    sc = steps_per_chunk(bits, K)
    if N <= 0 or N % 16:
        raise ValueError("N must be a positive multiple of 16")
    S = K // 32
    Q = S // sc
    k = np.arange(K, dtype=np.int64)[:, None]
    n = np.arange(N, dtype=np.int64)[None, :]
    c, j = n // 16, n % 16
    s, g, i = k // 32, (k % 32) // 8, k % 8
    slot = 16 * g + j
    p, s1 = s // sc, s % sc
    m = 8 * s1 + i
    chunk_bytes = 64 * sc * bits
    base = (c * Q + p) * chunk_bytes

    def plane(field_bits, lane_bytes, plane_off):
        per = 32 // field_bits
        word, t = m // per, m % per
        half, field = t & 1, t >> 1
        bit = 16 * half + field_bits * field
        off = base + plane_off + slot * lane_bytes + 4 * word + bit // 8
        return np.broadcast_to(off, (K, N)).copy(), np.broadcast_to(bit % 8, (K, N)).copy()

    if bits in (2, 4, 8):
        off, sh = plane(bits, sc * bits, 0)
        return [(0, (1 << bits) - 1, off, sh, bits)]
    if bits == 16:
        off, sh = plane(16, sc * 16, 0)
        return [(0, 255, off, sh, 8), (8, 255, off + 1, sh, 8)]
    lo_off, lo_sh = plane(2, sc * 2, 0)
    hi_off, hi_sh = plane(1, sc, 64 * sc * 2)
    return [(0, 3, lo_off, lo_sh, 2), (2, 1, hi_off, hi_sh, 1)]


def pack(q, bits: int) -> np.ndarray:
    """Codes int8 [E,K,N] -> uint8 [E, K*N*b/8] in the layout of code_positions."""
    q = np.asarray(q)
    squeeze = q.ndim == 2
    if squeeze:
        q = q[None]
    E, K, N = q.shape
    lo, hi = code_range(bits)
    if q.min(initial=0) < lo or q.max(initial=0) > hi:
        raise ValueError("code out of range")
    planes = code_positions(bits, K, N)
    nbytes = packed_bytes(bits, K, N)
    out = np.zeros((E, nbytes), dtype=np.uint8)
    for e in range(E):
        u = (q[e].astype(np.int64) + (1 << (bits - 1)))
        acc = np.zeros(nbytes, dtype=np.float64)
        for vshift, vmask, off, sh, _ in planes:
            v = ((u >> vshift) & vmask) << sh
            # fields are disjoint, so the sum of the shifted fields is their OR
            acc += np.bincount(off.ravel(), weights=v.ravel().astype(np.float64), minlength=nbytes)
        out[e] = acc.astype(np.uint8)
    return out[0] if squeeze else out


def pack_fp16(w) -> np.ndarray:
    """The unquantized 16-bit path's storage: A' = fp16(A) (one rounding, to nearest even), its
    bit patterns laid out by the same rule as the codes (code_positions with b = 16), so that
    the fp16 and the quantized experts go through the same kernels.
    w [E,K,N] (or [K,N]) -> uint8 [E, 2 K N]."""
    w = np.asarray(w)
    squeeze = w.ndim == 2
    if squeeze:
        w = w[None]
    E, K, N = w.shape
    planes = code_positions(16, K, N)
    nbytes = 2 * K * N
    out = np.zeros((E, nbytes), dtype=np.uint8)
    for e in range(E):
        u = w[e].astype(np.float16).view(np.uint16).astype(np.int64)
        for vshift, vmask, off, sh, _ in planes:
            out[e][off.ravel()] = ((u >> vshift) & vmask).ravel().astype(np.uint8)
    return out[0] if squeeze else out


def unpack_fp16(codes, K: int, N: int) -> np.ndarray:
    """Inverse of pack_fp16: uint8 [E, 2 K N] -> fp16 [E,K,N]."""
    codes = np.asarray(codes, dtype=np.uint8)
    squeeze = codes.ndim == 1
    if squeeze:
        codes = codes[None]
    if codes.shape[1] != 2 * K * N:
        raise ValueError("wrong packed length")
    planes = code_positions(16, K, N)
    out = np.empty((codes.shape[0], K, N), dtype=np.float16)
    for e in range(codes.shape[0]):
        u = np.zeros((K, N), dtype=np.int64)
        for vshift, vmask, off, sh, _ in planes:
            u |= (codes[e][off].astype(np.int64) & vmask) << vshift
        out[e] = u.astype(np.uint16).view(np.float16)
    return out[0] if squeeze else out


def unpack(codes, bits: int, K: int, N: int) -> np.ndarray:
    """Inverse of pack: uint8 [E, K*N*b/8] -> int8 [E,K,N]."""
    codes = np.asarray(codes, dtype=np.uint8)
    squeeze = codes.ndim == 1
    if squeeze:
        codes = codes[None]
    if codes.shape[1] != packed_bytes(bits, K, N):
        raise ValueError("wrong packed length")
    planes = code_positions(bits, K, N)
    E = codes.shape[0]
    q = np.empty((E, K, N), dtype=np.int8)
    for e in range(E):
        u = np.zeros((K, N), dtype=np.int64)
        for vshift, vmask, off, sh, _ in planes:
            u |= ((codes[e][off].astype(np.int64) >> sh) & vmask) << vshift
        q[e] = (u - (1 << (bits - 1))).astype(np.int8)
    return q[0] if squeeze else q


# --------------------------------------------------------------------------
# top-1 gating and dispatch (App. B "MoE architecture")
# --------------------------------------------------------------------------

def route_logits(x, w_gate) -> np.ndarray:
    """Router logits l = x W_g, x [T,d], W_g [d,E], fp64. No bias term."""
    return np.asarray(x).astype(np.float64) @ np.asarray(w_gate).astype(np.float64)


def route_from_logits(logits):
    """Top-1 gating from logits [T,E].

    expert_idx[t] = lowest index attaining max_e l[t,e]; gate[t] = softmax(l[t])
    at that index = 1 / sum_e exp(l[t,e] - l[t,e_t]).  Inference-time reading:
    no capacity limit or token dropping, no jitter, no gating dropout.  Dispatch
    bookkeeping: count per expert, exclusive prefix sum (seg_offsets[E] = T),
    and the stable permutation (tokens of one expert stay in ascending order).
    Non-finite logits are outside the method's domain; the definition is kept total all the
    same: a NaN counts as the row maximum (first NaN wins), a row of -inf takes expert 0, so
    the index is always in [0, E) and every token lands in exactly one segment (the gate of
    such a row is NaN).
    Returns (expert_idx int32 [T], gate f64 [T], seg_offsets int32 [E+1], perm int32 [T]).
    """
    l = np.asarray(logits, dtype=np.float64)
    T, E = l.shape
    expert_idx = np.argmax(l, axis=1).astype(np.int32) if T else np.zeros(0, np.int32)
    top = l[np.arange(T), expert_idx] if T else np.zeros(0)
    with np.errstate(invalid="ignore"):  # (-inf) - (-inf) and NaN rows give a NaN gate, by definition above
        gate = 1.0 / np.sum(np.exp(l - top[:, None]), axis=1) if T else np.zeros(0)
    counts = np.bincount(expert_idx, minlength=E)
    seg_offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    perm = np.argsort(expert_idx, kind="stable").astype(np.int32)
    return expert_idx, gate, seg_offsets, perm


def route(x, w_gate):
    """route_from_logits(route_logits(x, W_g))."""
    return route_from_logits(route_logits(x, w_gate))


def top2_margin(logits) -> np.ndarray:
    """Per-token gap between the largest and second largest logit (E >= 2)."""
    l = np.sort(np.asarray(logits, dtype=np.float64), axis=1)
    return l[:, -1] - l[:, -2]


# --------------------------------------------------------------------------
# expert FFN (Sec. 2.1: two-layer Transformer FFN; ReLU, biases)
# --------------------------------------------------------------------------

def expert_ffn(x, expert_idx, gate, w1, b1, w2, b2, residual=None) -> np.ndarray:
    """y_t = g_t * ( max(0, x_t W1'_e + b1_e) W2'_e + b2_e ),  e = expert_idx[t].

    x [T,d]; w1 [E,d,f], w2 [E,f,d] are the dequantized (or fp16) weights as
    fp64; b1 [E,f], b2 [E,d]; gate [T].  The gate multiplies the whole expert
    output, second bias included.  Nothing is rounded on the way.  With
    `residual` [T,d] the function returns residual + y (still fp64).
    Tokens are evaluated grouped by expert; rows are independent, so this is
    the per-token definition with a library matrix product as the step.
    """
    x = np.asarray(x).astype(np.float64)
    expert_idx = np.asarray(expert_idx)
    gate = np.asarray(gate, dtype=np.float64)
    T, d = x.shape
    y = np.zeros((T, d), dtype=np.float64)
    for e in np.unique(expert_idx):
        rows = np.nonzero(expert_idx == e)[0]
        h = np.maximum(0.0, x[rows] @ np.asarray(w1[e], dtype=np.float64)
                       + np.asarray(b1[e]).astype(np.float64))
        o = h @ np.asarray(w2[e], dtype=np.float64) + np.asarray(b2[e]).astype(np.float64)
        y[rows] = gate[rows, None] * o
    if residual is not None:
        y = np.asarray(residual).astype(np.float64) + y
    return y


def dense_ffn(x, w1, b1, w2, b2) -> np.ndarray:
    """Textbook dense FFN max(0, x W1 + b1) W2 + b2 in fp64 (one expert, gate 1)."""
    x = np.asarray(x).astype(np.float64)
    h = np.maximum(0.0, x @ np.asarray(w1, dtype=np.float64) + np.asarray(b1).astype(np.float64))
    return h @ np.asarray(w2, dtype=np.float64) + np.asarray(b2).astype(np.float64)


def quantize_layer(layer: dict, bits: int) -> dict:
    """Quantize one layer's expert weights.  layer holds fp32 'w1' [E,d,f],
    'w2' [E,f,d], fp16 'b1','b2', fp16 'w_gate'.  bits = 16 means the
    unquantized half-precision path."""
    out = dict(bits=bits, b1=layer["b1"], b2=layer["b2"], w_gate=layer["w_gate"])
    if bits == 16:
        out["w1d"] = quantize_fp16(layer["w1"])
        out["w2d"] = quantize_fp16(layer["w2"])
        return out
    out["q1"], out["s1"] = quantize(layer["w1"], bits)
    out["q2"], out["s2"] = quantize(layer["w2"], bits)
    return out


def layer_weights(qlayer: dict):
    """Dequantized fp64 weights (w1', w2') of a quantize_layer result."""
    if "w1d" in qlayer:
        return qlayer["w1d"], qlayer["w2d"]
    return dequantize(qlayer["q1"], qlayer["s1"]), dequantize(qlayer["q2"], qlayer["s2"])


def moe_layer(x, qlayer: dict, residual: bool = False, route_override=None):
    """One MoE layer: route, expert FFN, gate-weighted combine (top-1: a
    scaled un-permute).  Returns (y fp64 [T,d], routing tuple).
    route_override = (expert_idx, gate) evaluates the FFN under a given route."""
    r = route(x, qlayer["w_gate"])
    idx, gate = (r[0], r[1]) if route_override is None else route_override
    w1, w2 = layer_weights(qlayer)
    y = expert_ffn(x, idx, gate, w1, qlayer["b1"], w2, qlayer["b2"],
                   residual=x if residual else None)
    return y, r


def stack(x, qlayers) -> list:
    """Stack of MoE layers with an fp16 residual stream:
    x_{l+1} = fp16(x_l + MoE_l(x_l)).  Returns the list [x_0, x_1, ...] (fp16)."""
    xs = [np.asarray(x).astype(np.float16)]
    for ql in qlayers:
        y, _ = moe_layer(xs[-1], ql, residual=True)
        xs.append(y.astype(np.float16))
    return xs
