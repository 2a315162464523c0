"""Pins for the oracle's dense bit packing (Table 2 size column: exactly b bits
per expert weight) and the written layout function."""

import numpy as np
import pytest

from oracle import brute
from oracle import moqe_oracle as O

BITS = (2, 3, 4, 8)


def _codes(bits, E, K, N, seed):
    lo, hi = O.code_range(bits)
    return np.random.default_rng(seed).integers(lo, hi + 1, size=(E, K, N)).astype(np.int8)


@pytest.mark.parametrize("bits", BITS)
def test_density_is_exactly_b_bits_per_weight(bits):
    for K, N in ((128, 16), (1024, 4096), (4096, 1024), (768, 3072)):
        assert O.packed_bytes(bits, K, N) * 8 == K * N * bits
    q = _codes(bits, 2, 256, 32, 1)
    assert O.pack(q, bits).shape == (2, 256 * 32 * bits // 8)


def test_table2_size_column():
    # Table 2: int8 0.54X, int4 0.32X, int3 0.26X, int2 0.20X of the fp16 MoE.
    # With the expert fraction implied by the int8 row (f ~ 0.91) the model
    # 1 - f (1 - b/16) gives the other rows only if int3 costs exactly 3 bits.
    f = (1 - 0.54) / (1 - 8 / 16)
    for bits, printed in ((8, 0.54), (4, 0.32), (3, 0.26), (2, 0.20)):
        assert abs(O.model_size_ratio(f, bits) - printed) < 0.0125
    assert abs(O.model_size_ratio(f, 4) - 0.32) < abs(O.model_size_ratio(f, 3) - 0.32)  # int3 padded to 4 bits would read 0.32


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("K", (128, 256, 512))
def test_roundtrip_random(bits, K):
    q = _codes(bits, 2, K, 48, K + bits)
    p = O.pack(q, bits)
    assert np.array_equal(O.unpack(p, bits, K, 48), q)


@pytest.mark.parametrize("bits,K", ((4, 32), (4, 64), (2, 64), (4, 96), (2, 192), (3, 128), (3, 768)))
def test_roundtrip_small_K(bits, K):
    q = _codes(bits, 1, K, 16, 3)
    assert np.array_equal(O.unpack(O.pack(q, bits), bits, K, 16), q)


def test_rejected_shapes():
    with pytest.raises(ValueError):
        O.code_positions(2, 32, 16)
    with pytest.raises(ValueError):
        O.code_positions(3, 64, 16)
    with pytest.raises(ValueError):
        O.code_positions(4, 48, 16)
    with pytest.raises(ValueError):
        O.code_positions(4, 64, 24)
    with pytest.raises(ValueError):
        O.code_positions(4, 160, 16)      # 5 steps, chunk of 4 does not divide


@pytest.mark.parametrize("bits", BITS)
def test_positions_form_a_partition(bits):
    """Every bit of the packed string belongs to exactly one code field."""
    K, N = 256, 32
    planes = O.code_positions(bits, K, N)
    used = np.zeros(O.packed_bytes(bits, K, N) * 8, dtype=np.int32)
    for _, _, off, sh, fbits in planes:
        for b in range(fbits):
            np.add.at(used, (off * 8 + sh + b).ravel(), 1)
    assert np.all(used == 1)


@pytest.mark.parametrize("bits", BITS)
def test_every_value_at_every_slot_of_a_chunk(bits):
    K, N = (128, 16)
    lo, hi = O.code_range(bits)
    for v in range(lo, hi + 1):
        q = np.full((1, K, N), v, dtype=np.int8)
        assert np.array_equal(O.unpack(O.pack(q, bits), bits, K, N), q)
    # a ramp that gives every position a different neighbour pattern
    q = ((np.arange(K)[:, None] * 7 + np.arange(N)[None, :] * 3) % (hi - lo + 1) + lo).astype(np.int8)[None]
    assert np.array_equal(O.unpack(O.pack(q, bits), bits, K, N), q)


@pytest.mark.parametrize("bits", BITS)
def test_single_code_sensitivity(bits):
    K, N = 256, 32
    lo, hi = O.code_range(bits)
    q = _codes(bits, 1, K, N, 21)
    base = O.pack(q, bits)[0]
    planes = O.code_positions(bits, K, N)
    rng = np.random.default_rng(22)
    for _ in range(40):
        k, n = int(rng.integers(K)), int(rng.integers(N))
        q2 = q.copy()
        q2[0, k, n] = lo if q[0, k, n] != lo else hi
        diff = np.bitwise_xor(O.pack(q2, bits)[0], base)
        allowed = np.zeros_like(diff)
        for _, _, off, sh, fbits in planes:
            allowed[off[k, n]] |= ((1 << fbits) - 1) << sh[k, n]
        assert np.all(diff & ~allowed == 0) and diff.any()


@pytest.mark.parametrize("bits,K,N", ((4, 64, 16), (4, 256, 32), (2, 64, 16), (2, 512, 16), (3, 128, 16), (3, 512, 32),
                                      (8, 32, 16), (8, 256, 32)))
def test_matches_storage_order_enumeration(bits, K, N):
    """The oracle maps code -> position; the brute force walks positions -> code."""
    q = _codes(bits, 1, K, N, 31)[0]
    assert O.pack(q, bits).tobytes() == brute.pack_matrix(q.tolist(), bits)


def test_layout_spot_values():
    """A few positions worked out by hand from the layout function."""
    # int4, K=128 (one chunk of 4 steps): slot = 16*((k%32)//8) + n%16, 16 bytes per slot.
    pl = O.code_positions(4, 128, 32)[0]
    off, sh = pl[2], pl[3]
    assert (off[0, 0], sh[0, 0]) == (0, 0)          # k=0: word 0, half 0, field 0
    assert (off[1, 0], sh[1, 0]) == (2, 0)          # k=1: half 1 -> bit 16
    assert (off[2, 0], sh[2, 0]) == (0, 4)          # k=2: half 0, field 1
    assert (off[8, 0], sh[8, 0]) == (16 * 16, 0)    # k=8: row group 1 -> slot 16
    assert (off[32, 0], sh[32, 0]) == (4, 0)        # k=32: step 1 -> word 1
    assert (off[0, 16], sh[0, 16]) == (1024, 0)     # second column tile
    # int2, K=256: 8 steps per chunk, 16 codes per word
    pl = O.code_positions(2, 256, 16)[0]
    off, sh = pl[2], pl[3]
    assert (off[32, 0], sh[32, 0]) == (1, 0)        # step 1 -> t=8 -> field 4 -> bit 8
    assert (off[33, 0], sh[33, 0]) == (3, 0)        # half 1 -> bit 24
    assert (off[64, 0], sh[64, 0]) == (4, 0)        # step 2 -> word 1
    # int3, K=256: 2-bit plane 1024 B, then 1-bit plane 512 B per chunk
    lo_pl, hi_pl = O.code_positions(3, 256, 16)
    assert (lo_pl[2][0, 0], hi_pl[2][0, 0]) == (0, 1024)
    assert (hi_pl[2][96, 0], hi_pl[3][96, 0]) == (1024 + 1, 4)   # step 3 -> t=24 -> field 12
    assert (hi_pl[2][128, 0], hi_pl[3][128, 0]) == (1024 + 4, 0)  # step 4 -> word 1


def test_fp16_storage_roundtrip_order_and_spots():
    """The unquantized 16-bit path stores fp16(A) by the same layout rule: round trip, the
    position -> element brute force, positions worked out by hand, and one rounding to nearest."""
    rng = np.random.default_rng(41)
    w = (rng.standard_normal((2, 96, 32)) * 0.02).astype(np.float32)
    p = O.pack_fp16(w)
    assert p.shape == (2, 96 * 32 * 2)
    assert np.array_equal(O.unpack_fp16(p, 96, 32), w.astype(np.float16))
    pat = w[0].astype(np.float16).view(np.uint16).astype(int).tolist()
    assert p[0].tobytes() == brute.pack_matrix(pat, 16)
    # K=64 (chunks of one step): slot = 16*((k%32)//8) + n%16 owns 16 bytes = 8 halves, k%8 in order
    lo, hi = O.code_positions(16, 64, 32)
    off = lo[2]
    assert off[0, 0] == 0 and hi[2][0, 0] == 1      # low byte, high byte
    assert off[1, 0] == 2 and off[7, 0] == 14
    assert off[8, 0] == 16 * 16                     # row group 1 -> slot 16
    assert off[32, 0] == 1024                       # step 1 -> next chunk of the column tile
    assert off[0, 16] == 2048                       # second column tile (2 chunks of 1024 bytes each)
    # 1 + 2^-11 lies half way between two fp16 numbers: ties to even -> 1.0
    one = np.full((32, 16), 1.0 + 2.0 ** -11, dtype=np.float32)
    assert np.all(O.unpack_fp16(O.pack_fp16(one), 32, 16) == np.float16(1.0))
