"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol include/moqe.h declares, and rejects bad arguments before launching."""

import ctypes
import os
import re

import pytest

from paper_2310_02410_amd import moqe

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "moqe.h")

pytestmark = pytest.mark.skipif(not os.path.exists(moqe.LIB_PATH), reason="libmoqe.so not built")


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(moqe_[a-z0-9_]+)\s*\(", src)))


def test_every_declared_symbol_is_exported():
    L = ctypes.CDLL(moqe.LIB_PATH)
    names = declared_functions()
    assert len(names) >= 13
    for n in names:
        assert hasattr(L, n), n
    assert sorted(moqe.EXPORTS) == names


def test_version_and_strings():
    L = moqe.lib()
    assert L.moqe_version() == 2
    assert L.moqe_set_prefill_policy(0, 65, 16) == -1 and L.moqe_set_prefill_policy(5, 0, 16) == -1
    assert L.moqe_set_prefill_policy(5, 65, 0) == -1
    assert L.moqe_set_prefill_policy(moqe.PREFILL_MIN_SEGMENT_DEFAULT, moqe.PREFILL_MIN_BATCH_DEFAULT,
                                     moqe.PREFILL_ALL_TILED_DEFAULT) == 0
    assert L.moqe_set_launch_mode(99) == -1
    old = L.moqe_set_launch_mode(moqe.LAUNCH_SEPARATE)
    assert L.moqe_set_launch_mode(old) == moqe.LAUNCH_SEPARATE
    assert L.moqe_status_string(0) == b"MOQE_OK"
    for s in range(1, 8):
        assert L.moqe_status_string(s).decode().startswith(moqe.STATUS_NAMES[s])
    assert L.moqe_set_decode_kernel(5) == -1
    old = L.moqe_set_decode_kernel(moqe.DECODE_GENERAL)
    assert L.moqe_set_decode_kernel(moqe.DECODE_ROWS8) == moqe.DECODE_GENERAL
    assert L.moqe_set_decode_kernel(moqe.DECODE_ROWS4) == moqe.DECODE_ROWS8
    assert L.moqe_set_decode_kernel(old) == moqe.DECODE_ROWS4
    assert L.moqe_set_tiled_kernel(3) == -1 and L.moqe_set_tiled_kernel(-1) == -1
    old = L.moqe_set_tiled_kernel(moqe.TILED_STREAMED)
    assert old == moqe.TILED_AUTO and L.moqe_set_tiled_kernel(old) == moqe.TILED_STREAMED
    assert L.moqe_workspace_status(None, 4096, None) == 1 and L.moqe_workspace_status(P, 512, None) == 5
    assert L.moqe_stream_read(None, 1024, P, None) == 1 and L.moqe_stream_read(P, 1000, P, None) == 3
    assert L.moqe_stream_read(P, 0, P, None) == 3 and L.moqe_stream_read(P + 8, 1024, P, None) == 4
    assert L.moqe_status_string(99) == b"unknown status"


def test_contraction_path_follows_the_settings():
    """The path query is host-only: which kernels a contraction launches, by batch size, width
    and the process-wide settings (benchmark layer: E = 32, d = 1024, f = 4096)."""
    m = moqe
    path = m.moqe_contraction_path
    E, d, f = 32, 1024, 4096
    try:
        m.moqe_set_prefill_policy()
        m.moqe_set_decode_kernel(m.DECODE_AUTO)
        m.moqe_set_tiled_kernel(m.TILED_AUTO)
        # decode-sized batches: the kernel for them, for both contractions
        for T in (1, 24, 64):
            assert path(4, T, E, d, f) == m.PATH_DECODE_SMALL and path(2, T, E, f, d) == m.PATH_DECODE_SMALL
        assert path(8, 24, E, d, f) == m.PATH_DECODE            # int8: general kernel only
        assert path(4, 24, 256, d, f) == m.PATH_DECODE          # more than 128 experts
        # 65 to 128 tokens: still the decode-sized kernel where its pairs of 8 rows apply (wave
        # slices of 32 steps: K = 1024 or 4096); above, or where they do not, everything tiled from
        # 2 tokens per expert on (16 at 8 bits); token rows resident in LDS where K <= 1024, and
        # up to K = 4096 while T <= 16 E
        for b in (4, 3, 2):
            assert path(b, 65, E, d, f) == m.PATH_DECODE_SMALL and path(b, 128, E, f, d) == m.PATH_DECODE_SMALL
            assert path(b, 129, E, d, f) == m.PATH_TILED_RESIDENT and path(b, 129, E, f, d) == m.PATH_TILED_RESIDENT
            assert path(b, 100, E, 3072, 768) == m.PATH_TILED_RESIDENT
            assert path(b, 100, E, 768, 3072) == (m.PATH_TILED_RESIDENT if b == 4 else m.PATH_TILED_STAGED)
            assert path(b, 100, 256, d, f) == m.PATH_DECODE and path(b, 512, 256, d, f) == m.PATH_TILED_RESIDENT
            assert path(b, 512, E, f, d) == m.PATH_TILED_RESIDENT and path(b, 513, E, f, d) == m.PATH_TILED_STAGED
            assert path(b, 513, E, d, f) == m.PATH_TILED_RESIDENT
            assert path(b, 129, 80, d, f) == m.PATH_DECODE and path(b, 160, 80, d, f) == m.PATH_TILED_RESIDENT
        assert path(8, 511, E, d, f) == m.PATH_DECODE and path(8, 512, E, d, f) == m.PATH_TILED_STAGED
        assert path(16, 24, E, d, f) == m.PATH_TILED_STAGED     # fp16 weights: tiled at every size
        # the settings move the answer
        m.moqe_set_tiled_kernel(m.TILED_STREAMED)
        assert path(4, 196, E, d, f) == m.PATH_TILED_STAGED
        m.moqe_set_tiled_kernel(m.TILED_RESIDENT)
        assert path(4, 4096, E, f, d) == m.PATH_TILED_RESIDENT
        m.moqe_set_tiled_kernel(m.TILED_AUTO)
        m.moqe_set_decode_kernel(m.DECODE_GENERAL)
        assert path(4, 24, E, d, f) == m.PATH_DECODE and path(4, 100, E, d, f) == m.PATH_TILED_RESIDENT
        m.moqe_set_decode_kernel(m.DECODE_ROWS4)    # pairs of 4 rows stop at 64 tokens
        assert path(4, 64, E, d, f) == m.PATH_DECODE_SMALL and path(4, 100, E, d, f) == m.PATH_TILED_RESIDENT
        m.moqe_set_decode_kernel(m.DECODE_AUTO)
        m.moqe_set_prefill_policy(5, 65, m.PREFILL_NEVER)       # both side by side
        assert path(4, 100, E, d, f) == m.PATH_DECODE_SMALL | m.PATH_TILED_RESIDENT
        assert path(4, 256, E, d, f) == m.PATH_DECODE | m.PATH_TILED_RESIDENT
        assert path(4, 256, E, f, d) == m.PATH_DECODE | m.PATH_TILED_RESIDENT
        assert path(4, 1024, E, f, d) == m.PATH_DECODE | m.PATH_TILED_STAGED
        assert path(4, 64, E, d, f) == m.PATH_DECODE_SMALL
        m.moqe_set_prefill_policy(m.PREFILL_NEVER, m.PREFILL_NEVER, m.PREFILL_NEVER)
        assert path(4, 4096, E, d, f) == m.PATH_DECODE and path(4, 128, E, d, f) == m.PATH_DECODE_SMALL
        m.moqe_set_prefill_policy(m.PREFILL_MIN_SEGMENT_DEFAULT, 1, 1)   # everything tiled from one token per expert on
        assert path(4, 48, E, d, f) == m.PATH_TILED_RESIDENT and path(4, 24, E, d, f) == m.PATH_DECODE_SMALL
        assert path(4, 100, E, d, f) == m.PATH_DECODE_SMALL     # (the decode-sized kernel keeps 65 to 128 tokens)
        m.moqe_set_prefill_policy(1, 1, m.PREFILL_NEVER)        # every segment tiled, at any size
        assert path(4, 24, E, d, f) == m.PATH_TILED_RESIDENT and path(4, 100, E, f, d) == m.PATH_TILED_RESIDENT
        # a K the tiled kernels do not take stays with the decode kernel
        m.moqe_set_prefill_policy()
        assert path(4, 4096, E, 128, 512) == m.PATH_DECODE
        # refused: unknown width, no tokens, a K that cannot be packed
        L = m.lib()
        assert L.moqe_contraction_path(5, 24, E, d, f) == -1 and L.moqe_contraction_path(4, 0, E, d, f) == -1
        assert L.moqe_contraction_path(4, 24, E, 100, f) == -1 and L.moqe_contraction_path(4, 24, 0, d, f) == -1
        with pytest.raises(ValueError):
            path(4, 24, E, 100, f)
    finally:
        m.moqe_set_prefill_policy()
        m.moqe_set_decode_kernel(m.DECODE_AUTO)
        m.moqe_set_tiled_kernel(m.TILED_AUTO)


@pytest.mark.parametrize("bits", (2, 3, 4, 8))
def test_packed_bytes_density(bits):
    # Table 2's size column: exactly `bits` bits per expert weight
    for K, N in ((1024, 4096), (4096, 1024), (768, 3072), (256, 64)):
        assert moqe.moqe_packed_bytes(bits, K, N) == K * N * bits // 8
    assert moqe.moqe_packed_bytes(4, 64, 256) == 64 * 256 // 2


def test_shape_rules():
    L = moqe.lib()
    assert L.moqe_check_matrix(5, 1024, 1024) == 2
    assert L.moqe_check_matrix(4, 48, 16) == 3       # K not a multiple of 32
    assert L.moqe_check_matrix(4, 64, 24) == 3       # N not a multiple of 16
    assert L.moqe_check_matrix(2, 32, 16) == 3       # int2 needs K % 64
    assert L.moqe_check_matrix(3, 64, 16) == 3       # int3 needs K % 128
    assert L.moqe_check_matrix(4, 160, 16) == 3      # 5 steps, chunk of 4
    assert L.moqe_check_matrix(4, 64, 256) == 0
    assert L.moqe_check_matrix(3, 768, 3072) == 0
    assert L.moqe_check_matrix(8, 32, 16) == 0 and L.moqe_check_matrix(8, 96, 16) == 3   # 3 steps, chunk of 2
    assert L.moqe_check_layer(8, 32, 1024, 4096) == 0
    # fp16 weights: packable from K = 32 on, but as a layer only where the tiled kernel takes both
    # contractions (K at least 256 and a multiple of 128)
    assert L.moqe_check_matrix(16, 32, 16) == 0 and moqe.moqe_packed_bytes(16, 256, 64) == 256 * 64 * 2
    assert L.moqe_check_layer(16, 32, 1024, 4096) == 0 and L.moqe_check_layer(16, 4, 384, 256) == 0
    assert L.moqe_check_layer(16, 4, 64, 256) == 3 and L.moqe_check_layer(16, 4, 256, 320) == 3
    assert moqe.moqe_packed_bytes(2, 32, 16) == 0
    assert L.moqe_check_layer(4, 4, 64, 256) == 0
    assert L.moqe_check_layer(2, 32, 1024, 4096) == 0
    assert L.moqe_check_layer(3, 128, 768, 3072) == 0
    assert L.moqe_check_layer(4, 0, 64, 256) == 3
    assert L.moqe_check_layer(4, 4, 96 * 32 * 5, 256) == 3   # K/32 = 480: no supported split


def test_workspace_sizes():
    head = 2048 + 2 * (1 << 20)       # counters, router results, the two chained h buffers
    assert moqe.moqe_ffn_workspace_bytes(24, 32, 1024, 4096) == head + 24 * 4096 * 2
    assert moqe.moqe_ffn_workspace_bytes(0, 32, 1024, 4096) == head + 256
    assert moqe.moqe_ffn_workspace_bytes(4096, 32, 1024, 4096) == head + 4096 * 4096 * 2
    assert moqe.moqe_layer_workspace_bytes(24, 32, 1024, 4096) == head + 24 * 4096 * 2 + 256
    assert moqe.moqe_route_workspace_bytes(24, 32) == 256
    assert moqe.moqe_route_workspace_bytes(1 << 20, 128) >= (1 << 20) // 64 * 128 * 4


P = 0x10000  # a fake, aligned, non-NULL device address; never dereferenced on the host


def test_quantize_error_paths():
    L = moqe.lib()
    assert L.moqe_quantize(0, 1, 64, 16, 4, P, P, None) == 1
    assert L.moqe_quantize(P, 1, 64, 16, 7, P, P, None) == 2
    assert L.moqe_quantize(P, 1, 48, 16, 4, P, P, None) == 3
    assert L.moqe_quantize(P, 0, 64, 16, 4, P, P, None) == 3
    assert L.moqe_quantize(P + 4, 1, 64, 16, 4, P, P, None) == 4
    assert L.moqe_unpack(P, 1, 64, 16, 4, 0, None) == 1
    assert L.moqe_unpack(P, 1, 64, 16, 1, P, None) == 2
    assert L.moqe_unpack(P, 1, 64, 16, 16, P, None) == 2       # fp16 weights are not int8 codes
    assert L.moqe_quantize_tensor_scale(P, 1, 64, 16, 7, P, P, None) == 2
    assert L.moqe_unpack(P, 1, 64, 20, 4, P, None) == 3
    # log-scale codec: 2, 3 or 4 bits only
    assert L.moqe_quantize_log(P, 1, 64, 16, 8, P, P, None) == 2
    assert L.moqe_quantize_log(P, 1, 64, 16, 16, P, P, None) == 2
    assert L.moqe_quantize_log(0, 1, 64, 16, 4, P, P, None) == 1
    assert L.moqe_quantize_log(P, 1, 48, 16, 4, P, P, None) == 3
    assert L.moqe_dequantize_log(P, P, 1, 64, 16, 8, P, None) == 2
    assert L.moqe_dequantize_log(P, 0, 1, 64, 16, 4, P, None) == 1
    assert L.moqe_dequantize_log(P, P, 1, 64, 24, 4, P, None) == 3
    assert L.moqe_dequantize_log(P, P, 1, 64, 16, 4, P + 4, None) == 4


def test_route_error_paths():
    L = moqe.lib()
    assert L.moqe_route(0, P, 8, 64, 4, P, P, P, P, P, 256, None) == 1
    assert L.moqe_route(P, P, 8, 64, 4, P, 0, P, P, P, 256, None) == 1
    assert L.moqe_route(P, P, 8, 64, 4, P, P, 0, P, P, 256, None) == 1
    assert L.moqe_route(P, P, -1, 64, 4, P, P, P, P, P, 256, None) == 3
    assert L.moqe_route(P, P, 8, 60, 4, P, P, P, P, P, 256, None) == 3
    assert L.moqe_route(P, P, 8, 64, 0, P, P, P, P, P, 256, None) == 3
    assert L.moqe_route(P, P, 8, 64, 2000, P, P, P, P, P, 256, None) == 3
    assert L.moqe_route(P, P + 2, 8, 64, 4, P, P, P, P, P, 256, None) == 4
    assert L.moqe_route(P, P, 8, 64, 4, P, P, P, P, P, 16, None) == 5
    assert L.moqe_route(P, P, 1 << 20, 64, 128, P, P, P, P, P, 256, None) == 5
    assert L.moqe_route_logits(0, 8, 4, P, P, P, P, P, 256, None) == 1
    assert L.moqe_route_logits(P, 8, 4, P, P, P, P, P, 0, None) == 5


def test_expert_ffn_error_paths():
    L = moqe.lib()

    def layer(**kw):
        base = dict(bits=4, E=4, d=64, f=256, codes1=P, scales1=P, bias1=P, codes2=P, scales2=P, bias2=P, codec=0)
        base.update(kw)
        return moqe.CLayer(*[base[k] for k, _ in moqe.CLayer._fields_])

    def call(lay, x=P, T=8, idx=P, gate=P, seg=P, perm=P, res=None, y=P, ws=P, wsb=1 << 24):
        return L.moqe_expert_ffn(ctypes.byref(lay) if lay is not None else None, x, T, idx, gate, seg, perm, res, y,
                                 ws, wsb, None)

    assert call(None) == 1
    assert call(layer(codes2=0)) == 1
    assert call(layer(), x=0) == 1
    assert call(layer(), y=0) == 1
    assert call(layer(bits=5)) == 2
    assert call(layer(codec=2)) == 2          # unknown codec
    assert call(layer(codec=1, bits=8)) == 2  # log-scale codes have 2, 3 or 4 bits
    assert call(layer(d=48)) == 3
    assert call(layer(E=0)) == 3
    assert call(layer(), T=-2) == 3
    assert call(layer(scales1=P + 8)) == 4
    assert call(layer(), res=P + 2) == 4
    assert call(layer(), wsb=1 << 20) == 5
    assert call(layer(), T=0) == 0          # no tokens: valid no-op, nothing launched

    def fused(lay, wg=P, x=P, T=8, idx=P, gate=P, seg=P, perm=P, res=None, y=P, ws=P, wsb=1 << 24):
        return L.moqe_moe_layer(ctypes.byref(lay) if lay is not None else None, wg, x, T, idx, gate, seg, perm, res,
                                y, ws, wsb, None)

    assert fused(None) == 1
    assert fused(layer(), wg=0) == 1
    assert fused(layer(), seg=0) == 1
    assert fused(layer(bits=5)) == 2
    assert fused(layer(f=100)) == 3
    assert fused(layer(), wg=P + 2) == 4
    assert fused(layer(), wsb=moqe.moqe_ffn_workspace_bytes(8, 4, 64, 256)) == 5   # route scratch missing
    # the same step on the library's own scratch: same checks, and sizes beyond the array refused
    def static(lay, wg=P, x=P, T=8, idx=P, gate=P, seg=P, perm=P, res=None, y=P):
        return L.moqe_moe_layer_static(ctypes.byref(lay) if lay is not None else None, wg, x, T, idx, gate, seg, perm,
                                       res, y, None)

    assert static(None) == 1
    assert static(layer(), perm=0) == 1
    assert static(layer(bits=7)) == 2
    assert static(layer(d=48)) == 3
    assert static(layer(), T=-1) == 3
    assert static(layer(), y=P + 2) == 4
    big = layer(E=32, d=1024, f=4096)
    assert moqe.moqe_layer_workspace_bytes(255, 32, 1024, 4096) <= moqe.STATIC_SCRATCH_BYTES
    assert moqe.moqe_layer_workspace_bytes(300, 32, 1024, 4096) > moqe.STATIC_SCRATCH_BYTES
    assert static(big, T=300) == 5
    assert static(big, T=4096) == 5
    assert L.moqe_expert_ffn1(ctypes.byref(layer()), P, 8, P, P, 0, None) == 1
    assert L.moqe_expert_ffn2(ctypes.byref(layer()), P, 8, P, P, P, None, P + 4, None) == 4


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(moqe, "_lib", None)
    monkeypatch.setattr(moqe, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        moqe.lib()
