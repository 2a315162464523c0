"""Thin ctypes binding of libmoqe.so (the C ABI in include/moqe.h).

Argument marshalling only: every step of the path runs in the HIP kernels.
PyTorch is used for device memory and the current stream, nothing else.  There
is no CPU fallback: if the library has not been built, loading fails loudly.
"""

from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libmoqe.so")

MOQE_OK = 0
STATUS_NAMES = ("MOQE_OK", "MOQE_ERR_NULL", "MOQE_ERR_BITS", "MOQE_ERR_SHAPE", "MOQE_ERR_ALIGN",
                "MOQE_ERR_WORKSPACE", "MOQE_ERR_HIP", "MOQE_ERR_TIMEOUT")

EXPORTS = (
    "moqe_status_string", "moqe_last_hip_error", "moqe_version", "moqe_packed_bytes",
    "moqe_check_matrix", "moqe_check_layer", "moqe_route_workspace_bytes",
    "moqe_ffn_workspace_bytes", "moqe_quantize", "moqe_unpack", "moqe_route",
    "moqe_route_logits", "moqe_expert_ffn", "moqe_expert_ffn1", "moqe_expert_ffn2",
    "moqe_layer_workspace_bytes", "moqe_moe_layer", "moqe_set_launch_mode",
    "moqe_set_prefill_policy", "moqe_quantize_tensor_scale", "moqe_quantize_log", "moqe_dequantize_log",
    "moqe_moe_layer_static", "moqe_set_decode_kernel", "moqe_workspace_status",
    "moqe_stream_read", "moqe_set_tiled_kernel", "moqe_contraction_path",
)

LAUNCH_AUTO, LAUNCH_SEPARATE, LAUNCH_FUSED = 0, 1, 2
CODEC_LINEAR, CODEC_LOG = 0, 1


class MoqeError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().moqe_status_string(status).decode()
        if status == 6:
            msg += " (" + lib().moqe_last_hip_error().decode() + ")"
        super().__init__(f"{where}: {msg}")


class CLayer(ctypes.Structure):
    """moqe_layer of include/moqe.h."""
    _fields_ = [("bits", ctypes.c_int), ("E", ctypes.c_int64), ("d", ctypes.c_int64), ("f", ctypes.c_int64),
                ("codes1", ctypes.c_void_p), ("scales1", ctypes.c_void_p), ("bias1", ctypes.c_void_p),
                ("codes2", ctypes.c_void_p), ("scales2", ctypes.c_void_p), ("bias2", ctypes.c_void_p),
                ("codec", ctypes.c_int)]


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library; raises if it was never built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it first (python -m paper_2310_02410_amd.build, or "
            "__graft_entry__.build()). There is no fallback path.")
    L = ctypes.CDLL(LIB_PATH)
    vp, i64, sz, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_size_t, ctypes.c_int
    L.moqe_status_string.restype = ctypes.c_char_p
    L.moqe_status_string.argtypes = [ci]
    L.moqe_last_hip_error.restype = ctypes.c_char_p
    L.moqe_last_hip_error.argtypes = []
    L.moqe_version.restype = ci
    L.moqe_set_launch_mode.restype = ci
    L.moqe_set_launch_mode.argtypes = [ci]
    L.moqe_stream_read.restype = ci
    L.moqe_stream_read.argtypes = [vp, sz, vp, vp]
    L.moqe_workspace_status.restype = ci
    L.moqe_workspace_status.argtypes = [vp, sz, vp]
    L.moqe_set_decode_kernel.restype = ci
    L.moqe_set_decode_kernel.argtypes = [ci]
    L.moqe_set_tiled_kernel.restype = ci
    L.moqe_set_tiled_kernel.argtypes = [ci]
    L.moqe_set_prefill_policy.restype = ci
    L.moqe_set_prefill_policy.argtypes = [ci, ci, ci]
    L.moqe_contraction_path.restype = ci
    L.moqe_contraction_path.argtypes = [ci, i64, i64, i64, i64]
    L.moqe_packed_bytes.restype = sz
    L.moqe_packed_bytes.argtypes = [ci, i64, i64]
    L.moqe_check_matrix.restype = ci
    L.moqe_check_matrix.argtypes = [ci, i64, i64]
    L.moqe_check_layer.restype = ci
    L.moqe_check_layer.argtypes = [ci, i64, i64, i64]
    L.moqe_route_workspace_bytes.restype = sz
    L.moqe_route_workspace_bytes.argtypes = [i64, i64]
    L.moqe_ffn_workspace_bytes.restype = sz
    L.moqe_ffn_workspace_bytes.argtypes = [i64, i64, i64, i64]
    L.moqe_layer_workspace_bytes.restype = sz
    L.moqe_layer_workspace_bytes.argtypes = [i64, i64, i64, i64]
    L.moqe_moe_layer.restype = ci
    L.moqe_moe_layer.argtypes = [ctypes.POINTER(CLayer), vp, vp, i64, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.moqe_moe_layer_static.restype = ci
    L.moqe_moe_layer_static.argtypes = [ctypes.POINTER(CLayer), vp, vp, i64, vp, vp, vp, vp, vp, vp, vp]
    L.moqe_quantize.restype = ci
    L.moqe_quantize.argtypes = [vp, i64, i64, i64, ci, vp, vp, vp]
    L.moqe_quantize_tensor_scale.restype = ci
    L.moqe_quantize_tensor_scale.argtypes = [vp, i64, i64, i64, ci, vp, vp, vp]
    L.moqe_quantize_log.restype = ci
    L.moqe_quantize_log.argtypes = [vp, i64, i64, i64, ci, vp, vp, vp]
    L.moqe_dequantize_log.restype = ci
    L.moqe_dequantize_log.argtypes = [vp, vp, i64, i64, i64, ci, vp, vp]
    L.moqe_unpack.restype = ci
    L.moqe_unpack.argtypes = [vp, i64, i64, i64, ci, vp, vp]
    L.moqe_route.restype = ci
    L.moqe_route.argtypes = [vp, vp, i64, i64, i64, vp, vp, vp, vp, vp, sz, vp]
    L.moqe_route_logits.restype = ci
    L.moqe_route_logits.argtypes = [vp, i64, i64, vp, vp, vp, vp, vp, sz, vp]
    L.moqe_expert_ffn.restype = ci
    L.moqe_expert_ffn.argtypes = [ctypes.POINTER(CLayer), vp, i64, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.moqe_expert_ffn1.restype = ci
    L.moqe_expert_ffn1.argtypes = [ctypes.POINTER(CLayer), vp, i64, vp, vp, vp, vp]
    L.moqe_expert_ffn2.restype = ci
    L.moqe_expert_ffn2.argtypes = [ctypes.POINTER(CLayer), vp, i64, vp, vp, vp, vp, vp, vp]
    _lib = L
    return L


def _check(status: int, where: str) -> None:
    if status != MOQE_OK:
        raise MoqeError(status, where)


def _stream(stream=None) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def _ptr(t) -> int:
    return 0 if t is None else t.data_ptr()


def _dev(t: torch.Tensor, dtype, name: str) -> torch.Tensor:
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous {dtype} device tensor")
    return t


# ---------------------------------------------------------------------------
# pure host queries
# ---------------------------------------------------------------------------

def moqe_packed_bytes(bits: int, K: int, N: int) -> int:
    return lib().moqe_packed_bytes(bits, K, N)


def moqe_route_workspace_bytes(T: int, E: int) -> int:
    return lib().moqe_route_workspace_bytes(T, E)


def moqe_ffn_workspace_bytes(T: int, E: int, d: int, f: int) -> int:
    return lib().moqe_ffn_workspace_bytes(T, E, d, f)


def moqe_layer_workspace_bytes(T: int, E: int, d: int, f: int) -> int:
    return lib().moqe_layer_workspace_bytes(T, E, d, f)


def moqe_set_launch_mode(mode: int) -> int:
    """Process-wide launch policy (LAUNCH_AUTO / LAUNCH_SEPARATE / LAUNCH_FUSED); returns the old one."""
    old = lib().moqe_set_launch_mode(mode)
    if old < 0:
        raise ValueError(f"unknown launch mode {mode}")
    return old


DECODE_AUTO, DECODE_GENERAL, DECODE_ROWS8, DECODE_ROWS4 = 0, 1, 2, 3


def moqe_set_decode_kernel(which: int) -> int:
    """Process-wide: DECODE_AUTO (the kernel specialised for decode-sized batches where it applies:
    pairs of 4 token rows up to 32 tokens, of 8 from 33 on, up to 64 tokens and, in pairs of 8, up
    to 128), DECODE_GENERAL (always the
    general decode kernel), DECODE_ROWS8 / DECODE_ROWS4 (AUTO with 8 / 4 rows at every size);
    returns the old setting."""
    old = lib().moqe_set_decode_kernel(which)
    if old < 0:
        raise ValueError(f"unknown decode kernel choice {which}")
    return old


TILED_AUTO, TILED_STREAMED, TILED_RESIDENT = 0, 1, 2


def moqe_set_tiled_kernel(which: int) -> int:
    """Process-wide: TILED_AUTO (token rows resident in LDS where 64 fit, K <= 1024, and in tiles
    of 16 up to K = 4096 while T <= 16 E), TILED_STREAMED (always K staged in blocks) or
    TILED_RESIDENT (resident wherever it applies); returns the old setting."""
    old = lib().moqe_set_tiled_kernel(which)
    if old < 0:
        raise ValueError(f"unknown tiled kernel choice {which}")
    return old


PREFILL_MIN_SEGMENT_DEFAULT, PREFILL_MIN_BATCH_DEFAULT, PREFILL_ALL_TILED_DEFAULT = 0x40000000, 65, 2
PREFILL_NEVER = 2**31 - 1  # as all_tiled_tokens_per_expert: keep the decode kernel for small segments


def moqe_set_prefill_policy(min_segment_tokens: int = PREFILL_MIN_SEGMENT_DEFAULT,
                            min_batch_tokens: int = PREFILL_MIN_BATCH_DEFAULT,
                            all_tiled_tokens_per_expert: int = PREFILL_ALL_TILED_DEFAULT) -> None:
    """Process-wide path choice: in batches of at least min_batch_tokens, expert segments with at
    least min_segment_tokens tokens take the tiled MFMA kernel; with at least
    all_tiled_tokens_per_expert tokens per expert on average, all segments do.  No arguments:
    the defaults."""
    if lib().moqe_set_prefill_policy(min_segment_tokens, min_batch_tokens, all_tiled_tokens_per_expert) != 0:
        raise ValueError("thresholds must be >= 1")


PATH_DECODE_SMALL, PATH_DECODE, PATH_TILED_RESIDENT, PATH_TILED_STAGED = 1, 2, 4, 8


def moqe_contraction_path(bits: int, T: int, E: int, K: int, N: int) -> int:
    """Which kernels one contraction over [K, N] expert matrices launches under the current
    settings: a sum of PATH_* values (host only, launches nothing)."""
    m = lib().moqe_contraction_path(bits, T, E, K, N)
    if m < 0:
        raise ValueError(f"the expert FFN does not take bits={bits} T={T} E={E} K={K} N={N}")
    return m


def alloc_workspace(nbytes: int, device) -> torch.Tensor:
    """FFN / layer scratch: its head holds the inter-phase counters and must start zeroed."""
    return torch.zeros(nbytes, dtype=torch.uint8, device=device)


# ---------------------------------------------------------------------------
# the three calls
# ---------------------------------------------------------------------------

def moqe_quantize(w: torch.Tensor, bits: int, stream=None, tensor_scale: bool = False):
    """w fp32 [E,K,N] -> (codes uint8 [E, K*N*bits/8], scales fp16 [E,N]); tensor_scale: one scale
    per matrix instead of one per channel."""
    _dev(w, torch.float32, "w")
    E, K, N = w.shape
    nbytes = moqe_packed_bytes(bits, K, N)
    if nbytes == 0:
        _check(lib().moqe_check_matrix(bits, K, N) or 3, "moqe_quantize")
    codes = torch.empty((E, nbytes), dtype=torch.uint8, device=w.device)
    scales = torch.empty((E, N), dtype=torch.float16, device=w.device)
    fn = lib().moqe_quantize_tensor_scale if tensor_scale else lib().moqe_quantize
    _check(fn(w.data_ptr(), E, K, N, bits, codes.data_ptr(), scales.data_ptr(), _stream(stream)), "moqe_quantize")
    return codes, scales


def moqe_quantize_log(w: torch.Tensor, bits: int, stream=None):
    """Log-scale codec: w fp32 [E,K,N] -> (codes uint8 [E, K*N*bits/8], scales fp16 [E,N]); bits 2, 3 or 4."""
    _dev(w, torch.float32, "w")
    E, K, N = w.shape
    nbytes = moqe_packed_bytes(bits, K, N)
    if nbytes == 0:
        _check(lib().moqe_check_matrix(bits, K, N) or 3, "moqe_quantize_log")
    codes = torch.empty((E, nbytes), dtype=torch.uint8, device=w.device)
    scales = torch.empty((E, N), dtype=torch.float16, device=w.device)
    _check(lib().moqe_quantize_log(w.data_ptr(), E, K, N, bits, codes.data_ptr(), scales.data_ptr(), _stream(stream)),
           "moqe_quantize_log")
    return codes, scales


def moqe_dequantize_log(codes: torch.Tensor, scales: torch.Tensor, bits: int, K: int, N: int, stream=None) -> torch.Tensor:
    """Log-scale codes -> fp32 [E,K,N], A' = P s 2^Q (exact)."""
    _dev(codes, torch.uint8, "codes")
    _dev(scales, torch.float16, "scales")
    E = codes.shape[0]
    w = torch.empty((E, K, N), dtype=torch.float32, device=codes.device)
    _check(lib().moqe_dequantize_log(codes.data_ptr(), scales.data_ptr(), E, K, N, bits, w.data_ptr(), _stream(stream)),
           "moqe_dequantize_log")
    return w


def moqe_unpack(codes: torch.Tensor, bits: int, K: int, N: int, stream=None) -> torch.Tensor:
    """codes uint8 [E, K*N*bits/8] -> int8 [E,K,N]."""
    _dev(codes, torch.uint8, "codes")
    E = codes.shape[0]
    q = torch.empty((E, K, N), dtype=torch.int8, device=codes.device)
    _check(lib().moqe_unpack(codes.data_ptr(), E, K, N, bits, q.data_ptr(), _stream(stream)), "moqe_unpack")
    return q


@dataclass
class Route:
    expert_idx: torch.Tensor   # int32 [T]
    gate: torch.Tensor         # fp32 [T]
    seg_offsets: torch.Tensor  # int32 [E+1]
    perm: torch.Tensor         # int32 [T]


def alloc_route(T: int, E: int, device) -> tuple:
    r = Route(torch.empty(max(T, 1), dtype=torch.int32, device=device)[:T],
              torch.empty(max(T, 1), dtype=torch.float32, device=device)[:T],
              torch.empty(E + 1, dtype=torch.int32, device=device),
              torch.empty(max(T, 1), dtype=torch.int32, device=device)[:T])
    ws = torch.empty(moqe_route_workspace_bytes(T, E), dtype=torch.uint8, device=device)
    return r, ws


def moqe_route(x: torch.Tensor, w_gate: torch.Tensor, out: Route = None, workspace=None, stream=None) -> Route:
    """Top-1 gating of x fp16 [T,d] with w_gate fp16 [d,E]."""
    _dev(x, torch.float16, "x")
    _dev(w_gate, torch.float16, "w_gate")
    T, d = x.shape
    E = w_gate.shape[1]
    if out is None or workspace is None:
        out, workspace = alloc_route(T, E, x.device)
    _check(lib().moqe_route(x.data_ptr(), w_gate.data_ptr(), T, d, E, out.expert_idx.data_ptr(),
                            out.gate.data_ptr(), out.seg_offsets.data_ptr(), out.perm.data_ptr(),
                            workspace.data_ptr(), workspace.numel(), _stream(stream)), "moqe_route")
    return out


def moqe_route_logits(logits: torch.Tensor, out: Route = None, workspace=None, stream=None) -> Route:
    """Top-1 gating from given fp32 logits [T,E]."""
    _dev(logits, torch.float32, "logits")
    T, E = logits.shape
    if out is None or workspace is None:
        out, workspace = alloc_route(T, E, logits.device)
    _check(lib().moqe_route_logits(logits.data_ptr(), T, E, out.expert_idx.data_ptr(), out.gate.data_ptr(),
                                   out.seg_offsets.data_ptr(), out.perm.data_ptr(), workspace.data_ptr(),
                                   workspace.numel(), _stream(stream)), "moqe_route_logits")
    return out


@dataclass
class QuantLayer:
    """Device buffers of one quantized MoE layer plus its moqe_layer struct."""
    bits: int
    E: int
    d: int
    f: int
    codes1: torch.Tensor
    scales1: torch.Tensor
    bias1: torch.Tensor
    codes2: torch.Tensor
    scales2: torch.Tensor
    bias2: torch.Tensor
    w_gate: torch.Tensor = None
    codec: int = CODEC_LINEAR

    def c_struct(self) -> CLayer:
        return CLayer(self.bits, self.E, self.d, self.f, self.codes1.data_ptr(), self.scales1.data_ptr(),
                      self.bias1.data_ptr(), self.codes2.data_ptr(), self.scales2.data_ptr(),
                      self.bias2.data_ptr(), self.codec)

    def code_bytes(self) -> int:
        return self.codes1.numel() + self.codes2.numel()


def quantize_layer(w1: torch.Tensor, b1: torch.Tensor, w2: torch.Tensor, b2: torch.Tensor, bits: int,
                   w_gate: torch.Tensor = None, codec: int = CODEC_LINEAR) -> QuantLayer:
    """Quantize fp32 w1 [E,d,f], w2 [E,f,d] on the device; biases fp16 [E,f], [E,d]."""
    E, d, f = w1.shape
    _check(lib().moqe_check_layer(bits, E, d, f), "quantize_layer")
    quant = moqe_quantize_log if codec == CODEC_LOG else moqe_quantize
    c1, s1 = quant(w1, bits)
    c2, s2 = quant(w2, bits)
    return QuantLayer(bits, E, d, f, c1, s1, _dev(b1, torch.float16, "b1"), c2, s2,
                      _dev(b2, torch.float16, "b2"), w_gate, codec)


def moqe_expert_ffn(layer: QuantLayer, x: torch.Tensor, route: Route, residual: torch.Tensor = None,
                    out: torch.Tensor = None, workspace: torch.Tensor = None, stream=None) -> torch.Tensor:
    """FFN1 + bias + ReLU, FFN2 + bias, gate-weighted combine (+ residual) -> fp16 [T,d]."""
    _dev(x, torch.float16, "x")
    T, d = x.shape
    if d != layer.d:
        raise ValueError("x has the wrong width")
    if out is None:
        out = torch.empty_like(x)
    if workspace is None:
        workspace = alloc_workspace(moqe_ffn_workspace_bytes(T, layer.E, layer.d, layer.f), x.device)
    cl = layer.c_struct()
    _check(lib().moqe_expert_ffn(ctypes.byref(cl), x.data_ptr(), T, _ptr(route.expert_idx), _ptr(route.gate),
                                 route.seg_offsets.data_ptr(), _ptr(route.perm), _ptr(residual), out.data_ptr(),
                                 workspace.data_ptr(), workspace.numel(), _stream(stream)), "moqe_expert_ffn")
    return out


def moqe_expert_ffn1(layer: QuantLayer, x: torch.Tensor, route: Route, h: torch.Tensor, stream=None) -> torch.Tensor:
    """h = relu(x W1' + b1) into fp16 [T,f], rows in sorted-token order."""
    cl = layer.c_struct()
    _check(lib().moqe_expert_ffn1(ctypes.byref(cl), x.data_ptr(), x.shape[0], route.seg_offsets.data_ptr(),
                                  _ptr(route.perm), h.data_ptr(), _stream(stream)), "moqe_expert_ffn1")
    return h


def moqe_expert_ffn2(layer: QuantLayer, h: torch.Tensor, route: Route, out: torch.Tensor,
                     residual: torch.Tensor = None, stream=None) -> torch.Tensor:
    """y_t = gate_t (h W2' + b2) (+ residual) into fp16 [T,d], token order."""
    cl = layer.c_struct()
    _check(lib().moqe_expert_ffn2(ctypes.byref(cl), h.data_ptr(), h.shape[0], _ptr(route.gate),
                                  route.seg_offsets.data_ptr(), _ptr(route.perm), _ptr(residual), out.data_ptr(),
                                  _stream(stream)), "moqe_expert_ffn2")
    return out


def moqe_moe_layer(layer: QuantLayer, x: torch.Tensor, residual: torch.Tensor = None, out: torch.Tensor = None,
                   route: Route = None, workspace: torch.Tensor = None, stream=None):
    """Route with layer.w_gate, then the expert FFN: one call (one launch for decode-sized
    batches).  Returns (y fp16 [T,d], Route)."""
    _dev(x, torch.float16, "x")
    T, d = x.shape
    if layer.w_gate is None:
        raise ValueError("layer has no router weights")
    if out is None:
        out = torch.empty_like(x)
    if route is None:
        route, _ = alloc_route(T, layer.E, x.device)
    if workspace is None:
        workspace = alloc_workspace(moqe_layer_workspace_bytes(T, layer.E, layer.d, layer.f), x.device)
    cl = layer.c_struct()
    _check(lib().moqe_moe_layer(ctypes.byref(cl), layer.w_gate.data_ptr(), x.data_ptr(), T, _ptr(route.expert_idx),
                                _ptr(route.gate), route.seg_offsets.data_ptr(), _ptr(route.perm), _ptr(residual),
                                out.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream(stream)),
           "moqe_moe_layer")
    return out, route


STATIC_SCRATCH_BYTES = 4 << 20  # MOQE_STATIC_SCRATCH_BYTES of include/moqe.h


def moqe_moe_layer_static(layer: QuantLayer, x: torch.Tensor, out: torch.Tensor, route: Route,
                          residual: torch.Tensor = None, stream=None):
    """moqe_moe_layer on the library's own scratch: the call itself allocates nothing, so the
    caller brings every output (out fp16 [T,d], route)."""
    _dev(x, torch.float16, "x")
    if layer.w_gate is None:
        raise ValueError("layer has no router weights")
    cl = layer.c_struct()
    _check(lib().moqe_moe_layer_static(ctypes.byref(cl), layer.w_gate.data_ptr(), x.data_ptr(), x.shape[0],
                                       _ptr(route.expert_idx), _ptr(route.gate), route.seg_offsets.data_ptr(),
                                       _ptr(route.perm), _ptr(residual), out.data_ptr(), _stream(stream)),
           "moqe_moe_layer_static")
    return out, route


def workspace_error(workspace: torch.Tensor, stream=None) -> bool:
    """True if a wait of a single-launch (FUSED) step using this FFN / layer scratch has timed out
    (moqe_workspace_status; synchronises the stream)."""
    st = lib().moqe_workspace_status(workspace.data_ptr(), workspace.numel(), _stream(stream))
    if st not in (0, 7):
        raise MoqeError(st, "moqe_workspace_status")
    return st == 7
