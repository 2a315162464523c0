// C ABI of the MoQE hot path: argument validation on the host, then launches.
// Every error is detected before the first launch, so the error paths can be
// exercised without a GPU.
#include <limits.h>
#include <stdio.h>
#include <string.h>

#include "../../include/moqe.h"
#include "moqe_dev.h"
#include "moqe_kernels.h"

namespace {

thread_local char g_hip_error[256] = "no error";

moqe_status hip_fail(hipError_t e) {
  snprintf(g_hip_error, sizeof(g_hip_error), "%s: %s", hipGetErrorName(e), hipGetErrorString(e));
  return MOQE_ERR_HIP;
}

bool aligned16(const void* p) { return (((uintptr_t)p) & 15u) == 0; }

int num_cus() {
  // Compute units of the current device; cached per device id.
  static int cache[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  if (cache[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    cache[dev] = n;
  }
  return cache[dev];
}

#ifdef MOQE_PHASE_TRACE
long long* g_trace = nullptr;  // debug builds only: set through moqe_debug_set_trace
#endif

constexpr int64_t MAX_TOKENS = 1 << 22;
constexpr int64_t MAX_EXPERTS = 1024;

size_t round256(size_t b) { return b < 256 ? 256 : ((b + 255) & ~(size_t)255); }

}  // namespace

extern "C" {

const char* moqe_status_string(int status) {
  switch (status) {
    case MOQE_OK: return "MOQE_OK";
    case MOQE_ERR_NULL: return "MOQE_ERR_NULL: required pointer is NULL";
    case MOQE_ERR_BITS: return "MOQE_ERR_BITS: bits must be 2, 3 or 4";
    case MOQE_ERR_SHAPE: return "MOQE_ERR_SHAPE: unsupported dimension";
    case MOQE_ERR_ALIGN: return "MOQE_ERR_ALIGN: device pointer not 16-byte aligned";
    case MOQE_ERR_WORKSPACE: return "MOQE_ERR_WORKSPACE: workspace too small";
    case MOQE_ERR_HIP: return "MOQE_ERR_HIP: HIP runtime error";
    default: return "unknown status";
  }
}

const char* moqe_last_hip_error(void) { return g_hip_error; }

int moqe_version(void) { return 1; }

#ifdef MOQE_PHASE_TRACE
void moqe_debug_set_trace(long long* p) { g_trace = p; }
#endif

int moqe_check_matrix(int bits, int64_t K, int64_t N) {
  if (bits != 2 && bits != 3 && bits != 4) return MOQE_ERR_BITS;
  PackGeom g;
  return moqe_make_geom(bits, K, N, &g) ? MOQE_OK : MOQE_ERR_SHAPE;
}

size_t moqe_packed_bytes(int bits, int64_t K, int64_t N) {
  PackGeom g;
  if (!moqe_make_geom(bits, K, N, &g)) return 0;
  return (size_t)g.matrix_bytes;
}

int moqe_check_layer(int bits, int64_t E, int64_t d, int64_t f) {
  if (bits != 2 && bits != 3 && bits != 4) return MOQE_ERR_BITS;
  if (E < 1 || E > MAX_EXPERTS) return MOQE_ERR_SHAPE;
  int ks, r;
  if (moqe_check_matrix(bits, d, f) != MOQE_OK || moqe_check_matrix(bits, f, d) != MOQE_OK) return MOQE_ERR_SHAPE;
  if (!moqe_pick_ksplit(bits, d, &ks, &r) || !moqe_pick_ksplit(bits, f, &ks, &r)) return MOQE_ERR_SHAPE;
  return MOQE_OK;
}

size_t moqe_route_workspace_bytes(int64_t T, int64_t E) {
  if (T < 0 || E < 1) return 256;
  return moqe_route_ws_bytes(T, E);
}

size_t moqe_ffn_workspace_bytes(int64_t T, int64_t E, int64_t d, int64_t f) {
  (void)E;
  (void)d;
  if (T < 0 || f < 0) return 256;
  return round256((size_t)T * (size_t)f * 2);  // h: fp16 [T, f] in sorted-token order
}

moqe_status moqe_quantize(const float* w, int64_t E, int64_t K, int64_t N, int bits, void* codes_out,
                          moqe_f16* scales_out, void* stream) {
  if (!w || !codes_out || !scales_out) return MOQE_ERR_NULL;
  if (bits != 2 && bits != 3 && bits != 4) return MOQE_ERR_BITS;
  PackGeom g;
  if (E < 1 || E > MAX_EXPERTS || !moqe_make_geom(bits, K, N, &g)) return MOQE_ERR_SHAPE;
  if (!aligned16(w) || !aligned16(codes_out) || !aligned16(scales_out)) return MOQE_ERR_ALIGN;
  hipError_t e = moqe_launch_quantize(w, E, g, codes_out, scales_out, (hipStream_t)stream);
  return e == hipSuccess ? MOQE_OK : hip_fail(e);
}

moqe_status moqe_unpack(const void* codes, int64_t E, int64_t K, int64_t N, int bits, int8_t* q_out, void* stream) {
  if (!codes || !q_out) return MOQE_ERR_NULL;
  if (bits != 2 && bits != 3 && bits != 4) return MOQE_ERR_BITS;
  PackGeom g;
  if (E < 1 || E > MAX_EXPERTS || !moqe_make_geom(bits, K, N, &g)) return MOQE_ERR_SHAPE;
  if (!aligned16(codes) || !aligned16(q_out)) return MOQE_ERR_ALIGN;
  hipError_t e = moqe_launch_unpack(codes, E, g, q_out, (hipStream_t)stream);
  return e == hipSuccess ? MOQE_OK : hip_fail(e);
}

static moqe_status route_common(const moqe_f16* x, const moqe_f16* w_gate, const float* logits, int64_t T, int64_t d,
                                int64_t E, int32_t* expert_idx, float* gate, int32_t* seg_offsets, int32_t* perm,
                                void* workspace, size_t workspace_bytes, void* stream) {
  if (!seg_offsets || !workspace) return MOQE_ERR_NULL;
  if (T > 0 && (!expert_idx || !gate || !perm)) return MOQE_ERR_NULL;  // per-token arrays may be NULL when T = 0
  if (T < 0 || T > MAX_TOKENS || E < 1 || E > MAX_EXPERTS) return MOQE_ERR_SHAPE;
  if (!logits) {
    if (d < 8 || (d % 8) || d > 16384) return MOQE_ERR_SHAPE;
    // the 8-token score kernel stages its rows in LDS
    if (T >= 2048 && (size_t)8 * d * 2 + 256 * 8 * 4 + (size_t)8 * E * 4 > 64 * 1024) return MOQE_ERR_SHAPE;
  }
  if (!aligned16(expert_idx) || !aligned16(gate) || !aligned16(seg_offsets) || !aligned16(perm) ||
      !aligned16(workspace) || (x && !aligned16(x)) || (w_gate && !aligned16(w_gate)) ||
      (logits && !aligned16(logits)))
    return MOQE_ERR_ALIGN;
  if (workspace_bytes < moqe_route_ws_bytes(T, E)) return MOQE_ERR_WORKSPACE;
  hipError_t e = moqe_launch_route(x, w_gate, logits, (int)T, (int)d, (int)E, expert_idx, gate, seg_offsets, perm,
                                   workspace, (hipStream_t)stream);
  return e == hipSuccess ? MOQE_OK : hip_fail(e);
}

moqe_status moqe_route(const moqe_f16* x, const moqe_f16* w_gate, int64_t T, int64_t d, int64_t E, int32_t* expert_idx,
                       float* gate, int32_t* seg_offsets, int32_t* perm, void* workspace, size_t workspace_bytes,
                       void* stream) {
  if (!w_gate || (!x && T > 0)) return MOQE_ERR_NULL;
  return route_common(x, w_gate, nullptr, T, d, E, expert_idx, gate, seg_offsets, perm, workspace, workspace_bytes,
                      stream);
}

moqe_status moqe_route_logits(const float* logits, int64_t T, int64_t E, int32_t* expert_idx, float* gate,
                              int32_t* seg_offsets, int32_t* perm, void* workspace, size_t workspace_bytes,
                              void* stream) {
  if (!logits) return MOQE_ERR_NULL;
  return route_common(nullptr, nullptr, logits, T, 0, E, expert_idx, gate, seg_offsets, perm, workspace,
                      workspace_bytes, stream);
}

static moqe_status check_layer_ptrs(const moqe_layer* L) {
  if (!L) return MOQE_ERR_NULL;
  if (!L->codes1 || !L->scales1 || !L->bias1 || !L->codes2 || !L->scales2 || !L->bias2) return MOQE_ERR_NULL;
  if (L->bits != 2 && L->bits != 3 && L->bits != 4) return MOQE_ERR_BITS;
  int st = moqe_check_layer(L->bits, L->E, L->d, L->f);
  if (st != MOQE_OK) return (moqe_status)st;
  if (!aligned16(L->codes1) || !aligned16(L->scales1) || !aligned16(L->bias1) || !aligned16(L->codes2) ||
      !aligned16(L->scales2) || !aligned16(L->bias2))
    return MOQE_ERR_ALIGN;
  return MOQE_OK;
}

static void base_args(FfnArgs* a, const moqe_layer* L, int64_t T, const int32_t* seg_offsets, const int32_t* perm) {
  memset(a, 0, sizeof(*a));
  a->bits = L->bits;
  a->E = (int)L->E;
  a->seg_offsets = seg_offsets;
  a->perm = perm;
  a->T = (int)T;
  a->min_tokens = 1;
  a->max_tokens = INT_MAX;
#ifdef MOQE_PHASE_TRACE
  a->trace = g_trace;
#endif
}

moqe_status moqe_expert_ffn1(const moqe_layer* L, const moqe_f16* x, int64_t T, const int32_t* seg_offsets,
                             const int32_t* perm, moqe_f16* h, void* stream) {
  if (!L || !x || !seg_offsets || !perm || !h) return MOQE_ERR_NULL;
  moqe_status st = check_layer_ptrs(L);
  if (st != MOQE_OK) return st;
  if (T < 0 || T > MAX_TOKENS) return MOQE_ERR_SHAPE;
  if (!aligned16(x) || !aligned16(seg_offsets) || !aligned16(perm) || !aligned16(h)) return MOQE_ERR_ALIGN;
  if (T == 0) return MOQE_OK;
  FfnArgs a;
  base_args(&a, L, T, seg_offsets, perm);
  a.codes = (const uint32_t*)L->codes1;
  a.scales = L->scales1;
  a.bias = L->bias1;
  a.K = (int)L->d;
  a.N = (int)L->f;
  moqe_pick_ksplit(a.bits, a.K, &a.ksteps, &a.ksplit);
  a.a = x;
  a.h_out = h;
  a.mode = 0;
  hipError_t e = moqe_launch_ffn_decode(a, num_cus(), (hipStream_t)stream);
  return e == hipSuccess ? MOQE_OK : hip_fail(e);
}

moqe_status moqe_expert_ffn2(const moqe_layer* L, const moqe_f16* h, int64_t T, const float* gate,
                             const int32_t* seg_offsets, const int32_t* perm, const moqe_f16* residual, moqe_f16* y,
                             void* stream) {
  if (!L || !h || !gate || !seg_offsets || !perm || !y) return MOQE_ERR_NULL;
  moqe_status st = check_layer_ptrs(L);
  if (st != MOQE_OK) return st;
  if (T < 0 || T > MAX_TOKENS) return MOQE_ERR_SHAPE;
  if (!aligned16(h) || !aligned16(gate) || !aligned16(seg_offsets) || !aligned16(perm) || !aligned16(y) ||
      (residual && !aligned16(residual)))
    return MOQE_ERR_ALIGN;
  if (T == 0) return MOQE_OK;
  FfnArgs a;
  base_args(&a, L, T, seg_offsets, perm);
  a.gate = gate;
  a.codes = (const uint32_t*)L->codes2;
  a.scales = L->scales2;
  a.bias = L->bias2;
  a.K = (int)L->f;
  a.N = (int)L->d;
  moqe_pick_ksplit(a.bits, a.K, &a.ksteps, &a.ksplit);
  a.a = h;
  a.y_out = y;
  a.residual = residual;
  a.mode = 1;
  hipError_t e = moqe_launch_ffn_decode(a, num_cus(), (hipStream_t)stream);
  return e == hipSuccess ? MOQE_OK : hip_fail(e);
}

moqe_status moqe_expert_ffn(const moqe_layer* L, const moqe_f16* x, int64_t T, const int32_t* expert_idx,
                            const float* gate, const int32_t* seg_offsets, const int32_t* perm,
                            const moqe_f16* residual, moqe_f16* y, void* workspace, size_t workspace_bytes,
                            void* stream) {
  if (!L || !x || !expert_idx || !gate || !seg_offsets || !perm || !y || !workspace) return MOQE_ERR_NULL;
  moqe_status st = check_layer_ptrs(L);
  if (st != MOQE_OK) return st;
  if (T < 0 || T > MAX_TOKENS) return MOQE_ERR_SHAPE;
  if (!aligned16(x) || !aligned16(expert_idx) || !aligned16(gate) || !aligned16(seg_offsets) || !aligned16(perm) ||
      !aligned16(y) || !aligned16(workspace) || (residual && !aligned16(residual)))
    return MOQE_ERR_ALIGN;
  if (workspace_bytes < moqe_ffn_workspace_bytes(T, L->E, L->d, L->f)) return MOQE_ERR_WORKSPACE;
  if (T == 0) return MOQE_OK;
  // FFN1: h = relu(x W1' + b1), rows in sorted-token order (the workspace)
  st = moqe_expert_ffn1(L, x, T, seg_offsets, perm, (moqe_f16*)workspace, stream);
  if (st != MOQE_OK) return st;
  // FFN2 + bias, gate-weighted combine (+ residual), scattered back to token order
  return moqe_expert_ffn2(L, (const moqe_f16*)workspace, T, gate, seg_offsets, perm, residual, y, stream);
}

}  // extern "C"
