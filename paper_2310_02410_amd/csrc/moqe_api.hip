// C ABI of the MoQE hot path: argument validation on the host, then launches.
// Every error is detected before the first launch, so the error paths can be
// exercised without a GPU.
#include <limits.h>
#include <atomic>
#include <mutex>
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


constexpr int64_t MAX_TOKENS = 1 << 22;
constexpr int64_t MAX_EXPERTS = 1024;

size_t round256(size_t b) { return b < 256 ? 256 : ((b + 255) & ~(size_t)255); }

std::atomic<int> g_launch_mode{MOQE_LAUNCH_AUTO};
// Expert segments with at least this many tokens go to the tiled MFMA kernel.  The decode
// kernel re-streams an expert's weights once per 4 tokens; from a handful of such passes on,
// one pass of the tiled kernel (64-token tiles) is cheaper.
std::atomic<int> g_prefill_min{MOQE_PREFILL_MIN_SEGMENT_DEFAULT};
std::atomic<int> g_prefill_batch{MOQE_PREFILL_MIN_BATCH_DEFAULT};
std::atomic<int> g_prefill_all{MOQE_PREFILL_ALL_TILED_DEFAULT};
// Decode-sized batches take the lean decode kernel where it applies (moqe_set_decode_kernel).
// 0: general kernel always; 1: the decode-sized kernel where it applies, with pairs of 8 token
// rows from ROWS8_FROM_TOKENS tokens on; 2: the same with pairs of 8 rows at every size; 3: with
// pairs of 4 rows at every size
std::atomic<int> g_small_decode{1};
// Measured on the benchmark layer (E = 32, d = 1024, f = 4096), per step: pairs of 8 rows against
// pairs of 4 at 24 tokens 25.5 / 28.2 / 22.9 us against 25.9 / 27.5 / 22.1 (int4 / int3 / int2: the
// kernels are faster back to back, the step is not), at 64 tokens 33.6 against 35.1 us under
// uniform and 30.4 against 34.1 us under Zipf load (an expert's weights streamed once per 8
// instead of once per 4 of its tokens).
constexpr int ROWS8_FROM_TOKENS = 33;
// Which tiled kernel serves the many-token segments (moqe_set_tiled_kernel).
std::atomic<int> g_tiled_kernel{MOQE_TILED_AUTO};

}  // namespace

extern "C" {

const char* moqe_status_string(int status) {
  switch (status) {
    case MOQE_OK: return "MOQE_OK";
    case MOQE_ERR_NULL: return "MOQE_ERR_NULL: required pointer is NULL";
    case MOQE_ERR_BITS: return "MOQE_ERR_BITS: bits must be 2, 3, 4, 8 or 16 (fp16 weights)";
    case MOQE_ERR_SHAPE: return "MOQE_ERR_SHAPE: unsupported dimension";
    case MOQE_ERR_ALIGN: return "MOQE_ERR_ALIGN: device pointer not 16-byte aligned";
    case MOQE_ERR_WORKSPACE: return "MOQE_ERR_WORKSPACE: workspace too small";
    case MOQE_ERR_HIP: return "MOQE_ERR_HIP: HIP runtime error";
    case MOQE_ERR_TIMEOUT: return "MOQE_ERR_TIMEOUT: a wait inside a single-launch step timed out";
    default: return "unknown status";
  }
}

const char* moqe_last_hip_error(void) { return g_hip_error; }

int moqe_version(void) { return 2; }

int moqe_set_prefill_policy(int min_segment_tokens, int min_batch_tokens, int all_tiled_tokens_per_expert) {
  if (min_segment_tokens < 1 || min_batch_tokens < 1 || all_tiled_tokens_per_expert < 1) return -1;
  g_prefill_min.store(min_segment_tokens);
  g_prefill_batch.store(min_batch_tokens);
  g_prefill_all.store(all_tiled_tokens_per_expert);
  return 0;
}

int moqe_set_decode_kernel(int which) {
  if (which != MOQE_DECODE_AUTO && which != MOQE_DECODE_GENERAL && which != MOQE_DECODE_ROWS8 && which != MOQE_DECODE_ROWS4)
    return -1;
  const int now = which == MOQE_DECODE_GENERAL ? 0 : which == MOQE_DECODE_ROWS8 ? 2 : which == MOQE_DECODE_ROWS4 ? 3 : 1;
  const int old = g_small_decode.exchange(now);
  return old == 0 ? MOQE_DECODE_GENERAL : old == 2 ? MOQE_DECODE_ROWS8 : old == 3 ? MOQE_DECODE_ROWS4 : MOQE_DECODE_AUTO;
}

int moqe_set_tiled_kernel(int which) {
  if (which != MOQE_TILED_AUTO && which != MOQE_TILED_STREAMED && which != MOQE_TILED_RESIDENT) return -1;
  return g_tiled_kernel.exchange(which);
}

int moqe_set_launch_mode(int mode) {
  if (mode != MOQE_LAUNCH_AUTO && mode != MOQE_LAUNCH_SEPARATE && mode != MOQE_LAUNCH_FUSED) return -1;
  return g_launch_mode.exchange(mode);
}


// 2, 3, 4, 8: quantized codes; 16: unquantized fp16 weights (the paper's baseline row)
static bool valid_bits(int bits) { return bits == 2 || bits == 3 || bits == 4 || bits == 8 || bits == 16; }

int moqe_check_matrix(int bits, int64_t K, int64_t N) {
  if (!valid_bits(bits)) return MOQE_ERR_BITS;
  PackGeom g;
  return moqe_make_geom(bits, K, N, &g) ? MOQE_OK : MOQE_ERR_SHAPE;
}

size_t moqe_packed_bytes(int bits, int64_t K, int64_t N) {
  PackGeom g;
  if (!moqe_make_geom(bits, K, N, &g)) return 0;
  return (size_t)g.matrix_bytes;
}

int moqe_check_layer(int bits, int64_t E, int64_t d, int64_t f) {
  if (!valid_bits(bits)) return MOQE_ERR_BITS;
  if (E < 1 || E > MAX_EXPERTS) return MOQE_ERR_SHAPE;
  int ks, r;
  if (moqe_check_matrix(bits, d, f) != MOQE_OK || moqe_check_matrix(bits, f, d) != MOQE_OK) return MOQE_ERR_SHAPE;
  // fp16 weights run on the tiled kernel only
  if (bits == 16) return moqe_prefill_supported(bits, d, f) && moqe_prefill_supported(bits, f, d) ? MOQE_OK : MOQE_ERR_SHAPE;
  if (!moqe_pick_ksplit(bits, d, &ks, &r) || !moqe_pick_ksplit(bits, f, &ks, &r)) return MOQE_ERR_SHAPE;
  return MOQE_OK;
}

size_t moqe_route_workspace_bytes(int64_t T, int64_t E) {
  if (T < 0 || E < 1) return 256;
  return moqe_route_ws_bytes(T, E);
}

// FFN / layer workspace: [sync words 1024][router results 1024][h buffer 0][h buffer 1]
// (CHAIN_H_BYTES each, at fixed offsets whatever T is: they carry state from launch to
// launch), then plain h [T,f] fp16 for the launches that run one contraction each.
constexpr size_t WS_HEAD = 2048;
constexpr size_t CHAIN_H_BYTES = 1 << 20;

size_t moqe_ffn_workspace_bytes(int64_t T, int64_t E, int64_t d, int64_t f) {
  (void)E;
  (void)d;
  size_t base = WS_HEAD + 2 * CHAIN_H_BYTES;
  if (T < 0 || f < 0) return base;
  return base + round256((size_t)T * (size_t)f * 2);
}

size_t moqe_layer_workspace_bytes(int64_t T, int64_t E, int64_t d, int64_t f) {
  return moqe_ffn_workspace_bytes(T, E, d, f) + moqe_route_workspace_bytes(T, E);
}

moqe_status moqe_workspace_status(const void* workspace, size_t workspace_bytes, void* stream) {
  if (!workspace) return MOQE_ERR_NULL;
  if (workspace_bytes < 1024) return MOQE_ERR_WORKSPACE;
  unsigned flag = 0;
  hipError_t e = hipMemcpyAsync(&flag, (const char*)workspace + 640, sizeof(flag), hipMemcpyDeviceToHost, (hipStream_t)stream);
  if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e);
  return flag ? MOQE_ERR_TIMEOUT : MOQE_OK;
}

moqe_status moqe_stream_read(const void* src, size_t bytes, void* sink, void* stream) {
  if (!src || !sink) return MOQE_ERR_NULL;
  if (bytes == 0 || (bytes % 1024) != 0 || bytes >= ((size_t)1 << 31)) return MOQE_ERR_SHAPE;
  if (!aligned16(src) || !aligned16(sink)) return MOQE_ERR_ALIGN;
  hipError_t e = moqe_launch_stream_read(src, bytes, (uint32_t*)sink, num_cus(), (hipStream_t)stream);
  return e == hipSuccess ? MOQE_OK : hip_fail(e);
}

static moqe_status quantize_common(const float* w, int64_t E, int64_t K, int64_t N, int bits, void* codes_out,
                                   moqe_f16* scales_out, bool tensor_scale, int codec, void* stream) {
  if (!w || !codes_out || !scales_out) return MOQE_ERR_NULL;
  if (!valid_bits(bits) || (codec == MOQE_CODEC_LOG && bits > 4)) return MOQE_ERR_BITS;
  PackGeom g;
  if (E < 1 || E > MAX_EXPERTS || !moqe_make_geom(bits, K, N, &g)) return MOQE_ERR_SHAPE;
  if (!aligned16(w) || !aligned16(codes_out) || !aligned16(scales_out)) return MOQE_ERR_ALIGN;
  hipError_t e = moqe_launch_quantize(w, E, g, codes_out, scales_out, tensor_scale, codec, (hipStream_t)stream);
  return e == hipSuccess ? MOQE_OK : hip_fail(e);
}

moqe_status moqe_quantize(const float* w, int64_t E, int64_t K, int64_t N, int bits, void* codes_out,
                          moqe_f16* scales_out, void* stream) {
  return quantize_common(w, E, K, N, bits, codes_out, scales_out, false, MOQE_CODEC_LINEAR, stream);
}

moqe_status moqe_quantize_tensor_scale(const float* w, int64_t E, int64_t K, int64_t N, int bits, void* codes_out,
                                       moqe_f16* scales_out, void* stream) {
  return quantize_common(w, E, K, N, bits, codes_out, scales_out, true, MOQE_CODEC_LINEAR, stream);
}

moqe_status moqe_quantize_log(const float* w, int64_t E, int64_t K, int64_t N, int bits, void* codes_out,
                              moqe_f16* scales_out, void* stream) {
  return quantize_common(w, E, K, N, bits, codes_out, scales_out, false, MOQE_CODEC_LOG, stream);
}

moqe_status moqe_dequantize_log(const void* codes, const moqe_f16* scales, int64_t E, int64_t K, int64_t N, int bits,
                                float* w_out, void* stream) {
  if (!codes || !scales || !w_out) return MOQE_ERR_NULL;
  if (bits != 2 && bits != 3 && bits != 4) return MOQE_ERR_BITS;
  PackGeom g;
  if (E < 1 || E > MAX_EXPERTS || !moqe_make_geom(bits, K, N, &g)) return MOQE_ERR_SHAPE;
  if (!aligned16(codes) || !aligned16(scales) || !aligned16(w_out)) return MOQE_ERR_ALIGN;
  hipError_t e = moqe_launch_dequantize_log(codes, scales, E, g, w_out, (hipStream_t)stream);
  return e == hipSuccess ? MOQE_OK : hip_fail(e);
}

moqe_status moqe_unpack(const void* codes, int64_t E, int64_t K, int64_t N, int bits, int8_t* q_out, void* stream) {
  if (!codes || !q_out) return MOQE_ERR_NULL;
  if (!valid_bits(bits) || bits == 16) return MOQE_ERR_BITS;  // (fp16 weights are not int8 codes)
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

// ---------------------------------------------------------------------------
// expert FFN
// ---------------------------------------------------------------------------


static moqe_status check_layer_ptrs(const moqe_layer* L) {
  if (!L) return MOQE_ERR_NULL;
  if (!L->codes1 || !L->scales1 || !L->bias1 || !L->codes2 || !L->scales2 || !L->bias2) return MOQE_ERR_NULL;
  if (!valid_bits(L->bits)) return MOQE_ERR_BITS;
  if (L->codec != MOQE_CODEC_LINEAR && !(L->codec == MOQE_CODEC_LOG && L->bits >= 2 && L->bits <= 4)) return MOQE_ERR_BITS;
  int st = moqe_check_layer(L->bits, L->E, L->d, L->f);
  if (st != MOQE_OK) return (moqe_status)st;
  if (!aligned16(L->codes1) || !aligned16(L->scales1) || !aligned16(L->bias1) || !aligned16(L->codes2) ||
      !aligned16(L->scales2) || !aligned16(L->bias2))
    return MOQE_ERR_ALIGN;
  return MOQE_OK;
}

// Fills the launch description shared by every FFN entry point; phases are added by the caller.
static void base_args(DecodeArgs* a, const moqe_layer* L, int64_t T, const int32_t* expert_idx, const float* gate,
                      const int32_t* seg_offsets, const int32_t* perm) {
  memset(a, 0, sizeof(*a));
  a->bits = L->codec == MOQE_CODEC_LOG ? 100 + L->bits : L->bits;  // what the kernels are instantiated on (MOQE_LOG2..4)
  a->E = (int)L->E;
  a->T = (int)T;
  a->expert_idx = (int*)expert_idx;
  a->gate = (float*)gate;
  a->seg_offsets = (int*)seg_offsets;
  a->perm = (int*)perm;
  a->min_tokens = 1;
  a->max_tokens = INT_MAX;
}

static void set_ffn1(DecodeArgs* a, const moqe_layer* L, const moqe_f16* x, moqe_f16* h, int* ksteps) {
  PhaseArgs& p = a->ph[0];
  p.codes = (const uint32_t*)L->codes1;
  p.scales = L->scales1;
  p.bias = L->bias1;
  p.K = (int)L->d;
  p.N = (int)L->f;
  moqe_pick_ksplit(L->bits, p.K, ksteps, &p.ksplit);
  p.mode = 0;
  p.a = x;
  p.out = h;
  p.residual = nullptr;
}

static void set_ffn2(DecodeArgs* a, const moqe_layer* L, const moqe_f16* h, const moqe_f16* residual, moqe_f16* y,
                     int* ksteps) {
  PhaseArgs& p = a->ph[1];
  p.codes = (const uint32_t*)L->codes2;
  p.scales = L->scales2;
  p.bias = L->bias2;
  p.K = (int)L->f;
  p.N = (int)L->d;
  moqe_pick_ksplit(L->bits, p.K, ksteps, &p.ksplit);
  p.mode = 1;
  p.a = h;
  p.out = y;
  p.residual = residual;
}

// What one contraction launches: the decode kernel (which of the two), the tiled kernel (which of
// the two), or both, and the segment size from which the tiled kernel takes over.
struct PathChoice {
  bool split;     // the tiled kernel is launched, for segments of at least pmin tokens
  int pmin;
  bool decode;    // a decode kernel is launched (for all segments, or for those below pmin)
  bool small;     // ... and it is the one for decode-sized batches
  int rows;       // ... which works on (expert, this many of its tokens): 4 or 8
  bool resident;  // the tiled kernel is the one that keeps the token rows in LDS
  bool valid;     // false: fp16 weights on a shape the tiled kernel does not take
};

static PathChoice choose_path(int bits, int64_t T, int64_t E, int64_t K, int64_t N) {
  PathChoice c;
  // many tokens per expert on average, or fp16 weights (which only the tiled kernel takes):
  // everything through the tiled kernel
  const bool tiled_only = bits == 16;
  // (8-bit codes have no tiled kernel with resident token rows and a decode kernel that reads two
  // words per step: eight times the tokens per expert)
  const int64_t per_expert = (int64_t)g_prefill_all.load() * (moqe_field_bits(bits) == 8 ? 8 : 1);
  const bool all_tiled = T >= per_expert * E;
  c.pmin = (tiled_only || all_tiled) ? 1 : g_prefill_min.load();
  // (the tiled kernel addresses its input rows with 32-bit byte offsets and its output rows with
  // 32-bit element offsets)
  c.split = T >= c.pmin && (tiled_only || T >= g_prefill_batch.load()) && moqe_prefill_supported(bits, K, N) &&
            T * K * 2 < (1ll << 32) && T * N < (1ll << 31);
  // The decode-sized kernel, where it applies, keeps batches of up to 128 tokens to itself (in
  // pairs of 8 rows an expert's weights are still streamed about once there) unless segments are
  // asked onto the tiled kernel explicitly.
  const int sd = g_small_decode.load();
  c.rows = (sd == 2 || (sd == 1 && T >= ROWS8_FROM_TOKENS)) ? 8 : 4;
  const bool small_ok = sd && bits != 16 && moqe_decode_small_supported(bits, T, E, K, N, num_cus(), c.rows);
  if (small_ok && T > 64 && g_prefill_min.load() >= MOQE_PREFILL_MIN_SEGMENT_DEFAULT) c.split = false;
  c.valid = !tiled_only || c.split;
  // (with a threshold of one token every segment is the tiled kernel's: no decode launch)
  c.decode = !c.split || c.pmin > 1;
  c.small = c.decode && small_ok;
  // token rows resident in LDS: always where a tile of 64 tokens fits (K <= 1024); with the
  // tiles of 16 tokens that a longer K leaves room for, while most experts have no more tokens
  // than one such tile (beyond that the weights are read once per 16 tokens, and staging K in
  // blocks for 64 at a time is faster)
  const int tk = g_tiled_kernel.load();
  c.resident = c.split && tk != MOQE_TILED_STREAMED && E <= 1024 && T * N < (1ll << 30) &&
               moqe_resident_supported(bits, K, N) && (K <= 1024 || tk == MOQE_TILED_RESIDENT || T <= 16 * E);
  return c;
}

int moqe_contraction_path(int bits, int64_t T, int64_t E, int64_t K, int64_t N) {
  if (!valid_bits(bits) || T < 1 || T > MAX_TOKENS || E < 1 || E > MAX_EXPERTS || K < 1 || N < 1) return -1;
  int ks = 0, r = 0;
  if (bits != 16 && !moqe_pick_ksplit(bits, K, &ks, &r)) return -1;
  const PathChoice c = choose_path(bits, T, E, K, N);
  if (!c.valid) return -1;
  int m = 0;
  if (c.decode) m |= c.small ? MOQE_PATH_DECODE_SMALL : MOQE_PATH_DECODE;
  if (c.split) m |= c.resident ? MOQE_PATH_TILED_RESIDENT : MOQE_PATH_TILED_STAGED;
  return m;
}

// One contraction as its own launch(es): the decode kernel takes the small segments, the
// tiled MFMA kernel the large ones (none can exist when T is below the threshold).
static hipError_t launch_contraction(DecodeArgs& a, int phase, int ksteps, hipStream_t stream) {
  const PhaseArgs& p = a.ph[phase];
  const PathChoice c = choose_path(a.bits, a.T, a.E, p.K, p.N);
  const bool split = c.split;
  const int pmin = c.pmin;
  if (!c.valid) return hipErrorInvalidValue;  // (sizes are checked by the callers)
  a.ksteps = ksteps;
  a.phase_mask = 2 << phase;
  a.min_tokens = 1;
  a.max_tokens = split ? pmin : INT_MAX;
  if (c.decode) {
    hipError_t e;
    if (c.small) {
      // decode-sized batch: the lean kernel (one pair per workgroup)
      SmallDecodeArgs s;
      memset(&s, 0, sizeof(s));
      s.bits = a.bits;
      s.ksteps = ksteps;
      s.ksplit = p.ksplit;
      s.rows = c.rows;
      s.mode = p.mode;
      s.E = a.E;
      s.T = a.T;
      s.N = p.N;
      s.min_tokens = a.min_tokens;
      s.max_tokens = a.max_tokens;
      s.codes = p.codes;
      s.scales = p.scales;
      s.bias = p.bias;
      s.a = p.a;
      s.out = p.out;
      s.residual = p.residual;
      s.gate = a.gate;
      s.seg_offsets = a.seg_offsets;
      s.perm = a.perm;
      e = moqe_launch_decode_small(s, num_cus(), stream);
    } else {
      e = moqe_launch_decode(a, num_cus(), stream);
    }
    if (e != hipSuccess || !split) return e;
  }
  PrefillArgs q;
  memset(&q, 0, sizeof(q));
  q.bits = a.bits;
  q.E = a.E;
  q.T = a.T;
  q.K = p.K;
  q.N = p.N;
  q.mode = p.mode;
  q.min_tokens = pmin;
  q.codes = p.codes;
  q.scales = p.scales;
  q.bias = p.bias;
  q.a = p.a;
  q.out = p.out;
  q.residual = p.residual;
  q.seg_offsets = a.seg_offsets;
  q.perm = a.perm;
  q.gate = a.gate;
  if (c.resident) return moqe_launch_resident(q, num_cus(), stream);
  return moqe_launch_prefill(q, num_cus(), stream);
}

// Unit counts are 32-bit inside the kernel.
static bool units_fit(int64_t T, int64_t E, int64_t N) { return ((T + 3) / 4 + E) * (N / 16) < (1ll << 31); }
// fp16 weights: the tiled kernel's 32-bit offsets must hold for both contractions
static bool fp16_fits(const moqe_layer* L, int64_t T) {
  const int64_t m = L->d > L->f ? L->d : L->f;
  return L->bits != 16 || (T * m * 2 < (1ll << 32));
}

moqe_status moqe_expert_ffn1(const moqe_layer* L, const moqe_f16* x, int64_t T, const int32_t* seg_offsets,
                             const int32_t* perm, moqe_f16* h, void* stream) {
  if (!L || !x || !seg_offsets || !perm || !h) return MOQE_ERR_NULL;
  moqe_status st = check_layer_ptrs(L);
  if (st != MOQE_OK) return st;
  if (T < 0 || T > MAX_TOKENS || !units_fit(T, L->E, L->f) || !fp16_fits(L, T)) return MOQE_ERR_SHAPE;
  if (!aligned16(x) || !aligned16(seg_offsets) || !aligned16(perm) || !aligned16(h)) return MOQE_ERR_ALIGN;
  if (T == 0) return MOQE_OK;
  DecodeArgs a;
  base_args(&a, L, T, nullptr, nullptr, seg_offsets, perm);
  int ks = 0;
  set_ffn1(&a, L, x, h, &ks);
  hipError_t e = launch_contraction(a, 0, ks, (hipStream_t)stream);
  return e == hipSuccess ? MOQE_OK : hip_fail(e);
}

moqe_status moqe_expert_ffn2(const moqe_layer* L, const moqe_f16* h, int64_t T, const float* gate,
                             const int32_t* seg_offsets, const int32_t* perm, const moqe_f16* residual, moqe_f16* y,
                             void* stream) {
  if (!L || !h || !gate || !seg_offsets || !perm || !y) return MOQE_ERR_NULL;
  moqe_status st = check_layer_ptrs(L);
  if (st != MOQE_OK) return st;
  if (T < 0 || T > MAX_TOKENS || !units_fit(T, L->E, L->d) || !fp16_fits(L, T)) return MOQE_ERR_SHAPE;
  if (!aligned16(h) || !aligned16(gate) || !aligned16(seg_offsets) || !aligned16(perm) || !aligned16(y) ||
      (residual && !aligned16(residual)))
    return MOQE_ERR_ALIGN;
  if (T == 0) return MOQE_OK;
  DecodeArgs a;
  base_args(&a, L, T, nullptr, gate, seg_offsets, perm);
  int ks = 0;
  set_ffn2(&a, L, h, residual, y, &ks);
  hipError_t e = launch_contraction(a, 1, ks, (hipStream_t)stream);
  return e == hipSuccess ? MOQE_OK : hip_fail(e);
}

// Runs FFN1 and FFN2 (and, with w_gate, the router in front of them).  One launch when both
// contractions use the same wave slice length (and the router fits the kernel's own), else
// one launch per phase.
static moqe_status run_layer(const moqe_layer* L, const moqe_f16* w_gate, const moqe_f16* x, int64_t T,
                             int32_t* expert_idx, float* gate, int32_t* seg_offsets, int32_t* perm,
                             const moqe_f16* residual, moqe_f16* y, void* workspace, size_t workspace_bytes,
                             void* stream) {
  moqe_status st = check_layer_ptrs(L);
  if (st != MOQE_OK) return st;
  if (T < 0 || T > MAX_TOKENS || !units_fit(T, L->E, L->f) || !units_fit(T, L->E, L->d) || !fp16_fits(L, T))
    return MOQE_ERR_SHAPE;
  if (!aligned16(x) || !aligned16(expert_idx) || !aligned16(gate) || !aligned16(seg_offsets) || !aligned16(perm) ||
      !aligned16(y) || !aligned16(workspace) || (residual && !aligned16(residual)) ||
      (w_gate && !aligned16(w_gate)))
    return MOQE_ERR_ALIGN;
  const size_t ffn_bytes = moqe_ffn_workspace_bytes(T, L->E, L->d, L->f);
  const size_t need = w_gate ? moqe_layer_workspace_bytes(T, L->E, L->d, L->f) : ffn_bytes;
  if (workspace_bytes < need) return MOQE_ERR_WORKSPACE;
  const size_t h_bytes = (size_t)T * (size_t)L->f * 2;
  unsigned* sync = (unsigned*)workspace;
  moqe_f16* h_chain = (moqe_f16*)((char*)workspace + WS_HEAD);
  moqe_f16* h_plain = (moqe_f16*)((char*)workspace + WS_HEAD + 2 * CHAIN_H_BYTES);
  void* route_ws = (char*)workspace + ffn_bytes;

  if (T == 0) {
    if (!w_gate) return MOQE_OK;
    return moqe_route(x, w_gate, T, L->d, L->E, expert_idx, gate, seg_offsets, perm, route_ws,
                      workspace_bytes - ffn_bytes, stream);
  }

  DecodeArgs a;
  base_args(&a, L, T, expert_idx, gate, seg_offsets, perm);
  int ks1 = 0, ks2 = 0;
  set_ffn1(&a, L, x, h_plain, &ks1);
  set_ffn2(&a, L, h_plain, residual, y, &ks2);
  // one launch for both contractions when they share the wave slice length and h fits the
  // chained buffers; the router joins when it fits the kernel's own
  const int launch_mode = g_launch_mode.load();
  const bool can_chain = L->bits != 16 && ks1 == ks2 && h_bytes <= CHAIN_H_BYTES;
  const bool can_fuse_route = w_gate && can_chain && moqe_decode_can_route(T, L->d, L->E);
  // Measured on the decode workload, one launch per step of the path is as fast as the
  // single launch or faster (the phases of the single launch wait for each other through
  // memory, which costs about what the extra launches cost), so AUTO takes separate launches.
  const bool chain = launch_mode == MOQE_LAUNCH_FUSED && can_chain;
  const bool fuse_route = chain && can_fuse_route;

  if (w_gate && !fuse_route) {
    st = moqe_route(x, w_gate, T, L->d, L->E, expert_idx, gate, seg_offsets, perm, route_ws,
                    workspace_bytes - ffn_bytes, stream);
    if (st != MOQE_OK) return st;
  }
  hipError_t e;
  if (chain) {
    a.ksteps = ks1;
    a.phase_mask = fuse_route ? 7 : 6;
    a.x = x;
    a.w_gate = w_gate;
    a.d_route = (int)L->d;
    a.sync = sync;
    a.route_entries = (unsigned long long*)((char*)workspace + 1024);
    a.h_base = h_chain;
    a.h_stride = CHAIN_H_BYTES / 2;
    a.h_bytes = (unsigned)h_bytes;
    e = moqe_launch_decode(a, num_cus(), (hipStream_t)stream);
    return e == hipSuccess ? MOQE_OK : hip_fail(e);
  }
  e = launch_contraction(a, 0, ks1, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e);
  e = launch_contraction(a, 1, ks2, (hipStream_t)stream);
  return e == hipSuccess ? MOQE_OK : hip_fail(e);
}

moqe_status moqe_expert_ffn(const moqe_layer* L, const moqe_f16* x, int64_t T, const int32_t* expert_idx,
                            const float* gate, const int32_t* seg_offsets, const int32_t* perm,
                            const moqe_f16* residual, moqe_f16* y, void* workspace, size_t workspace_bytes,
                            void* stream) {
  if (!L || !x || !expert_idx || !gate || !seg_offsets || !perm || !y || !workspace) return MOQE_ERR_NULL;
  return run_layer(L, nullptr, x, T, (int32_t*)expert_idx, (float*)gate, (int32_t*)seg_offsets, (int32_t*)perm,
                   residual, y, workspace, workspace_bytes, stream);
}

moqe_status moqe_moe_layer(const moqe_layer* L, const moqe_f16* w_gate, const moqe_f16* x, int64_t T,
                           int32_t* expert_idx, float* gate, int32_t* seg_offsets, int32_t* perm,
                           const moqe_f16* residual, moqe_f16* y, void* workspace, size_t workspace_bytes,
                           void* stream) {
  if (!L || !w_gate || !x || !expert_idx || !gate || !seg_offsets || !perm || !y || !workspace) return MOQE_ERR_NULL;
  return run_layer(L, w_gate, x, T, expert_idx, gate, seg_offsets, perm, residual, y, workspace, workspace_bytes,
                   stream);
}

// ---------------------------------------------------------------------------
// the layer step on the library's own scratch (callers that cannot allocate)
// ---------------------------------------------------------------------------
}  // extern "C"

// What moqe_moe_layer takes as `workspace`, held by the library: one copy per GPU the library
// runs on, zero when the code object is loaded (the state the single-launch mode wants to find)
// and kept from call to call like a caller's buffer.  In host code this name is only a handle
// for hipGetSymbolAddress; kernels get the address that call returns.
static __device__ __align__(256) unsigned char moqe_static_scratch[MOQE_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
void* g_scratch_ptr[MAX_DEVICES];  // device address of moqe_static_scratch on each device, once known
std::mutex g_scratch_mutex;

// Address of the current device's copy of the scratch array (looked up once per device).
moqe_status static_scratch(void** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e);
  if (dev < 0 || dev >= MAX_DEVICES) return hip_fail(hipErrorInvalidDevice);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(moqe_static_scratch));
    if (e != hipSuccess) return hip_fail(e);
    if (!p) return hip_fail(hipErrorInvalidSymbol);
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return MOQE_OK;
}
}  // namespace

extern "C" {

moqe_status moqe_moe_layer_static(const moqe_layer* L, const moqe_f16* w_gate, const moqe_f16* x, int64_t T,
                                  int32_t* expert_idx, float* gate, int32_t* seg_offsets, int32_t* perm,
                                  const moqe_f16* residual, moqe_f16* y, void* stream) {
  if (!L || !w_gate || !x || !expert_idx || !gate || !seg_offsets || !perm || !y) return MOQE_ERR_NULL;
  moqe_status st = check_layer_ptrs(L);
  if (st != MOQE_OK) return st;
  if (T < 0 || T > MAX_TOKENS) return MOQE_ERR_SHAPE;
  if (!aligned16(x) || !aligned16(expert_idx) || !aligned16(gate) || !aligned16(seg_offsets) || !aligned16(perm) ||
      !aligned16(y) || (residual && !aligned16(residual)) || !aligned16(w_gate))
    return MOQE_ERR_ALIGN;
  // the scratch a caller of moqe_moe_layer would bring for these sizes must fit the array
  const size_t need = moqe_layer_workspace_bytes(T, L->E, L->d, L->f);
  if (need > (size_t)MOQE_STATIC_SCRATCH_BYTES) return MOQE_ERR_WORKSPACE;
  void* scratch = nullptr;
  st = static_scratch(&scratch);
  if (st != MOQE_OK) return st;
  return run_layer(L, w_gate, x, T, expert_idx, gate, seg_offsets, perm, residual, y, scratch, need, stream);
}

}  // extern "C"
