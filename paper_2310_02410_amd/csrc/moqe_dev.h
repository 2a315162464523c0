// Device-side helpers shared by the MoQE kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t uint4_t __attribute__((ext_vector_type(4)));
typedef uint32_t uint2_t __attribute__((ext_vector_type(2)));

#define MOQE_WAVE 64

// ---------------------------------------------------------------------------
// Geometry of the packed code layout (one [K,N] matrix).  See include/moqe.h.
// ---------------------------------------------------------------------------
struct PackGeom {
  int bits;  // 16: unquantized fp16 values in place of codes (field = the fp16 bit pattern)
  int K, N;
  int S;            // 32-row steps = K / 32
  int SC;           // steps per chunk
  int Q;            // chunks per column tile = S / SC
  int chunk_bytes;  // 64 * SC * bits
  int lo_lane_bytes;  // bytes one slot owns in the main (2-, 4- or 8-bit) plane of a chunk
  int hi_lane_bytes;  // bytes one slot owns in the 1-bit plane (int3 only, else 0)
  int64_t matrix_bytes;
};

// What the kernels are instantiated on for b-bit log-scale codes (App. A: sign bit + (b-1)-bit
// exponent): fields and layout are those of the linear b-bit codes, only the unpack differs.
constexpr int MOQE_LOG2 = 102, MOQE_LOG3 = 103, MOQE_LOG4 = 104;
__host__ __device__ constexpr bool moqe_is_log(int bits) { return bits >= MOQE_LOG2 && bits <= MOQE_LOG4; }
__host__ __device__ constexpr int moqe_field_bits(int bits) { return moqe_is_log(bits) ? bits - 100 : bits; }

// (a slot owns at most 16 bytes of a chunk's main plane)
__host__ __device__ inline int moqe_sc_max(int bits) { return bits == 16 ? 1 : bits == 8 ? 2 : bits == 4 ? 4 : 8; }

// Returns false when (bits, K, N) cannot be packed.
__host__ __device__ inline bool moqe_make_geom(int bits, int64_t K, int64_t N, PackGeom* g) {
  if (bits != 2 && bits != 3 && bits != 4 && bits != 8 && bits != 16) return false;
  if (K <= 0 || N <= 0 || (K % 32) || (N % 16)) return false;
  if (K > (1 << 20) || N > (1 << 20)) return false;
  int S = (int)(K / 32);
  int sc = moqe_sc_max(bits) < S ? moqe_sc_max(bits) : S;
  if (S % sc) return false;
  if (bits == 2 && (sc % 2)) return false;
  if (bits == 3 && (sc % 4)) return false;
  g->bits = bits;
  g->K = (int)K;
  g->N = (int)N;
  g->S = S;
  g->SC = sc;
  g->Q = S / sc;
  g->chunk_bytes = 64 * sc * bits;
  g->lo_lane_bytes = (bits == 3) ? sc * 2 : sc * bits;
  g->hi_lane_bytes = (bits == 3) ? sc : 0;
  g->matrix_bytes = (int64_t)K * N * bits / 8;
  return true;
}

// fp16 <-> bits
__device__ inline half_t half_from_bits(uint16_t u) {
  union { uint16_t u; half_t h; } c;
  c.u = u;
  return c.h;
}
__device__ inline uint16_t half_to_bits(half_t h) {
  union { uint16_t u; half_t h; } c;
  c.h = h;
  return c.u;
}

// wave-level helpers (64 lanes)
__device__ inline int lane_id() { return (int)(threadIdx.x & 63); }
__device__ inline uint32_t uniform_u32(uint32_t v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ inline int uniform_i32(int v) { return (int)__builtin_amdgcn_readfirstlane((uint32_t)v); }

// A constant the optimizer cannot see through, kept in a scalar / vector register.
// (a & mask) | magic then compiles to one v_and_or_b32, whose VOP3 encoding cannot
// take literals, instead of an and plus an or with literal operands.
__device__ inline uint32_t opaque_sgpr(uint32_t c) {
  asm volatile("" : "+s"(c));
  return c;
}
__device__ inline uint32_t opaque_vgpr(uint32_t c) {
  asm volatile("" : "+v"(c));
  return c;
}

// ---------------------------------------------------------------------------
// Top-1 and softmax denominator of a row of logits (App. B top-1 gating)
// ---------------------------------------------------------------------------
// Logits are compared through an integer key with the order of the values: one integer compare
// per decision, no branches.  -0 and +0 get the same key; a NaN gets the largest key of all, so
// it ranks above every number and ties with another NaN, as in the plain definition "first
// index of the row maximum" once a NaN is met (non-finite logits are outside the method's
// domain; what matters is that the index stays in [0, E) and is unique).
__device__ inline int logit_key(float v) {
  const int u = __builtin_bit_cast(int, v + 0.0f);  // (-0 + 0 = +0)
  const int k = u ^ ((u >> 31) & 0x7fffffff);
  return v != v ? 0x7fffffff : k;
}
__device__ inline float logit_of_key(int k) { return __builtin_bit_cast(float, k ^ ((k >> 31) & 0x7fffffff)); }
constexpr int LOGIT_KEY_LOWEST = (int)0x807fffffu;  // the key of -inf

// Cross-lane moves inside a row of 16 lanes, as DPP operands of ordinary vector instructions (no
// trip through the LDS crossbar, which is what a general shuffle costs): lane ^ 1, lane ^ 2, then
// the mirror images within 8 and within 16 lanes.  After the four steps of a symmetric reduction
// every lane of a row holds the row's result; the four rows meet through readlane.
template <int CTRL>
__device__ inline float dpp_f32(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, false));
}
template <int CTRL>
__device__ inline int dpp_i32(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, false);
}
constexpr int DPP_XOR1 = 0xB1, DPP_XOR2 = 0x4E, DPP_HALF_MIRROR = 0x141, DPP_MIRROR = 0x140;

__device__ inline float readlane_f32(float v, int l) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), l));
}

// (key, index) pairs meet: the larger key wins, the lower index among equal keys (a symmetric
// rule, so both lanes of a DPP pair end up with the same winner).
__device__ inline void top1_meet(int& key, int& idx, int okey, int oidx) {
  const bool take = (okey > key) | ((okey == key) & (oidx < idx));
  key = take ? okey : key;
  idx = take ? oidx : idx;
}
// The 16 lanes of a row -> the pair all of them agree on.
__device__ inline void row16_top1(int& key, int& idx) {
  top1_meet(key, idx, dpp_i32<DPP_XOR1>(key), dpp_i32<DPP_XOR1>(idx));
  top1_meet(key, idx, dpp_i32<DPP_XOR2>(key), dpp_i32<DPP_XOR2>(idx));
  top1_meet(key, idx, dpp_i32<DPP_HALF_MIRROR>(key), dpp_i32<DPP_HALF_MIRROR>(idx));
  top1_meet(key, idx, dpp_i32<DPP_MIRROR>(key), dpp_i32<DPP_MIRROR>(idx));
}
__device__ inline float row16_sum(float sum) {
  sum += dpp_f32<DPP_XOR1>(sum);
  sum += dpp_f32<DPP_XOR2>(sum);
  sum += dpp_f32<DPP_HALF_MIRROR>(sum);
  sum += dpp_f32<DPP_MIRROR>(sum);
  return sum;
}

// The order in which every router here scans a row of E <= 256 logits: a row of 16 lanes, lane q
// owning the experts q, q + 16, q + 32, ... (one after the other, ascending), the 16 lanes then
// meeting in the four DPP steps above.  Top-1 is exact whatever the order; the softmax
// denominator is a sum of roundings, and with one order everywhere a token gets the same gate
// from every kernel.  `read(e)` returns logit e of the row; NPL > 0 says at compile time that
// every lane owns exactly NPL experts (E = 16 NPL).  Every lane of the 16 gets the result.
// A row without any value above -inf keeps index 0.
template <int NPL, typename Read>
__device__ inline void row16_pick(Read read, int q, int E, int* idx_out, float* gate_out) {
  int key = LOGIT_KEY_LOWEST, idx = 0;
  float sum = 0.0f;
  if constexpr (NPL > 0) {
    float v[NPL];
#pragma unroll
    for (int i = 0; i < NPL; ++i) {
      v[i] = read(q + 16 * i);
      const int k = logit_key(v[i]);
      const bool take = k > key;  // ascending: strictly above keeps the lowest index
      key = take ? k : key;
      idx = take ? q + 16 * i : idx;
    }
    row16_top1(key, idx);
    const float best = logit_of_key(key);
#pragma unroll
    for (int i = 0; i < NPL; ++i) sum += expf(v[i] - best);
  } else {
    for (int e = q; e < E; e += 16) {
      const int k = logit_key(read(e));
      const bool take = k > key;
      key = take ? k : key;
      idx = take ? e : idx;
    }
    row16_top1(key, idx);
    const float best = logit_of_key(key);
    for (int e = q; e < E; e += 16) sum += expf(read(e) - best);
  }
  *idx_out = idx;
  *gate_out = 1.0f / row16_sum(sum);
}

// One wave, one row of E logits in LDS or global memory: every lane gets the same (idx, gate).
// Up to 256 experts in the order above (the wave's four rows of lanes all scan the same row);
// beyond that, where no second kernel has to agree, the 64 lanes share the row.
__device__ inline void wave_pick(const float* row, int E, int* idx_out, float* gate_out) {
  const int lane = lane_id();
  if (E <= 256) {
    row16_pick<0>([row](int e) { return row[e]; }, lane & 15, E, idx_out, gate_out);
    return;
  }
  int key = LOGIT_KEY_LOWEST, idx = 0;
  for (int e = lane; e < E; e += 64) {
    const int k = logit_key(row[e]);
    const bool take = k > key;
    key = take ? k : key;
    idx = take ? e : idx;
  }
  row16_top1(key, idx);
  int wkey = __builtin_amdgcn_readlane(key, 0), widx = __builtin_amdgcn_readlane(idx, 0);
#pragma unroll
  for (int r = 1; r < 4; ++r) top1_meet(wkey, widx, __builtin_amdgcn_readlane(key, 16 * r), __builtin_amdgcn_readlane(idx, 16 * r));
  const float best = logit_of_key(wkey);
  float sum = 0.0f;
  for (int e = lane; e < E; e += 64) sum += expf(row[e] - best);
  sum = row16_sum(sum);
  const float total = (readlane_f32(sum, 0) + readlane_f32(sum, 16)) + (readlane_f32(sum, 32) + readlane_f32(sum, 48));
  *idx_out = widx;
  *gate_out = 1.0f / total;
}

// Inclusive prefix sum over the 64 lanes: shifts inside the rows of 16 lanes as DPP operands
// (lanes a shift would take from outside the row read 0), then the row totals by readlane.
template <int N>
__device__ inline int dpp_row_shr(int v) {
  return __builtin_amdgcn_update_dpp(0, v, 0x110 + N, 0xF, 0xF, true);
}
__device__ inline int wave_inclusive_scan(int v) {
  v += dpp_row_shr<1>(v);
  v += dpp_row_shr<2>(v);
  v += dpp_row_shr<4>(v);
  v += dpp_row_shr<8>(v);
  const int t0 = __builtin_amdgcn_readlane(v, 15), t1 = __builtin_amdgcn_readlane(v, 31),
            t2 = __builtin_amdgcn_readlane(v, 47);
  const int row = lane_id() >> 4;
  return v + (row == 0 ? 0 : row == 1 ? t0 : row == 2 ? t0 + t1 : t0 + t1 + t2);
}
