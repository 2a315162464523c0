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
// Wave-level top-1 and sum (the router's argmax and softmax denominator; App. B top-1 gating)
// ---------------------------------------------------------------------------
// Order of the top-1 comparison: a NaN ranks above every number and ties with another NaN, as
// in the plain definition "first index of the row maximum" once a NaN is met (non-finite logits
// are outside the method's domain; what matters is that the index stays in [0, E) and is unique).
__device__ inline bool logit_above(float a, float b) { return (a > b) || (a != a && b == b); }
__device__ inline bool logit_same(float a, float b) { return (a == b) || (a != a && b != b); }

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

// All lanes' (value, index) pairs -> the pair every lane agrees on: the largest value, the lowest
// index among equals (a symmetric rule, so both lanes of a DPP pair end up with the same winner).
__device__ inline void wave_top1(float best, int bidx, float* best_out, int* idx_out) {
#define MOQE_PICK_STEP(CTRL)                                                        \
  {                                                                                 \
    const float ov = dpp_f32<CTRL>(best);                                           \
    const int oi = dpp_i32<CTRL>(bidx);                                             \
    const bool take = logit_above(ov, best) || (logit_same(ov, best) && oi < bidx); \
    best = take ? ov : best;                                                        \
    bidx = take ? oi : bidx;                                                        \
  }
  MOQE_PICK_STEP(DPP_XOR1)
  MOQE_PICK_STEP(DPP_XOR2)
  MOQE_PICK_STEP(DPP_HALF_MIRROR)
  MOQE_PICK_STEP(DPP_MIRROR)
#undef MOQE_PICK_STEP
  float wbest = readlane_f32(best, 0);
  int widx = __builtin_amdgcn_readlane(bidx, 0);
#pragma unroll
  for (int r = 1; r < 4; ++r) {
    const float ov = readlane_f32(best, 16 * r);
    const int oi = __builtin_amdgcn_readlane(bidx, 16 * r);
    const bool take = logit_above(ov, wbest) || (logit_same(ov, wbest) && oi < widx);
    wbest = take ? ov : wbest;
    widx = take ? oi : widx;
  }
  *best_out = wbest;
  *idx_out = widx;
}

// Sum over the 64 lanes in a fixed order (the same in every kernel that computes a gate, so that
// the gate does not depend on which kernel routed).
__device__ inline float wave_sum(float sum) {
  sum += dpp_f32<DPP_XOR1>(sum);
  sum += dpp_f32<DPP_XOR2>(sum);
  sum += dpp_f32<DPP_HALF_MIRROR>(sum);
  sum += dpp_f32<DPP_MIRROR>(sum);
  return (readlane_f32(sum, 0) + readlane_f32(sum, 16)) + (readlane_f32(sum, 32) + readlane_f32(sum, 48));
}

