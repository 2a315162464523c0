// Expert FFN contraction for few tokens per expert (decode steps): fused
// dequantize-in-register grouped GEMM, bound by the packed weight bytes it reads.
//
// out[rows of expert e, n] = epilogue( sum_k a[row, k] * (Q_e[k, n] * s_e[n]) + b_e[n] )
// (paper Sec. 2.1 two-layer FFN, App. A dequantization A' = Q s; the per-channel
// scale multiplies the finished K-sum because it does not depend on k).
//
// Work decomposition
//   pair  = (expert e, tile of 16 routed tokens of e)       P pairs, found on device
//   unit  = (pair, column tile of 16 output channels)       U = P * N/16
//   team  = `ksplit` waves of a workgroup sharing one unit along K; each wave keeps
//           its K-slice (32*KSTEPS rows) of the 16 token rows in registers as MFMA
//           A-fragments and streams the unit's packed codes with 16-byte loads.
//   Units are split evenly over the persistent grid; inside a workgroup the teams
//   take them round-robin.  Codes are unpacked to fp16 with mask/or tricks (the
//   fp16 exponent field supplies the integer bias) and go straight from registers
//   into v_mfma_f32_16x16x32_f16 as the B operand (16 channels x 32 rows).
#include "moqe_dev.h"
#include "moqe_kernels.h"

#ifdef MOQE_PHASE_TRACE
#define STAMP(i)                                                                         \
  do {                                                                                   \
    if (a.trace && (threadIdx.x == 0)) a.trace[blockIdx.x * 8 + (i)] = wall_clock64();   \
  } while (0)
#define KEEP(v) asm volatile("" ::"v"(v))
#else
#define STAMP(i)
#define KEEP(v)
#endif

namespace {

constexpr int WG_THREADS = 256;
constexpr int WG_WAVES = 4;
constexpr int MAX_E = 1024;

__device__ inline half8_t frag_from_words(uint32_t r0, uint32_t r1, uint32_t r2, uint32_t r3) {
  uint4_t v = {r0, r1, r2, r3};
  return __builtin_bit_cast(half8_t, v);
}

__device__ inline uint32_t pk_sub(uint32_t v, float c) {
  half2_t h = __builtin_bit_cast(half2_t, v);
  half2_t k = {(half_t)c, (half_t)c};
  h = h - k;
  return __builtin_bit_cast(uint32_t, h);
}

__device__ inline half8_t const_frag(float c0, float c1, float c2, float c3) {
  half8_t v = {(half_t)c0, (half_t)c0, (half_t)c1, (half_t)c1, (half_t)c2, (half_t)c2, (half_t)c3, (half_t)c3};
  return v;
}

// Masks (scalar registers) and fp16 exponent patterns (vector registers; base << 16 | base
// with a zero mantissa) of the unpack sequences, created once per kernel.
template <int BITS>
struct UnpackConsts {
  uint32_t m_000f, m_00f0;                  // int4 nibble masks
  uint32_t m_0030, m_00c0, m_0300;          // 2-bit field masks at bits 4, 6, 8
  uint32_t m_0040, m_0080, m_0100, m_0200;  // single-bit masks at bits 6..9 (int3 high plane)
  uint32_t x1024, x64, x32, x16, x8, x4;    // exponent patterns
  __device__ inline void init() {
    if (BITS == 4) {
      m_000f = opaque_sgpr(0x000F000Fu);
      m_00f0 = opaque_sgpr(0x00F000F0u);
      x1024 = opaque_vgpr(0x64006400u);
      x64 = opaque_vgpr(0x54005400u);
    } else {
      m_0030 = opaque_sgpr(0x00300030u);
      m_00c0 = opaque_sgpr(0x00C000C0u);
      m_0300 = opaque_sgpr(0x03000300u);
      x64 = opaque_vgpr(0x54005400u);
      x16 = opaque_vgpr(0x4C004C00u);
      x4 = opaque_vgpr(0x44004400u);
    }
    if (BITS == 3) {
      m_0040 = opaque_sgpr(0x00400040u);
      m_0080 = opaque_sgpr(0x00800080u);
      m_0100 = opaque_sgpr(0x01000100u);
      m_0200 = opaque_sgpr(0x02000200u);
      x32 = opaque_vgpr(0x50005000u);
      x8 = opaque_vgpr(0x48004800u);
    }
  }
};

// ---- int4: one word per step; word bit position of code i (i = k % 8): 16 (i & 1) + 4 (i >> 1).
// Nibbles at bits 0-3 get base 1024 and are made exact with a packed subtract (a bias that
// large would cost accuracy if carried through the K-sum); nibbles at bits 4-7 keep base 64
// and their 64 + 8 is removed after the K-sum like the int2 fields.
template <class C>
__device__ inline half8_t unpack4(uint32_t d, const C& c) {
  uint32_t d8 = d >> 8;
  uint32_t r0 = pk_sub((d & c.m_000f) | c.x1024, 1032.0f);
  uint32_t r1 = (d & c.m_00f0) | c.x64;
  uint32_t r2 = pk_sub((d8 & c.m_000f) | c.x1024, 1032.0f);
  uint32_t r3 = (d8 & c.m_00f0) | c.x64;
  return frag_from_words(r0, r1, r2, r3);
}

// ---- int2: one word per two steps.  Fields are left with their exponent bias
// (value = base + u); the bias and the zero point are removed after the K-sum
// through bias_frag(): sum_k a_k (base_k + u_k) - sum_k a_k (base_k + 2).
// even step: fields at bits 0,2,4,6 of each half; odd step: bits 8,10,12,14.
template <int PARITY, class C>
__device__ inline half8_t unpack2(uint32_t d, const C& c) {
  if (PARITY == 0) {
    uint32_t dl = d << 4;
    uint32_t r0 = (dl & c.m_0030) | c.x64;  // bits 0-1 -> 4-5
    uint32_t r1 = (dl & c.m_00c0) | c.x16;  // bits 2-3 -> 6-7
    uint32_t r2 = (d & c.m_0030) | c.x64;   // bits 4-5
    uint32_t r3 = (d & c.m_00c0) | c.x16;   // bits 6-7
    return frag_from_words(r0, r1, r2, r3);
  } else {
    uint32_t dr = d >> 6;
    uint32_t r0 = (d & c.m_0300) | c.x4;    // bits 8-9
    uint32_t r1 = (dr & c.m_0030) | c.x64;  // bits 10-11 -> 4-5
    uint32_t r2 = (dr & c.m_00c0) | c.x16;  // bits 12-13 -> 6-7
    uint32_t r3 = (dr & c.m_0300) | c.x4;   // bits 14-15 -> 8-9
    return frag_from_words(r0, r1, r2, r3);
  }
}

// ---- int3 high plane: one word per four steps, one bit per code, worth 4.
// step ss (0..3) owns bits 4 ss .. 4 ss + 3 of each half; they are moved to
// mantissa bits 6..9 where, with bases 64, 32, 16, 8, a set bit adds exactly 4.
template <int SS, class C>
__device__ inline half8_t unpack1x4(uint32_t d, const C& c) {
  uint32_t v = SS == 0 ? (d << 6) : SS == 1 ? (d << 2) : SS == 2 ? (d >> 2) : (d >> 6);
  uint32_t r0 = (v & c.m_0040) | c.x64;
  uint32_t r1 = (v & c.m_0080) | c.x32;
  uint32_t r2 = (v & c.m_0100) | c.x16;
  uint32_t r3 = (v & c.m_0200) | c.x8;
  return frag_from_words(r0, r1, r2, r3);
}

// Constant B fragment holding, per code position, the amount the unpacked value
// exceeds the signed code: exponent bias(es) + zero point.
template <int BITS>
__device__ inline half8_t bias_frag(int parity) {
  if (BITS == 4) return const_frag(0, 72, 0, 72);
  if (BITS == 2) return parity == 0 ? const_frag(66, 18, 66, 18) : const_frag(6, 66, 18, 6);
  // int3: low-plane bias + high-plane bias + zero point 4
  return parity == 0 ? const_frag(64 + 64 + 4, 16 + 32 + 4, 64 + 16 + 4, 16 + 8 + 4)
                     : const_frag(4 + 64 + 4, 64 + 32 + 4, 16 + 16 + 4, 4 + 8 + 4);
}

template <int BITS, int KSTEPS>
struct Shape {
  static constexpr int SCMAX = BITS == 4 ? 4 : 8;
  static constexpr int SC = KSTEPS < SCMAX ? KSTEPS : SCMAX;  // steps per chunk
  static constexpr int NCH = KSTEPS / SC;                     // chunks per wave slice
  static constexpr int LO_BITS = BITS == 3 ? 2 : BITS;
  static constexpr int LW = SC * LO_BITS / 4;                 // main-plane words per lane per chunk
  static constexpr int HW = BITS == 3 ? SC / 4 : 0;           // 1-bit-plane words per lane per chunk
  static constexpr int CHUNK_WORDS = 16 * SC * BITS;          // 64 * SC * BITS / 4
  static_assert(KSTEPS % SC == 0, "slice must hold whole chunks");
  static_assert(LW >= 1, "lane owns at least a word");
  static_assert(BITS != 3 || HW >= 1, "int3 needs 4 steps per chunk");
};

template <int N>
__device__ inline void load_words(const uint32_t* p, uint32_t* dst) {
  if (N == 4) {
    uint4_t v = __builtin_nontemporal_load((const uint4_t*)p);
    dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
  } else if (N == 2) {
    uint2_t v = __builtin_nontemporal_load((const uint2_t*)p);
    dst[0] = v.x; dst[1] = v.y;
  } else {
    dst[0] = __builtin_nontemporal_load(p);
  }
}

// Packed words of one unit (16 channels x this wave's K-slice) as one lane holds them.
template <int BITS, int KSTEPS>
struct UnitBuf {
  using S = Shape<BITS, KSTEPS>;
  uint32_t lo[S::NCH * S::LW];
  uint32_t hi[BITS == 3 ? S::NCH * S::HW : 1];
};

// What a wave needs to know about a unit besides its packed words (all wave-uniform
// except sc/bi, which belong to the lane's output channel).
struct UnitMeta {
  int pair, col, e;
  uint16_t sc, bi;  // fp16 scale and bias of the lane's channel, untouched until the epilogue
  bool active;
};

constexpr int LDS_TOKENS = 1024;  // perm and gate are staged in LDS up to this many tokens
#ifndef MOQE_MIN_WAVES
#define MOQE_MIN_WAVES 2  // waves per SIMD the register budget is sized for
#endif

template <int BITS, int KSTEPS>
__global__ __launch_bounds__(WG_THREADS, MOQE_MIN_WAVES) void ffn_decode_kernel(FfnArgs a) {
  using S = Shape<BITS, KSTEPS>;
  using Buf = UnitBuf<BITS, KSTEPS>;
  constexpr bool HOIST = true;  // every width leaves some exponent bias in the K-sum

  __shared__ int s_seg[MAX_E + 1];   // seg_offsets
  __shared__ int s_incl[MAX_E];      // inclusive prefix of token tiles per expert (E > 64 only)
  __shared__ int s_perm[LDS_TOKENS];
  __shared__ float s_gate[LDS_TOKENS];
  __shared__ float4_t s_red[2][WG_WAVES][64];
  constexpr int STAGE_ROWS = 4;                 // pairs with at most this many rows stage them in LDS
  constexpr int ROW_PIECES = KSTEPS * 4 + 4;    // 16-byte pieces per staged row slice, padded by 64 bytes
  __shared__ uint4_t s_x[WG_WAVES][STAGE_ROWS][ROW_PIECES];

  STAMP(0);
  UnpackConsts<BITS> uc;
  uc.init();
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = uniform_i32(tid >> 6);
  const int grp = lane >> 4;  // MFMA row group (k sub-block for A/B, token quad for D)
  const int j = lane & 15;    // token row for A, channel for B and D
  const int E = a.E;
  const bool small_e = E <= 64;
  const bool lds_tokens = a.T <= LDS_TOKENS;

  // ---- one round trip: routing tables into LDS ----
  for (int e = tid; e <= E; e += WG_THREADS) s_seg[e] = a.seg_offsets[e];
  if (lds_tokens) {
    for (int t = tid; t < a.T; t += WG_THREADS) {
      s_perm[t] = a.perm[t];
      if (a.mode == 1) s_gate[t] = a.gate[t];
    }
  }
  __syncthreads();

  // ---- token tiles per expert and their inclusive prefix (expert -> first pair) ----
  // E <= 64: each wave keeps the prefix in registers (lane e); else wave 0 scans into LDS.
  int my_tiles = 0, my_incl = 0;
  int P;
  if (small_e) {
    if (lane < E) {
      const int n = s_seg[lane + 1] - s_seg[lane];
      my_tiles = (n >= a.min_tokens && n < a.max_tokens) ? (n + 15) >> 4 : 0;
    }
    my_incl = my_tiles;
    for (int off = 1; off < 64; off <<= 1) {
      const int o = __shfl_up(my_incl, off, 64);
      if (lane >= off) my_incl += o;
    }
    P = __builtin_amdgcn_readlane(my_incl, 63);
  } else {
    if (wave == 0) {
      int carry = 0;
      for (int eg = 0; eg < E; eg += 64) {
        const int e = eg + lane;
        int v = 0;
        if (e < E) {
          const int n = s_seg[e + 1] - s_seg[e];
          v = (n >= a.min_tokens && n < a.max_tokens) ? (n + 15) >> 4 : 0;
        }
        for (int off = 1; off < 64; off <<= 1) {
          const int o = __shfl_up(v, off, 64);
          if (lane >= off) v += o;
        }
        if (e < E) s_incl[e] = carry + v;
        carry += __shfl(v, 63, 64);
      }
    }
    __syncthreads();
    P = s_incl[E - 1];
  }
  P = uniform_i32(P);
  STAMP(1);

  // ---- this workgroup's share of the units, teams take them round-robin ----
  const int CT = a.N >> 4;
  const int U = P * CT;
  const int ksplit = a.ksplit;
  const int teams = WG_WAVES / ksplit;
  const int team = wave / ksplit;
  const int ks = wave % ksplit;
  const int G = (int)gridDim.x, bid = (int)blockIdx.x;
  const int ubase = U / G, urem = U - ubase * G;
  const int u_begin = bid * ubase + min(bid, urem);
  const int u_end = u_begin + ubase + (bid < urem ? 1 : 0);
  const int nloop = (u_end - u_begin + teams - 1) / teams;
  if (nloop == 0) return;  // whole workgroup leaves together

  const int Q = a.K / (32 * S::SC);  // chunks per column tile
  const int64_t matrix_words = (int64_t)a.K * a.N * BITS / 32;

  // pair index -> expert (wave-uniform)
  auto expert_of = [&](int p) -> int {
    if (small_e) return __popcll(__ballot(lane < E && my_incl <= p));
    int lo = 0, hi = E - 1;
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (s_incl[mid] > p) hi = mid; else lo = mid + 1;
    }
    return uniform_i32(lo);
  };

  auto make_meta = [&](int it) -> UnitMeta {
    UnitMeta m;
    const int u = u_begin + it * teams + team;
    m.active = (it < nloop) && (u < u_end);
    m.pair = 0; m.col = 0; m.e = 0; m.sc = 0; m.bi = 0;
    if (m.active) {
      m.pair = u / CT;
      m.col = u - m.pair * CT;
      m.e = expert_of(m.pair);
      const uint32_t ch_off = (uint32_t)(16 * m.col + j);
      m.sc = (a.scales + (int64_t)m.e * a.N)[ch_off];
      m.bi = (a.bias + (int64_t)m.e * a.N)[ch_off];
    }
    return m;
  };

  auto chunk_ptr = [&](const UnitMeta& m, int ch) -> const uint32_t* {
    return a.codes + (int64_t)m.e * matrix_words + ((int64_t)m.col * Q + ks * S::NCH + ch) * S::CHUNK_WORDS;
  };
  const uint32_t lane_lo = (uint32_t)lane * S::LW, lane_hi = 64u * S::LW + (uint32_t)lane * S::HW;
  auto issue_chunk = [&](Buf& b, const uint32_t* cp, int ch) {
    load_words<S::LW>(cp + lane_lo, &b.lo[ch * S::LW]);
    if constexpr (BITS == 3) load_words<S::HW>(cp + lane_hi, &b.hi[ch * S::HW]);
  };

  // ---- per-pair state: the 16 token rows of this wave's K-slice as A fragments ----
  half8_t xf[KSTEPS];
  float4_t corr = {0, 0, 0, 0};
  int cur_pair = -1;
  int rows_valid = 0, row0 = 0;

  auto load_pair = [&](int p, int e) {
    cur_pair = p;
    int first;
    if (small_e) {
      first = __builtin_amdgcn_readlane(my_incl - my_tiles, e);
    } else {
      first = e > 0 ? s_incl[e - 1] : 0;
    }
    const int m = p - first;
    const int seg0 = s_seg[e];
    const int n_e = s_seg[e + 1] - seg0;
    row0 = seg0 + 16 * m;
    rows_valid = min(16, n_e - 16 * m);
    // lane (grp, j) holds row j, k = 32 s + 8 grp .. +7 of this wave's slice
    const bool av = j < rows_valid;
    const half8_t zero = {0, 0, 0, 0, 0, 0, 0, 0};
    const int64_t slice = (int64_t)ks * KSTEPS * 32;
    if (rows_valid <= STAGE_ROWS) {
      // Few rows (the decode case): fetch each row's slice with full-width coalesced loads
      // (16 bytes per lane), park it in this wave's LDS patch and pick the fragments from
      // there; 2 loads per row instead of one sparse load per step.
      uint4_t* patch = &s_x[wave][0][0];
      constexpr int PIECES = KSTEPS * 4;  // 16-byte pieces per row slice
#pragma unroll
      for (int r = 0; r < STAGE_ROWS; ++r) {
        if (r < rows_valid) {
          const int arow = a.mode == 0 ? (lds_tokens ? s_perm[row0 + r] : a.perm[row0 + r]) : (row0 + r);
          const uint4_t* src = (const uint4_t*)((const half_t*)a.a + (int64_t)arow * a.K + slice);
#pragma unroll
          for (int q0 = 0; q0 < PIECES; q0 += 64) {
            const int q = q0 + lane;
            if (q < PIECES) patch[r * ROW_PIECES + q] = src[q];
          }
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int s = 0; s < KSTEPS; ++s)
        xf[s] = av ? __builtin_bit_cast(half8_t, patch[j * ROW_PIECES + 4 * s + grp]) : zero;
      __builtin_amdgcn_wave_barrier();  // the patch may be rewritten by the next pair
    } else {
      int64_t arow = 0;
      if (av) arow = a.mode == 0 ? (lds_tokens ? s_perm[row0 + j] : a.perm[row0 + j]) : (row0 + j);
      const half_t* ap = (const half_t*)a.a + arow * a.K + slice + 8 * grp;
#pragma unroll
      for (int s = 0; s < KSTEPS; ++s) xf[s] = av ? *(const half8_t*)(ap + 32 * s) : zero;
    }
  };

  // bias + zero point carried by the unpacked values, summed against the rows
  auto pair_correction = [&]() {
    if constexpr (HOIST) {
      float4_t c0 = {0, 0, 0, 0}, c1 = {0, 0, 0, 0};
#pragma unroll
      for (int s = 0; s < KSTEPS; s += 2) {
        c0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(xf[s], bias_frag<BITS>(0), c0, 0, 0, 0);
        if (s + 1 < KSTEPS) c1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(xf[s + 1], bias_frag<BITS>(1), c1, 0, 0, 0);
      }
      corr = c0 + c1;
    }
  };

  // Consumes the unit in `b` chunk by chunk; as soon as a chunk's words are unpacked the
  // same registers are refilled with the matching chunk of unit `nx` (two units ahead).
  auto compute_unit = [&](Buf& b, const UnitMeta& m, const UnitMeta& nx) {
    float4_t acc0 = {0, 0, 0, 0}, acc1 = {0, 0, 0, 0};
    if (m.active) {
      if (m.pair != cur_pair) {
        load_pair(m.pair, m.e);
        pair_correction();
      }
      const uint32_t* nbase = nx.active ? chunk_ptr(nx, 0) : nullptr;
#pragma unroll
      for (int ch = 0; ch < S::NCH; ++ch) {
#ifdef MOQE_DBG_NOCOMPUTE
        {
          uint32_t x = 0;
          for (int q = 0; q < S::LW; ++q) x ^= b.lo[ch * S::LW + q];
          if (BITS == 3) for (int q = 0; q < S::HW; ++q) x ^= b.hi[ch * S::HW + q];
          acc0[0] += __builtin_bit_cast(float, x & 0x3fffffffu);
        }
        for (int s1 = 0; s1 < 0; ++s1) {
#else
#pragma unroll
        for (int s1 = 0; s1 < S::SC; ++s1) {
#endif
          const int s = ch * S::SC + s1;
          half8_t w;
          if constexpr (BITS == 4) {
            w = unpack4(b.lo[ch * S::LW + s1], uc);
          } else {
            const uint32_t d = b.lo[ch * S::LW + (s1 >> 1)];
            w = (s1 & 1) ? unpack2<1>(d, uc) : unpack2<0>(d, uc);
          }
          if (s & 1)
            acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(xf[s], w, acc1, 0, 0, 0);
          else
            acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(xf[s], w, acc0, 0, 0, 0);
          if constexpr (BITS == 3) {
            const uint32_t hd = b.hi[ch * S::HW + (s1 >> 2)];
            const half8_t wh = (s1 & 3) == 0 ? unpack1x4<0>(hd, uc) : (s1 & 3) == 1 ? unpack1x4<1>(hd, uc)
                             : (s1 & 3) == 2 ? unpack1x4<2>(hd, uc) : unpack1x4<3>(hd, uc);
            if (s & 1)
              acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(xf[s], wh, acc0, 0, 0, 0);
            else
              acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(xf[s], wh, acc1, 0, 0, 0);
          }
        }
        // the chunk's words are consumed: refill the same registers two units ahead
#ifndef MOQE_NO_ROLL
        if (nx.active) issue_chunk(b, nbase + ch * S::CHUNK_WORDS, ch);
#endif
      }
#ifdef MOQE_NO_ROLL
      if (nx.active) {
#pragma unroll
        for (int ch = 0; ch < S::NCH; ++ch) issue_chunk(b, nbase + ch * S::CHUNK_WORDS, ch);
      }
#endif
    } else if (nx.active) {
      const uint32_t* nbase = chunk_ptr(nx, 0);
#pragma unroll
      for (int ch = 0; ch < S::NCH; ++ch) issue_chunk(b, nbase + ch * S::CHUNK_WORDS, ch);
    }
    float4_t part = acc0 + acc1;
    if (HOIST) part = part - corr;
    return part;
  };

  int par = 0;
  auto finish_unit = [&](const UnitMeta& m, float4_t part) {
    if (ksplit > 1) {
      s_red[par][wave][lane] = part;
      __syncthreads();
      if (ks == 0) {
        for (int q = 1; q < ksplit; ++q) part = part + s_red[par][wave + q][lane];
      }
      par ^= 1;
    }
    if (!m.active || ks != 0) return;
    const float sc = (float)half_from_bits(m.sc);
    const float bi = (float)half_from_bits(m.bi);
    const int col = 16 * m.col + j;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      if (4 * grp + r < rows_valid) {
        float o = fmaf(part[r], sc, bi);
        if (a.mode == 0) {
          o = fmaxf(o, 0.0f);
          ((half_t*)a.h_out)[(int64_t)(row0 + 4 * grp + r) * a.N + col] = (half_t)o;
        } else {
          const int srow = row0 + 4 * grp + r;
          const int tk = lds_tokens ? s_perm[srow] : a.perm[srow];
          float v = (lds_tokens ? s_gate[tk] : a.gate[tk]) * o;
          const int64_t at = (int64_t)tk * a.N + col;
          if (a.residual) v += (float)((const half_t*)a.residual)[at];
          ((half_t*)a.y_out)[at] = (half_t)v;
        }
      }
    }
  };

  // ---- stream of units: two register buffers, refilled chunk by chunk ----
  Buf bufA, bufB;
  UnitMeta m0 = make_meta(0), m1 = make_meta(1);
  // the token rows go first (small, latency-critical), then the bulk weight loads
  if (m0.active) load_pair(m0.pair, m0.e);
  if (m0.active) {
    const uint32_t* cp = chunk_ptr(m0, 0);
#pragma unroll
    for (int ch = 0; ch < S::NCH; ++ch) issue_chunk(bufA, cp + ch * S::CHUNK_WORDS, ch);
  }
  if (m1.active) {
    const uint32_t* cp = chunk_ptr(m1, 0);
#pragma unroll
    for (int ch = 0; ch < S::NCH; ++ch) issue_chunk(bufB, cp + ch * S::CHUNK_WORDS, ch);
  }
  STAMP(2);
  if (m0.active) pair_correction();
#ifdef MOQE_PHASE_TRACE
  KEEP(xf[KSTEPS - 1][0]);
  STAMP(3);
#endif
  for (int it = 0; it < nloop; it += 2) {
    {
      const UnitMeta n0 = make_meta(it + 2);
      float4_t part = compute_unit(bufA, m0, n0);
#ifdef MOQE_PHASE_TRACE
      KEEP(part[0]);
      if (it == 0) STAMP(4);
#endif
      finish_unit(m0, part);
#ifdef MOQE_PHASE_TRACE
      if (it == 0) STAMP(5);
#endif
      m0 = n0;
    }
    if (it + 1 < nloop) {
      const UnitMeta n1 = make_meta(it + 3);
      float4_t part = compute_unit(bufB, m1, n1);
      finish_unit(m1, part);
      m1 = n1;
    }
  }
  STAMP(6);
}

template <int BITS, int KSTEPS>
hipError_t launch_one(const FfnArgs& a, int grid, hipStream_t stream) {
  hipLaunchKernelGGL((ffn_decode_kernel<BITS, KSTEPS>), dim3(grid), dim3(WG_THREADS), 0, stream, a);
  return hipGetLastError();
}

template <int BITS>
hipError_t launch_bits(const FfnArgs& a, int grid, hipStream_t stream) {
  switch (a.ksteps) {
    case 32: return launch_one<BITS, 32>(a, grid, stream);
    case 24: return launch_one<BITS, 24>(a, grid, stream);
    case 16: return launch_one<BITS, 16>(a, grid, stream);
    case 8: return launch_one<BITS, 8>(a, grid, stream);
    case 4: return launch_one<BITS, 4>(a, grid, stream);
    case 2:
      if constexpr (BITS != 3) return launch_one<BITS, 2>(a, grid, stream);
      return hipErrorInvalidValue;
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

bool moqe_pick_ksplit(int bits, int64_t K, int* ksteps, int* ksplit) {
  PackGeom g;
  if (!moqe_make_geom(bits, K, 16, &g)) return false;
  static const int cand[] = {32, 24, 16, 8, 4, 2};
  for (int ks : cand) {
    if (g.S % ks) continue;
    int r = g.S / ks;
    if (r != 1 && r != 2 && r != 4) continue;
    if (ks % g.SC) continue;
    if (bits == 3 && ks < 4) continue;
    *ksteps = ks;
    *ksplit = r;
    return true;
  }
  return false;
}

hipError_t moqe_launch_ffn_decode(const FfnArgs& a, int num_cus, hipStream_t stream) {
  const int grid = 2 * num_cus;  // two resident workgroups per CU (<= 256 VGPRs per wave)
  switch (a.bits) {
    case 4: return launch_bits<4>(a, grid, stream);
    case 3: return launch_bits<3>(a, grid, stream);
    case 2: return launch_bits<2>(a, grid, stream);
    default: return hipErrorInvalidValue;
  }
}
