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

// fp16 exponent patterns: (base << 16 | base) with a zero mantissa.
#define MAGIC_1024 0x64006400u
#define MAGIC_64 0x54005400u
#define MAGIC_32 0x50005000u
#define MAGIC_16 0x4C004C00u
#define MAGIC_8 0x48004800u
#define MAGIC_4 0x44004400u

// ---- int4: one word per step; exact (bias removed with a packed subtract) ----
// word bit position of code i (i = k % 8): 16 (i & 1) + 4 (i >> 1)
__device__ inline half8_t unpack4(uint32_t d) {
  uint32_t d8 = d >> 8;
  uint32_t r0 = pk_sub(and_or(d, 0x000F000Fu, MAGIC_1024), 1032.0f);
  uint32_t r1 = pk_sub(and_or(d, 0x00F000F0u, MAGIC_64), 72.0f);
  uint32_t r2 = pk_sub(and_or(d8, 0x000F000Fu, MAGIC_1024), 1032.0f);
  uint32_t r3 = pk_sub(and_or(d8, 0x00F000F0u, MAGIC_64), 72.0f);
  return frag_from_words(r0, r1, r2, r3);
}

// ---- int2: one word per two steps.  Fields are left with their exponent bias
// (value = base + u); the bias and the zero point are removed after the K-sum
// through bias_frag2(): sum_k a_k (base_k + u_k) - sum_k a_k (base_k + 2).
// even step: fields at bits 0,2,4,6 of each half; odd step: bits 8,10,12,14.
template <int PARITY>
__device__ inline half8_t unpack2(uint32_t d) {
  if (PARITY == 0) {
    uint32_t dl = d << 4;
    uint32_t r0 = and_or(dl, 0x00300030u, MAGIC_64);  // bits 0-1 -> 4-5
    uint32_t r1 = and_or(dl, 0x00C000C0u, MAGIC_16);  // bits 2-3 -> 6-7
    uint32_t r2 = and_or(d, 0x00300030u, MAGIC_64);   // bits 4-5
    uint32_t r3 = and_or(d, 0x00C000C0u, MAGIC_16);   // bits 6-7
    return frag_from_words(r0, r1, r2, r3);
  } else {
    uint32_t dr = d >> 6;
    uint32_t r0 = and_or(d, 0x03000300u, MAGIC_4);    // bits 8-9
    uint32_t r1 = and_or(dr, 0x00300030u, MAGIC_64);  // bits 10-11 -> 4-5
    uint32_t r2 = and_or(dr, 0x00C000C0u, MAGIC_16);  // bits 12-13 -> 6-7
    uint32_t r3 = and_or(dr, 0x03000300u, MAGIC_4);   // bits 14-15 -> 8-9
    return frag_from_words(r0, r1, r2, r3);
  }
}

// ---- int3 high plane: one word per four steps, one bit per code, worth 4.
// step ss (0..3) owns bits 4 ss .. 4 ss + 3 of each half; they are moved to
// mantissa bits 6..9 where, with bases 64, 32, 16, 8, a set bit adds exactly 4.
template <int SS>
__device__ inline half8_t unpack1x4(uint32_t d) {
  uint32_t v = SS == 0 ? (d << 6) : SS == 1 ? (d << 2) : SS == 2 ? (d >> 2) : (d >> 6);
  uint32_t r0 = and_or(v, 0x00400040u, MAGIC_64);
  uint32_t r1 = and_or(v, 0x00800080u, MAGIC_32);
  uint32_t r2 = and_or(v, 0x01000100u, MAGIC_16);
  uint32_t r3 = and_or(v, 0x02000200u, MAGIC_8);
  return frag_from_words(r0, r1, r2, r3);
}

// Constant B fragment holding, per code position, the amount the unpacked value
// exceeds the signed code: exponent bias(es) + zero point.
template <int BITS>
__device__ inline half8_t bias_frag(int parity) {
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

template <int BITS, int KSTEPS>
struct UnitBuf {
  using S = Shape<BITS, KSTEPS>;
  uint32_t lo[S::NCH * S::LW];
  uint32_t hi[BITS == 3 ? S::NCH * S::HW : 1];
  uint16_t sc, bi;
  int pair, col;  // wave-uniform
};

template <int BITS, int KSTEPS>
__global__ __launch_bounds__(WG_THREADS, 2) void ffn_decode_kernel(FfnArgs a) {
  using S = Shape<BITS, KSTEPS>;
  using Buf = UnitBuf<BITS, KSTEPS>;
  constexpr bool HOIST = BITS != 4;

  __shared__ int s_incl[MAX_E];
  __shared__ float4_t s_red[2][WG_WAVES][64];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = uniform_i32(tid >> 6);
  const int grp = lane >> 4;  // MFMA row group (k sub-block for A/B, token quad for D)
  const int j = lane & 15;    // token row for A, channel for B and D

  // ---- token tiles per expert, inclusive prefix (expert -> first pair) ----
  for (int e = tid; e < a.E; e += WG_THREADS) {
    int n = a.seg_offsets[e + 1] - a.seg_offsets[e];
    s_incl[e] = (n >= a.min_tokens && n < a.max_tokens) ? (n + 15) >> 4 : 0;
  }
  __syncthreads();
  if (wave == 0) {
    int carry = 0;
    for (int eg = 0; eg < a.E; eg += 64) {
      int e = eg + lane;
      int v = (e < a.E) ? s_incl[e] : 0;
      for (int off = 1; off < 64; off <<= 1) {
        int o = __shfl_up(v, off, 64);
        if (lane >= off) v += o;
      }
      if (e < a.E) s_incl[e] = carry + v;
      carry += __shfl(v, 63, 64);
    }
  }
  __syncthreads();

  const int P = s_incl[a.E - 1];
  const int CT = a.N >> 4;
  const int64_t U = (int64_t)P * CT;
  const int ksplit = a.ksplit;
  const int teams = WG_WAVES / ksplit;
  const int team = wave / ksplit;
  const int ks = wave % ksplit;
  const int64_t u_begin = U * blockIdx.x / gridDim.x;
  const int64_t u_end = U * (blockIdx.x + 1) / gridDim.x;
  const int nloop = (int)((u_end - u_begin + teams - 1) / teams);
  if (nloop == 0) return;  // whole workgroup leaves together

  const int Q = a.K / (32 * S::SC);  // chunks per column tile
  const int64_t matrix_words = (int64_t)a.K * a.N * BITS / 32;

  // ---- per-pair state ----
  half8_t xf[KSTEPS];
  float4_t corr = {0, 0, 0, 0};
  int cur_pair = -1;
  int seg0 = 0, rows_valid = 0, cur_e = 0, row0 = 0;
  int tok[4] = {0, 0, 0, 0};
  float gt[4] = {0, 0, 0, 0};

  auto expert_of = [&](int p) -> int {
    int lo = 0, hi = a.E - 1;
    while (lo < hi) {
      int mid = (lo + hi) >> 1;
      if (s_incl[mid] > p) hi = mid; else lo = mid + 1;
    }
    return uniform_i32(lo);
  };

  auto load_unit = [&](Buf& b, int64_t u) {
    const int p = (int)(u / CT), c = (int)(u % CT);
    const int e = expert_of(p);
    b.pair = p;
    b.col = c;
    const uint32_t* base = a.codes + (int64_t)e * matrix_words + ((int64_t)c * Q + ks * S::NCH) * S::CHUNK_WORDS;
#pragma unroll
    for (int ch = 0; ch < S::NCH; ++ch) {
      load_words<S::LW>(base + ch * S::CHUNK_WORDS + lane * S::LW, &b.lo[ch * S::LW]);
      if (BITS == 3)
        load_words<(BITS == 3 ? S::HW : 1)>(base + ch * S::CHUNK_WORDS + 64 * S::LW + lane * S::HW, &b.hi[ch * S::HW]);
    }
    b.sc = a.scales[(int64_t)e * a.N + 16 * c + j];
    b.bi = a.bias[(int64_t)e * a.N + 16 * c + j];
  };

  auto load_pair = [&](int p) {
    cur_pair = p;
    const int e = expert_of(p);
    cur_e = e;
    const int first = e > 0 ? s_incl[e - 1] : 0;
    const int m = p - first;
    seg0 = a.seg_offsets[e];
    const int n_e = a.seg_offsets[e + 1] - seg0;
    row0 = seg0 + 16 * m;
    rows_valid = min(16, n_e - 16 * m);
    // A fragments: lane (grp, j) holds row j, k = 32 s + 8 grp .. +7 of this wave's slice
    const bool av = j < rows_valid;
    int64_t arow = 0;
    if (av) arow = a.mode == 0 ? a.perm[row0 + j] : (row0 + j);
    const half_t* ap = (const half_t*)a.a + arow * a.K + (int64_t)ks * KSTEPS * 32 + 8 * grp;
    const half8_t zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) xf[s] = av ? *(const half8_t*)(ap + 32 * s) : zero;
    // output rows of this lane: 4 grp + r
    if (a.mode == 1) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const bool v = 4 * grp + r < rows_valid;
        tok[r] = v ? a.perm[row0 + 4 * grp + r] : 0;
        gt[r] = v ? a.gate[tok[r]] : 0.0f;
      }
    }
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

  auto compute_unit = [&](Buf& b, bool active) {
    float4_t acc0 = {0, 0, 0, 0}, acc1 = {0, 0, 0, 0};
    if (active) {
      if (b.pair != cur_pair) load_pair(b.pair);
#pragma unroll
      for (int ch = 0; ch < S::NCH; ++ch) {
#pragma unroll
        for (int s1 = 0; s1 < S::SC; ++s1) {
          const int s = ch * S::SC + s1;
          half8_t w;
          if (BITS == 4) {
            w = unpack4(b.lo[ch * S::LW + s1]);
          } else {
            const uint32_t d = b.lo[ch * S::LW + (s1 >> 1)];
            w = (s1 & 1) ? unpack2<1>(d) : unpack2<0>(d);
          }
          if (s & 1)
            acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(xf[s], w, acc1, 0, 0, 0);
          else
            acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(xf[s], w, acc0, 0, 0, 0);
          if (BITS == 3) {
            const uint32_t hd = b.hi[ch * S::HW + (s1 >> 2)];
            half8_t wh = (s1 & 3) == 0 ? unpack1x4<0>(hd) : (s1 & 3) == 1 ? unpack1x4<1>(hd)
                       : (s1 & 3) == 2 ? unpack1x4<2>(hd) : unpack1x4<3>(hd);
            if (s & 1)
              acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(xf[s], wh, acc0, 0, 0, 0);
            else
              acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(xf[s], wh, acc1, 0, 0, 0);
          }
        }
      }
    }
    float4_t part = acc0 + acc1;
    if (HOIST) part = part - corr;
    return part;
  };

  int par = 0;
  auto finish_unit = [&](Buf& b, float4_t part, bool active) {
    if (ksplit > 1) {
      s_red[par][wave][lane] = part;
      __syncthreads();
      if (ks == 0) {
        for (int q = 1; q < ksplit; ++q) part = part + s_red[par][wave + q][lane];
      }
      par ^= 1;
    }
    if (!active || ks != 0) return;
    const float sc = (float)half_from_bits(b.sc);
    const float bi = (float)half_from_bits(b.bi);
    const int col = 16 * b.col + j;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      if (4 * grp + r < rows_valid) {
        float o = fmaf(part[r], sc, bi);
        if (a.mode == 0) {
          o = fmaxf(o, 0.0f);
          ((half_t*)a.h_out)[(int64_t)(row0 + 4 * grp + r) * a.N + col] = (half_t)o;
        } else {
          float v = gt[r] * o;
          const int64_t at = (int64_t)tok[r] * a.N + col;
          if (a.residual) v += (float)((const half_t*)a.residual)[at];
          ((half_t*)a.y_out)[at] = (half_t)v;
        }
      }
    }
  };

  // ---- software pipeline over this team's units: two buffers ----
  Buf bufA, bufB;
  auto unit_of = [&](int it) -> int64_t { return u_begin + (int64_t)it * teams + team; };
  if (unit_of(0) < u_end) load_unit(bufA, unit_of(0));
  for (int it = 0; it < nloop; it += 2) {
    const bool a0 = unit_of(it) < u_end;
    const bool a1 = (it + 1 < nloop) && unit_of(it + 1) < u_end;
    if (a1) load_unit(bufB, unit_of(it + 1));
    {
      float4_t part = compute_unit(bufA, a0);
      finish_unit(bufA, part, a0);
    }
    if (it + 1 < nloop) {
      if (it + 2 < nloop && unit_of(it + 2) < u_end) load_unit(bufA, unit_of(it + 2));
      float4_t part = compute_unit(bufB, a1);
      finish_unit(bufB, part, a1);
    }
  }
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
