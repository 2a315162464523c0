// Decode-step MoE layer kernel: (optionally) top-1 routing, then the two expert FFN
// contractions for few tokens per expert as a fused dequantize-in-register grouped GEMM,
// bound by the packed weight bytes it reads.
//
//   out[rows of expert e, n] = epilogue( sum_k a[row, k] * (Q_e[k, n] * s_e[n]) + b_e[n] )
// (paper Sec. 2.1 two-layer FFN, App. A dequantization A' = Q s; the per-channel scale
// multiplies the finished K-sum because it does not depend on k; App. B top-1 gating).
//
// Work decomposition of one contraction
//   pair  = (expert e, tile of 4 routed tokens of e)        P pairs, found on device
//   unit  = (pair, column tile of 16 output channels)       U = P * N/16
//   team  = `ksplit` waves of a workgroup sharing one unit along K; each wave parks its
//           K-slice (32*KSTEPS columns) of the pair's token rows in LDS, reads one MFMA
//           A-fragment per step from there (rows 4..15 of the fragment come from a row of
//           zeros) and streams the unit's packed codes with 16-byte loads, two units in
//           flight, refilled chunk by chunk as they are consumed.  Keeping the rows out of
//           the register file is what lets three waves share a SIMD without spilling.
//   Units are split evenly over the persistent grid; inside a workgroup the teams take
//   them round-robin.  Codes go straight from registers into v_mfma_f32_16x16x32_f16 as
//   the B operand (16 channels x 32 rows); see moqe_unpack.h.
//
// One launch can run several phases back to back: router -> FFN1 -> FFN2.  A phase waits
// for exactly the data it consumes (all workgroups are resident: the grid is sized from the
// occupancy query).  Waits are bounded: a wait that does not complete sets the error word
// and every workgroup still runs to its end.
#include "moqe_dev.h"
#include "moqe_kernels.h"
#include "moqe_unpack.h"

#define MOQE_MIN_WAVES 3  // waves per SIMD the register and LDS budgets are sized for

namespace {

constexpr int WG_THREADS = 256;
constexpr int WG_WAVES = 4;
constexpr int MAX_E = 1024;
constexpr int LDS_TOKENS = 256;         // perm and gate are staged in LDS up to this many tokens
constexpr int TILE_ROWS = 4;            // token rows of a pair (the MFMA's other 12 rows are zero)
constexpr int FUSED_ROUTE_TOKENS = 64;  // the in-kernel router handles one wave of tokens
constexpr unsigned SPIN_LIMIT = 1u << 18;
// Sync words of the workspace head: launch epoch, start counter, bytes of h the last writer
// left in each of the two h buffers (everything beyond is zero), error flag.
enum { SY_EPOCH = 0, SY_START = 32, SY_EXT = 64, SY_ERR = 160 };

// Packed words of one unit (16 channels x this wave's K-slice) as one lane holds them.
template <int BITS, int KSTEPS>
struct UnitBuf {
  using S = Shape<BITS, KSTEPS>;
  uint32_t lo[S::NCH * S::LW];
  uint32_t hi[S::FB == 3 ? S::NCH * S::HW : 1];
};

// What a wave needs to know about a unit besides its packed words (all wave-uniform
// except sc/bi, which belong to the lane's output channel).
struct UnitMeta {
  int pair, col, e;
  const uint32_t* cp;  // first packed word of this wave's K-slice of the unit
  uint16_t sc, bi;     // fp16 scale and bias of the lane's channel, untouched until the epilogue
  bool active;         // an inactive unit has cp == nullptr and loads nothing
  int phase;
};

// Lanes holding the same key, as a 64-bit mask (nb = number of key bits).
__device__ inline uint64_t match_any(int key, int nb) {
  uint64_t m = ~0ull;
  for (int b = 0; b < nb; ++b) {
    const bool bit = (key >> b) & 1;
    const uint64_t bb = __ballot(bit);
    m &= bit ? bb : ~bb;
  }
  return m;
}

// ---- data that crosses a phase boundary inside one launch ---------------------------
// The router's results and the hidden activations h are written with device-scope stores
// and read with device-scope loads: they go past the per-XCD L2 to memory, so no
// cache-wide write-back or invalidate is needed (those cost several microseconds each on
// this part).  There are no grid barriers either: every datum says by itself whether it
// has been written.  A router result carries the launch's tag.  h is stored as its fp16
// bit pattern plus one (h >= 0 after ReLU, so the pattern is below 0x7C01 and never wraps)
// into a buffer that starts all zero: a zero half means "not there yet", and a consumer
// re-reads its rows until none is left.  Every wait is bounded: on timeout the error word
// is set and the kernel runs on to its end (its results are then garbage).
template <class T>
__device__ inline void store_coherent(T* p, T v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <class T>
__device__ inline T load_coherent(const T* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline uint4_t load16_coherent(const uint4_t* p) {
  const unsigned long long* q = (const unsigned long long*)p;
  const unsigned long long a = load_coherent(q), b = load_coherent(q + 1);
  return uint4_t{(uint32_t)a, (uint32_t)(a >> 32), (uint32_t)b, (uint32_t)(b >> 32)};
}
// True if any 16-bit half of the word is zero.
__device__ inline bool has_zero_half(uint32_t v) { return ((v - 0x00010001u) & ~v & 0x80008000u) != 0u; }

// Waves per SIMD the register budget is sized for: int8 holds two words per step, so its long
// slices (two units of 2 x 24 or 2 x 32 words in flight) need the registers of two waves.
constexpr int min_waves(int bits, int ksteps) { return (bits == 8 && ksteps > 16) ? 2 : MOQE_MIN_WAVES; }

template <int BITS, int KSTEPS, int PM>
__global__ __launch_bounds__(WG_THREADS, min_waves(BITS, KSTEPS)) void moe_decode_kernel(DecodeArgs A) {
  // PM != 0 fixes the phase mask at compile time (the single-contraction launches), so that
  // everything the other phases need drops out of the code
  const int phase_mask = PM ? PM : A.phase_mask;
  using S = Shape<BITS, KSTEPS>;
  using Buf = UnitBuf<BITS, KSTEPS>;
  constexpr int ROW_PIECES = KSTEPS * 4 + 4;  // 16-byte pieces per staged row slice, padded by 64 bytes
  constexpr int ZERO_ROW = WG_WAVES * TILE_ROWS;

  __shared__ int s_seg[MAX_E + 1];  // seg_offsets
  __shared__ int s_perm[LDS_TOKENS];
  __shared__ float s_gate[LDS_TOKENS];
  __shared__ float4_t s_red[2][WG_WAVES][16];
  // token rows: TILE_ROWS per wave, then one row of zeros for the unused rows of a fragment
  __shared__ uint4_t s_x[WG_WAVES * TILE_ROWS + 1][ROW_PIECES];
  // router: per-wave partial logits, then the logits; afterwards (E > 64 only) the inclusive
  // prefix of token tiles per expert
  __shared__ float4_t s_multi[(WG_WAVES + 1) * 256 / 4];
  float(*const s_route)[256] = reinterpret_cast<float(*)[256]>(s_multi);
  int* const s_incl = reinterpret_cast<int*>(s_multi);
  static_assert(sizeof(s_multi) >= MAX_E * sizeof(int), "prefix table does not fit");
  constexpr int STASH_UNITS = 4;  // finished units a wave parks before writing them out
  __shared__ float4_t s_out[WG_WAVES][STASH_UNITS][16];
  __shared__ int s_ometa[WG_WAVES][STASH_UNITS][4];
  __shared__ int s_share[2][4];  // per contraction: this workgroup's first unit, end, iterations
  UnpackConsts<BITS> uc;
  uc.init();
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = uniform_i32(tid >> 6);
  const int grp = lane >> 4;  // MFMA row group (k sub-block for A/B, token quad for D)
  const int j = lane & 15;    // token row for A, channel for B and D
  const int E = A.E, T = A.T;
  const int G = (int)gridDim.x, bid = (int)blockIdx.x;
  const bool small_e = E <= 64;
  const bool lds_tokens = T <= LDS_TOKENS;
  const bool multi_phase = (phase_mask & (phase_mask - 1)) != 0;
  // FFN1 and FFN2 in one launch: h travels through the workspace as a dataflow (see below)
  const bool chained = (phase_mask & 6) == 6;

  // ---- launch epoch (multi-phase launches only) ----
  // The workspace counts launches.  Every workgroup reads the count, then checks in at the
  // start counter; whoever checks in last knows that all have read it and bumps it for the
  // next launch.  Nobody waits for this.  The epoch tags the router's results and picks
  // which of the two h buffers this launch fills (the other one is cleared for the next).
  __shared__ unsigned s_epoch, s_ext_other;
  unsigned epoch = 0, start_old = 0, ext_other = 0;
  if (multi_phase && wave == 0) {  // the other waves get these below
    epoch = load_coherent(&A.sync[SY_EPOCH]);
    const unsigned e0 = load_coherent(&A.sync[SY_EXT]), e1 = load_coherent(&A.sync[SY_EXT + 1]);
    ext_other = (epoch & 1u) ? e0 : e1;
  }
  const unsigned tag = epoch + 1u;

  // =========================== routing tables ===========================
  if (phase_mask & 1) {
    // ---- router: workgroup t < T scores token t (E a multiple of 8, E <= 256, T <= 64) ----
    if (bid < T) {
      const half_t* xr = (const half_t*)A.x + (int64_t)bid * A.d_route;
      const half_t* wg = (const half_t*)A.w_gate;
      const int d = A.d_route;
      int EGP = 1;
      while (EGP < (E >> 3)) EGP <<= 1;
      const int EG = E >> 3, KQ = WG_THREADS / EGP;
      const int eg = tid % EGP, kq = tid / EGP;
      float acc[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] = 0.0f;
      constexpr int BATCH = 16;
      if (eg < EG) {
        for (int k0 = kq; k0 < d; k0 += KQ * BATCH) {
          uint4_t w[BATCH];
          half_t xv[BATCH];
#pragma unroll
          for (int i = 0; i < BATCH; ++i) {
            const int k = k0 + i * KQ;
            const bool ok = k < d;
            w[i] = ok ? *(const uint4_t*)(wg + (int64_t)k * E + 8 * eg) : uint4_t{0, 0, 0, 0};
            xv[i] = ok ? xr[k] : (half_t)0;
          }
#pragma unroll
          for (int i = 0; i < BATCH; ++i) {
            const half8_t h = __builtin_bit_cast(half8_t, w[i]);
            const float xf32 = (float)xv[i];
#pragma unroll
            for (int q = 0; q < 8; ++q) acc[q] = fmaf(xf32, (float)h[q], acc[q]);
          }
        }
      }
      for (int off = 32; off >= EGP; off >>= 1) {
#pragma unroll
        for (int q = 0; q < 8; ++q) acc[q] += __shfl_xor(acc[q], off, 64);
      }
      if (lane < EGP && eg < EG) {
#pragma unroll
        for (int q = 0; q < 8; ++q) s_route[wave][eg * 8 + q] = acc[q];
      }
      __syncthreads();
      for (int e = tid; e < E; e += WG_THREADS) {
        float sum = 0.0f;
        for (int w = 0; w < WG_WAVES; ++w) sum += s_route[w][e];
        s_route[WG_WAVES][e] = sum;
      }
      __syncthreads();
      if (wave == 0) {
        // wavefront-level argmax (lowest index on ties) and softmax probability, with the same
        // comparisons and the same order of additions as the router kernels
        int bidx;
        float g;
        wave_pick(s_route[WG_WAVES], E, &bidx, &g);
        if (lane == 0) {
          A.expert_idx[bid] = bidx;
          A.gate[bid] = g;
          // the result other workgroups wait for: two words, each carrying this launch's tag
          store_coherent(&A.route_entries[2 * bid], ((unsigned long long)tag << 32) | (unsigned)bidx);
          store_coherent(&A.route_entries[2 * bid + 1],
                         ((unsigned long long)tag << 32) | __builtin_bit_cast(unsigned, g));
        }
      }
    }
    // ---- every workgroup collects the T results and rebuilds the dispatch tables ----
    if (wave == 0) {
      const bool valid = lane < T;
      unsigned long long w0 = 0, w1 = 0;
      for (unsigned it = 0;; ++it) {
        if (valid) {
          w0 = load_coherent(&A.route_entries[2 * lane]);
          w1 = load_coherent(&A.route_entries[2 * lane + 1]);
        }
        const bool ready = !valid || ((unsigned)(w0 >> 32) == tag && (unsigned)(w1 >> 32) == tag);
        if (__all(ready)) break;
        if (it > SPIN_LIMIT || load_coherent(&A.sync[SY_ERR]) != 0u) {
          store_coherent(&A.sync[SY_ERR], 1u);
          break;
        }
        __builtin_amdgcn_s_sleep(8);
      }
      const int key = valid ? min((int)(unsigned)w0, E - 1) : E;
      const float g = valid ? __builtin_bit_cast(float, (unsigned)w1) : 0.0f;
      int nb = 0;
      while ((1 << nb) <= E) ++nb;
      const uint64_t m = match_any(key, nb);
      const int rank = __popcll(m & ((1ull << lane) - 1ull));
      const bool leader = (__ffsll((long long)m) - 1) == lane;
      for (int e = lane; e <= E; e += 64) s_seg[e] = 0;
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      if (valid && leader) s_seg[key] = __popcll(m);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      int carry = 0;
      for (int eg = 0; eg < E; eg += 64) {
        const int e = eg + lane;
        const int v = (e < E) ? s_seg[e] : 0;
        int inc = v;
        for (int off = 1; off < 64; off <<= 1) {
          const int o = __shfl_up(inc, off, 64);
          if (lane >= off) inc += o;
        }
        __builtin_amdgcn_wave_barrier();
        if (e < E) s_seg[e] = carry + inc - v;
        carry += __shfl(inc, 63, 64);
      }
      if (lane == 0) s_seg[E] = T;
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      if (valid) {
        const int pos = s_seg[key] + rank;
        s_perm[pos] = lane;
        s_gate[lane] = g;
        if (bid == 0) A.perm[pos] = lane;
      }
      if (bid == 0) {
        for (int e = lane; e <= E; e += 64) A.seg_offsets[e] = s_seg[e];
      }
    }
    if (tid == 0) {
      s_epoch = epoch;
      s_ext_other = ext_other;
    }
    __syncthreads();
  } else {
    // ---- one round trip: the caller's routing tables into LDS ----
    for (int e = tid; e <= E; e += WG_THREADS) s_seg[e] = A.seg_offsets[e];
    if (lds_tokens) {
      for (int t = tid; t < T; t += WG_THREADS) {
        s_perm[t] = A.perm[t];
        if (A.gate) s_gate[t] = A.gate[t];
      }
    }
    if (tid == 0) {
      s_epoch = epoch;
      s_ext_other = ext_other;
    }
    __syncthreads();
  }
  epoch = s_epoch;
  ext_other = s_ext_other;
  uint16_t* const h_cur = A.h_base + (size_t)(epoch & 1u) * A.h_stride;

  // ---- token tiles per expert and their inclusive prefix (expert -> first pair) ----
  // E <= 64: each wave keeps the prefix in registers (lane e); else wave 0 scans into LDS.
  int my_tiles = 0, my_incl = 0;
  int P;
  if (small_e) {
    if (lane < E) {
      const int n = s_seg[lane + 1] - s_seg[lane];
      my_tiles = (n >= A.min_tokens && n < A.max_tokens) ? (n + TILE_ROWS - 1) / TILE_ROWS : 0;
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
          v = (n >= A.min_tokens && n < A.max_tokens) ? (n + TILE_ROWS - 1) / TILE_ROWS : 0;
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

  // the row of zeros, and this workgroup's share of each contraction's units
  for (int q = tid; q < ROW_PIECES; q += WG_THREADS) s_x[ZERO_ROW][q] = uint4_t{0, 0, 0, 0};
  if (tid < 2) {
    const int teams = WG_WAVES / max(1, A.ph[tid].ksplit);
    const int U = P * (A.ph[tid].N >> 4);
    const int ubase = U / G, urem = U - ubase * G;
    const int u_begin = bid * ubase + min(bid, urem);
    const int u_end = u_begin + ubase + (bid < urem ? 1 : 0);
    s_share[tid][0] = u_begin;
    s_share[tid][1] = u_end;
    s_share[tid][2] = (phase_mask & (2 << tid)) ? (u_end - u_begin + teams - 1) / teams : 0;
  }
  __syncthreads();

  int par = 0;

  // ---- the stream of units ----
  // Unit `it` of contraction `phz` as this wave sees it.  (Fetching a wave's first FFN2 units
  // while it still works on FFN1 was tried and lost: FFN2 cannot start before the slowest
  // FFN1 unit of its pair has delivered h, and the early FFN2 requests queue in front of
  // other waves' FFN1 requests.)
  auto make_meta = [&](int phz, int it) -> UnitMeta {
    UnitMeta m;
    m.active = false;
    m.pair = 0; m.col = 0; m.e = 0; m.sc = 0; m.bi = 0; m.cp = nullptr;
    m.phase = phz;
    const PhaseArgs& p = A.ph[phz];
    const int ksplit = p.ksplit, N = p.N, K = p.K;
    const int teams = WG_WAVES / ksplit, team = wave / ksplit, ks = wave % ksplit;
    const int u = uniform_i32(s_share[m.phase][0]) + it * teams + team;
    m.active = (it < uniform_i32(s_share[m.phase][2])) && (u < uniform_i32(s_share[m.phase][1]));
    const half_t *scales = nullptr, *bias = nullptr;
    if (m.active) {
      const int CT = N >> 4;
      m.pair = u / CT;
      m.col = u - m.pair * CT;
      m.e = expert_of(m.pair);
      scales = (const half_t*)p.scales + (int64_t)m.e * N;
      bias = (const half_t*)p.bias + (int64_t)m.e * N;
      const int Q = K / (32 * S::SC);  // chunks per column tile
      const int64_t matrix_words = (int64_t)K * N * moqe_field_bits(BITS) / 32;
      m.cp = p.codes + (int64_t)m.e * matrix_words + ((int64_t)m.col * Q + ks * S::NCH) * S::CHUNK_WORDS;
    }
    // issued whether or not the unit exists (an empty descriptor loads nothing)
    const uint32_t ch_off = (uint32_t)(16 * m.col + j) * 2u;
    const uint32_t row_bytes = m.active ? (uint32_t)N * 2u : 0u;
    m.sc = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(make_rsrc(scales, row_bytes), ch_off, 0, 0);
    m.bi = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(make_rsrc(bias, row_bytes), ch_off, 0, 0);
    return m;
  };
  constexpr uint32_t UNIT_BYTES = S::NCH * S::CHUNK_WORDS * 4;
  const uint32_t lane_lo = (uint32_t)lane * S::LW * 4, lane_hi = (64u * S::LW + (uint32_t)lane * S::HW) * 4;
  auto unit_rsrc = [&](const UnitMeta& m) -> rsrc_t { return make_rsrc(m.cp, m.active ? UNIT_BYTES : 0u); };
  auto issue_chunk = [&](Buf& b, rsrc_t r, int ch) {
    load_words<S::LW>(r, lane_lo + ch * S::CHUNK_WORDS * 4, &b.lo[ch * S::LW]);
    if constexpr (S::FB == 3) load_words<S::HW>(r, lane_hi + ch * S::CHUNK_WORDS * 4, &b.hi[ch * S::HW]);
  };
  auto issue_unit = [&](Buf& b, const UnitMeta& m) {
    const rsrc_t r = unit_rsrc(m);
#pragma unroll
    for (int ch = 0; ch < S::NCH; ++ch) issue_chunk(b, r, ch);
  };
  Buf bufA, bufB;  // two register buffers, refilled chunk by chunk

  // =========================== the contractions ===========================
  for (int phase = 0; phase < 2; ++phase) {
    if (!(phase_mask & (2 << phase))) continue;
    const PhaseArgs& ph = A.ph[phase];
    const int K = ph.K, N = ph.N, mode = ph.mode, ksplit = ph.ksplit;
    const bool produces_h = chained && phase == 0;  // output rows are consumed later in this launch
    const bool consumes_h = chained && phase == 1;  // input rows are written by workgroups of this launch
    const uint16_t* const a_rows = consumes_h ? h_cur : ph.a;
    uint16_t* const out_rows = produces_h ? h_cur : ph.out;
    const int ks = wave % ksplit;
    const int nl = uniform_i32(s_share[phase][2]);

    // ---- per-pair state: the 16 token rows of this wave's K-slice as A fragments ----
    float4_t corr = {0, 0, 0, 0};
    int cur_pair = -1;
    int rows_valid = 0, row0 = 0;
    int n_stash = 0;  // outputs parked in LDS by this wave

    // This lane's A-fragment of step s is afrag[4 * s]: row j of the patch, or the zero row.
    const uint4_t* afrag = &s_x[ZERO_ROW][grp];

    auto load_pair = [&](int p, int e, auto&& between) {
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
      row0 = seg0 + TILE_ROWS * m;
      rows_valid = min(TILE_ROWS, n_e - TILE_ROWS * m);
      const int64_t slice = (int64_t)ks * KSTEPS * 32;
      // Rows produced earlier in this launch (h) are read past the caches and are complete
      // only once no half of them is zero; their values are stored plus one.
      const bool coherent = mode == 1;
      // Each row's slice comes in with full-width coalesced loads (16 bytes per lane) and is
      // parked in this wave's LDS patch.
      uint4_t(*patch)[ROW_PIECES] = &s_x[wave * TILE_ROWS];
      constexpr int PIECES = KSTEPS * 4;       // 16-byte pieces per row slice
      constexpr int NPL = (PIECES + 63) / 64;  // pieces per lane and row
      __builtin_amdgcn_wave_barrier();         // earlier fragment reads of the patch are done
      for (unsigned it = 0;; ++it) {
        bool missing = false;
        uint4_t tmp[TILE_ROWS * NPL];
#pragma unroll
        for (int r = 0; r < TILE_ROWS; ++r) {
          if (r < rows_valid) {
            const int arow = mode == 0 ? (lds_tokens ? s_perm[row0 + r] : A.perm[row0 + r]) : (row0 + r);
            const uint4_t* src = (const uint4_t*)((const half_t*)a_rows + (int64_t)arow * K + slice);
#pragma unroll
            for (int i = 0; i < NPL; ++i) {
              const int q = 64 * i + lane;
              if (q < PIECES) tmp[r * NPL + i] = coherent ? load16_coherent(src + q) : src[q];
            }
          }
        }
        if (it == 0) between();  // requests that should queue right behind the rows
#pragma unroll
        for (int r = 0; r < TILE_ROWS; ++r) {
          if (r < rows_valid) {
#pragma unroll
            for (int i = 0; i < NPL; ++i) {
              const int q = 64 * i + lane;
              if (q < PIECES) {
                uint4_t v = tmp[r * NPL + i];
                if (consumes_h) {
                  missing |= has_zero_half(v.x) | has_zero_half(v.y) | has_zero_half(v.z) | has_zero_half(v.w);
                  v -= uint4_t{0x00010001u, 0x00010001u, 0x00010001u, 0x00010001u};
                }
                patch[r][q] = v;
              }
            }
          }
        }
        if (!consumes_h || !__any(missing)) break;
        if (it > SPIN_LIMIT || load_coherent(&A.sync[SY_ERR]) != 0u) {
          store_coherent(&A.sync[SY_ERR], 1u);
          break;
        }
        __builtin_amdgcn_s_sleep(8);
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      // lane (grp, j) reads row j, k = 32 s + 8 grp .. +7 of this wave's slice
      afrag = j < rows_valid ? &patch[j][grp] : &s_x[ZERO_ROW][grp];
      // bias + zero point carried by the unpacked values, summed against the rows
      // (log-scale codes unpack to their exact values: nothing to remove)
      if constexpr (!moqe_is_log(BITS)) {
        float4_t c0 = {0, 0, 0, 0}, c1 = {0, 0, 0, 0};
#pragma unroll
        for (int s = 0; s < KSTEPS; s += 2) {
          c0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, afrag[4 * s]), bias_frag<BITS>(0), c0,
                                                      0, 0, 0);
          if (s + 1 < KSTEPS)
            c1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, afrag[4 * s + 4]),
                                                        bias_frag<BITS>(1), c1, 0, 0, 0);
        }
        corr = c0 + c1;
      }
    };

    // Consumes the unit in `b` chunk by chunk; as soon as a chunk's words are unpacked the
    // same registers are refilled with the matching chunk of unit `nx` (two units ahead).
    auto compute_unit = [&](Buf& b, const UnitMeta& m, const UnitMeta& nx) {
      float4_t acc0 = {0, 0, 0, 0}, acc1 = {0, 0, 0, 0};
      const rsrc_t nr = unit_rsrc(nx);
      if (m.active) {
        if (m.pair != cur_pair) load_pair(m.pair, m.e, [] {});

#pragma unroll
        for (int ch = 0; ch < S::NCH; ++ch) {
#pragma unroll
          for (int s1 = 0; s1 < S::SC; ++s1) {
            const int s = ch * S::SC + s1;
            half8_t w;
            if constexpr (BITS == 8) {
              w = unpack8(b.lo[ch * S::LW + 2 * s1], b.lo[ch * S::LW + 2 * s1 + 1], uc);
            } else if constexpr (BITS == 4) {
              w = unpack4(b.lo[ch * S::LW + s1], uc);
            } else if constexpr (BITS == MOQE_LOG4) {
              w = unpack4_log(b.lo[ch * S::LW + s1], uc);
            } else if constexpr (BITS == MOQE_LOG3) {
              const uint32_t d = b.lo[ch * S::LW + (s1 >> 1)], hd = b.hi[ch * S::HW + (s1 >> 2)];
              w = (s1 & 3) == 0 ? unpack3_log<0>(d, hd, uc) : (s1 & 3) == 1 ? unpack3_log<1>(d, hd, uc)
                : (s1 & 3) == 2 ? unpack3_log<2>(d, hd, uc) : unpack3_log<3>(d, hd, uc);
            } else if constexpr (BITS == MOQE_LOG2) {
              const uint32_t d = b.lo[ch * S::LW + (s1 >> 1)];
              w = (s1 & 1) ? unpack2_log<1>(d, uc) : unpack2_log<0>(d, uc);
            } else {
              const uint32_t d = b.lo[ch * S::LW + (s1 >> 1)];
              w = (s1 & 1) ? unpack2<1>(d, uc) : unpack2<0>(d, uc);
            }
            // one accumulator suffices when a step's unpack outlasts the MFMA; int3 issues two
            // MFMAs per step and alternates between two
            const half8_t a = __builtin_bit_cast(half8_t, afrag[4 * s]);
            acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, w, acc0, 0, 0, 0);
            if constexpr (BITS == 3) {
              const uint32_t hd = b.hi[ch * S::HW + (s1 >> 2)];
              const half8_t wh = (s1 & 3) == 0 ? unpack1x4<0>(hd, uc) : (s1 & 3) == 1 ? unpack1x4<1>(hd, uc)
                               : (s1 & 3) == 2 ? unpack1x4<2>(hd, uc) : unpack1x4<3>(hd, uc);
              acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, wh, acc1, 0, 0, 0);
            }
          }
          // the chunk's words are consumed: refill the same registers two units ahead
          issue_chunk(b, nr, ch);
        }
      } else {
#pragma unroll
        for (int ch = 0; ch < S::NCH; ++ch) issue_chunk(b, nr, ch);
      }
      return acc0 + acc1 - corr;
    };

    auto finish_unit = [&](const UnitMeta& m, float4_t part) {
      // the pair's rows are rows 0..3 of the MFMA tile: lanes 0..15 hold them, one channel each
      if (ksplit > 1) {
        if (lane < 16) s_red[par][wave][lane] = part;
        __syncthreads();
        if (ks == 0 && lane < 16) {
          for (int q = 1; q < ksplit; ++q) part = part + s_red[par][wave + q][lane];
        }
        par ^= 1;
      }
      if (!m.active || ks != 0) return;
      const float sc = (float)half_from_bits(m.sc);
      const float bi = (float)half_from_bits(m.bi);
      float4_t o4;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        float o = fmaf(part[r], sc, bi);
        if (mode == 0) o = fmaxf(o, 0.0f);  // also turns a NaN into 0: the fp16 pattern is at most 0x7C00
        o4[r] = o;
      }
      // park the result; it is written out by flush_outputs()
      if (lane < 16) s_out[wave][n_stash][lane] = o4;
      if (lane == 0) {
        s_ometa[wave][n_stash][0] = row0;
        s_ometa[wave][n_stash][1] = rows_valid;
        s_ometa[wave][n_stash][2] = m.col;
      }
      ++n_stash;
    };

    // Writes the parked outputs.  Stores (and the few loads they need) are kept out of the
    // streaming loop: loads and stores share one in-order counter, so a store between the
    // streamed weight loads would make the next wait drain the whole load queue.
    auto flush_outputs = [&]() {
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      for (int u = 0; u < n_stash; ++u) {
        // lane (grp, j): row grp of the tile, channel j
        const float o = reinterpret_cast<const float*>(&s_out[wave][u][j])[grp];
        const int u_row0 = s_ometa[wave][u][0], u_rows = s_ometa[wave][u][1];
        const int col = 16 * s_ometa[wave][u][2] + j;
        if (grp < u_rows) {
          const int srow = u_row0 + grp;
          if (mode == 0) {
            const uint16_t hb = half_to_bits((half_t)o);
            if (produces_h)
              store_coherent(&out_rows[(int64_t)srow * N + col], (uint16_t)(hb + 1u));
            else
              out_rows[(int64_t)srow * N + col] = hb;
          } else {
            const int tk = lds_tokens ? s_perm[srow] : A.perm[srow];
            float v = (lds_tokens ? s_gate[tk] : A.gate[tk]) * o;
            const int64_t at = (int64_t)tk * N + col;
            if (ph.residual) v += (float)((const half_t*)ph.residual)[at];
            ((half_t*)out_rows)[at] = (half_t)v;
          }
        }
      }
      __builtin_amdgcn_wave_barrier();
      n_stash = 0;
    };

    // Order of the first requests.  Rows that are already in memory (x) go out before the
    // bulk weight loads: a CU's requests come back in order, so rows asked for after 16 KiB
    // of weights per wave would only arrive behind them.  Rows that are still being
    // produced by this launch (h) are asked for last: the weights do not depend on them and
    // stream in while they are awaited.
    UnitMeta m0 = make_meta(phase, 0), m1 = make_meta(phase, 1);
    if (!consumes_h && m0.active) {
      load_pair(m0.pair, m0.e, [&] {
        issue_unit(bufA, m0);
        issue_unit(bufB, m1);
      });
    } else {
      issue_unit(bufA, m0);
      issue_unit(bufB, m1);
    }
    for (int it = 0; it < nl; it += 2) {
      {
        const UnitMeta n0 = make_meta(phase, it + 2);
        const float4_t part = compute_unit(bufA, m0, n0);
        finish_unit(m0, part);
        m0 = n0;
      }
      {
        const UnitMeta n1 = make_meta(phase, it + 3);
        const float4_t part = compute_unit(bufB, m1, n1);
        finish_unit(m1, part);
        m1 = n1;
      }
      if (n_stash + 2 > STASH_UNITS) flush_outputs();
    }
    flush_outputs();
  }

  // ---- end of launch (multi-phase launches) ----
  // Kept at the end: device-scope stores and the contended counter would otherwise sit in
  // front of the streamed loads in this wave's in-order memory counter.
  if (chained) {
    // clear what its last writer left in the other h buffer: all zero = "not written yet"
    // for the launch after this one
    unsigned long long* other = (unsigned long long*)(A.h_base + (size_t)((epoch + 1u) & 1u) * A.h_stride);
    const size_t words = ext_other / 8;
    for (size_t i = (size_t)bid * WG_THREADS + tid; i < words; i += (size_t)G * WG_THREADS) store_coherent(&other[i], 0ull);
  }
  if (multi_phase) {
    // check in; whoever is last knows that every workgroup is done with this epoch's state
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's clearing stores are acknowledged
    __syncthreads();
    if (tid == 0) {
      start_old = __hip_atomic_fetch_add(&A.sync[SY_START], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (start_old == (unsigned)G - 1u) {
        store_coherent(&A.sync[SY_START], 0u);
        if (chained) {
          store_coherent(&A.sync[SY_EXT + (epoch & 1u)], A.h_bytes);
          store_coherent(&A.sync[SY_EXT + ((epoch + 1u) & 1u)], 0u);
        }
        store_coherent(&A.sync[SY_EPOCH], epoch + 1u);
      }
    }
  }
}

template <int BITS, int KSTEPS, int PM>
hipError_t launch_mask(const DecodeArgs& a, int num_cus, hipStream_t stream) {
  // Persistent grid: every workgroup must be resident at once (phases meet at grid-wide
  // counters), so the grid is what the occupancy query says fits, at most MOQE_MIN_WAVES
  // workgroups (of four waves: one wave per SIMD each) per CU.
  static int per_cu_of[64];  // asked once per device
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  if (per_cu_of[dev] == 0) {
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, moe_decode_kernel<BITS, KSTEPS, PM>, WG_THREADS, 0) != hipSuccess ||
        n < 1)
      n = 1;
    per_cu_of[dev] = n > min_waves(BITS, KSTEPS) ? min_waves(BITS, KSTEPS) : n;
  }
  const int per_cu = per_cu_of[dev];
  hipLaunchKernelGGL((moe_decode_kernel<BITS, KSTEPS, PM>), dim3(per_cu * num_cus), dim3(WG_THREADS), 0, stream, a);
  return hipGetLastError();
}

template <int BITS, int KSTEPS>
hipError_t launch_one(const DecodeArgs& a, int num_cus, hipStream_t stream) {
  if (a.phase_mask == 2) return launch_mask<BITS, KSTEPS, 2>(a, num_cus, stream);
  if (a.phase_mask == 4) return launch_mask<BITS, KSTEPS, 4>(a, num_cus, stream);
  return launch_mask<BITS, KSTEPS, 0>(a, num_cus, stream);
}

template <int BITS>
hipError_t launch_bits(const DecodeArgs& a, int num_cus, hipStream_t stream) {
  switch (a.ksteps) {
    case 32: return launch_one<BITS, 32>(a, num_cus, stream);
    case 24: return launch_one<BITS, 24>(a, num_cus, stream);
    case 16: return launch_one<BITS, 16>(a, num_cus, stream);
    case 8: return launch_one<BITS, 8>(a, num_cus, stream);
    case 4: return launch_one<BITS, 4>(a, num_cus, stream);
    case 2:
      if constexpr (moqe_field_bits(BITS) != 3) return launch_one<BITS, 2>(a, num_cus, stream);
      return hipErrorInvalidValue;
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

bool moqe_pick_ksplit(int bits, int64_t K, int* ksteps, int* ksplit) {
  PackGeom g;
  if (!moqe_make_geom(bits, K, 16, &g)) return false;
  // longest slice first; int8 (two words per step) prefers 16 steps, which still fit three waves
  // per SIMD
  static const int cand_default[] = {32, 24, 16, 8, 4, 2};
  static const int cand_int8[] = {16, 32, 24, 8, 4, 2};
  const int(&cand)[6] = bits == 8 ? cand_int8 : cand_default;
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

bool moqe_decode_can_route(int64_t T, int64_t d, int64_t E) {
  return T >= 1 && T <= FUSED_ROUTE_TOKENS && E >= 8 && E <= 256 && (E % 8) == 0 && d >= 8 && (d % 8) == 0;
}

hipError_t moqe_launch_decode(const DecodeArgs& a, int num_cus, hipStream_t stream) {
  switch (a.bits) {
    case 8: return launch_bits<8>(a, num_cus, stream);
    case 4: return launch_bits<4>(a, num_cus, stream);
    case MOQE_LOG4: return launch_bits<MOQE_LOG4>(a, num_cus, stream);
    case MOQE_LOG3: return launch_bits<MOQE_LOG3>(a, num_cus, stream);
    case MOQE_LOG2: return launch_bits<MOQE_LOG2>(a, num_cus, stream);
    case 3: return launch_bits<3>(a, num_cus, stream);
    case 2: return launch_bits<2>(a, num_cus, stream);
    default: return hipErrorInvalidValue;
  }
}
