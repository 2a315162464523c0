// Top-1 gating and dispatch bookkeeping (paper App. B "MoE architecture": top-1
// learned gating as in Switch).  Two kernels in general:
//   route_score_kernel    logits = x W_g (fp32), wavefront-level argmax with
//                         lowest-index tie break, gate = softmax probability
//   route_segments_kernel per-expert histogram, exclusive scan into contiguous
//                         expert segments, stable token permutation
// and one, route_small_kernel, that does both for a decode-sized batch with MFMA scoring;
// without its table step it also serves as the scoring kernel of larger batches.
// Everything is deterministic: no atomics decide an order anywhere.
#include "moqe_dev.h"
#include "moqe_kernels.h"

namespace {

constexpr int SCORE_THREADS = 256;
constexpr int SEG_THREADS = 1024;
constexpr int SEG_LDS_INTS = 9216;

// Block = 256 threads, TB tokens.  Thread (e_l, kp): partial logit of expert
// e_l over the kp-th slice of d for each of the TB tokens.
template <int TB>
__global__ __launch_bounds__(SCORE_THREADS) void route_score_kernel(const half_t* __restrict__ x,
                                                                     const half_t* __restrict__ wg, int T, int d,
                                                                     int E, int EP, int* __restrict__ expert_idx,
                                                                     float* __restrict__ gate) {
  extern __shared__ __align__(16) unsigned char smem[];
  // layout: xs [TB][d] half | red [256][TB] float | logit [TB][E] float
  half_t* xs = (half_t*)smem;
  float* red = (float*)(smem + (((size_t)TB * d * 2 + 15) & ~(size_t)15));
  float* logit = red + SCORE_THREADS * TB;

  const int tid = threadIdx.x;
  const int t0 = blockIdx.x * TB;
  const int nt = min(TB, T - t0);

  // stage the token rows (16 B per thread step; d is a multiple of 8)
  const int vec_per_row = d / 8;
  for (int v = tid; v < TB * vec_per_row; v += SCORE_THREADS) {
    int tb = v / vec_per_row, c = v % vec_per_row;
    uint4_t val = {0, 0, 0, 0};
    if (tb < nt) val = *(const uint4_t*)(x + (int64_t)(t0 + tb) * d + c * 8);
    *(uint4_t*)(xs + tb * d + c * 8) = val;
  }
  __syncthreads();

  const int KP = SCORE_THREADS / EP;  // k slices
  const int e_l = tid % EP;
  const int kp = tid / EP;
  const int kchunk = (d + KP - 1) / KP;
  const int k_begin = min(d, kp * kchunk);
  const int k_end = min(d, k_begin + kchunk);

  for (int eg = 0; eg < E; eg += EP) {
    const int e = eg + e_l;
    float acc[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) acc[tb] = 0.0f;
    if (e < E) {
#pragma unroll 4
      for (int k = k_begin; k < k_end; ++k) {
        float wv = (float)wg[(int64_t)k * E + e];
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) acc[tb] = fmaf((float)xs[tb * d + k], wv, acc[tb]);
      }
    }
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) red[tid * TB + tb] = acc[tb];
    __syncthreads();
    // thread (e_l, tb') sums the KP slices in a fixed order
    for (int o = tid; o < EP * TB; o += SCORE_THREADS) {
      int el = o % EP, tb = o / EP;
      if (eg + el < E) {
        float s = 0.0f;
        for (int p = 0; p < KP; ++p) s += red[(p * EP + el) * TB + tb];
        logit[tb * E + eg + el] = s;
      }
    }
    __syncthreads();
  }

  const int wave = tid / 64;
  for (int tb = wave; tb < nt; tb += SCORE_THREADS / 64) {
    int idx;
    float g;
    wave_pick(logit + tb * E, E, &idx, &g);
    if (lane_id() == 0) {
      expert_idx[t0 + tb] = idx;
      gate[t0 + tb] = g;
    }
  }
}

// One token per block, for E a multiple of 8: thread (kq, eg) reads rows k = kq + KQ i of
// W_g, eight experts (16 bytes) at a time, with all loads of a batch in flight together.
__global__ __launch_bounds__(SCORE_THREADS) void route_score8_kernel(const half_t* __restrict__ x,
                                                                      const half_t* __restrict__ wg, int T, int d,
                                                                      int E, int EGP, int* __restrict__ expert_idx,
                                                                      float* __restrict__ gate) {
  __shared__ float red[SCORE_THREADS / 64][256];  // [wave][expert], E <= 256
  __shared__ float logit[256];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int t = blockIdx.x;
  const int EG = E >> 3;
  const int KQ = SCORE_THREADS / EGP;
  const int eg = tid % EGP, kq = tid / EGP;
  const half_t* xr = x + (int64_t)t * d;
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
        const float xf = (float)xv[i];
#pragma unroll
        for (int q = 0; q < 8; ++q) acc[q] = fmaf(xf, (float)h[q], acc[q]);
      }
    }
  }
  // EGP <= 32: lanes of a wave that share eg fold their k-slices together, then the
  // four waves meet in LDS and are summed in a fixed order
  for (int off = 32; off >= EGP; off >>= 1) {
#pragma unroll
    for (int q = 0; q < 8; ++q) acc[q] += __shfl_xor(acc[q], off, 64);
  }
  if (lane < EGP && eg < EG) {
#pragma unroll
    for (int q = 0; q < 8; ++q) red[wave][eg * 8 + q] = acc[q];
  }
  __syncthreads();
  for (int e = tid; e < E; e += SCORE_THREADS) {
    float sum = 0.0f;
    for (int w = 0; w < SCORE_THREADS / 64; ++w) sum += red[w][e];
    logit[e] = sum;
  }
  __syncthreads();
  if (wave == 0) {
    int idx;
    float g;
    wave_pick(logit, E, &idx, &g);
    if (lane == 0) {
      expert_idx[t] = idx;
      gate[t] = g;
    }
  }
}

// One wave per token, logits given.
__global__ __launch_bounds__(256) void route_pick_kernel(const float* __restrict__ logits, int T, int E,
                                                          int* __restrict__ expert_idx, float* __restrict__ gate) {
  int t = blockIdx.x * 4 + threadIdx.x / 64;
  if (t >= T) return;
  int idx;
  float g;
  wave_pick(logits + (int64_t)t * E, E, &idx, &g);
  if (lane_id() == 0) {
    expert_idx[t] = idx;
    gate[t] = g;
  }
}

// Lanes holding the same key, as a 64-bit mask (nb = number of key bits).
__device__ inline uint64_t match_any(int key, int nb) {
  uint64_t m = ~0ull;
  for (int b = 0; b < nb; ++b) {
    bool bit = (key >> b) & 1;
    uint64_t bb = __ballot(bit);
    m &= bit ? bb : ~bb;
  }
  return m;
}

// Single block.  cnt[expert][chunk] (chunks of 64 consecutive tokens, rows of an odd length so
// that neither a wave that walks along the chunks of one expert nor one that scatters over the
// experts of one chunk meets bank conflicts) lives in LDS when it fits, else in the caller's
// workspace.
__global__ __launch_bounds__(SEG_THREADS) void route_segments_kernel(const int* __restrict__ expert_idx, int T, int E,
                                                                      int* __restrict__ seg_offsets,
                                                                      int* __restrict__ perm, int* ws_cnt) {
  __shared__ int s_cnt[SEG_LDS_INTS];
  __shared__ int s_off[1024 + 1];
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int nthreads = (int)blockDim.x;
  const int nwaves = nthreads / 64;
  const int nchunks = (T + 63) / 64;
  const int CP = nchunks | 1;  // row length of cnt
  int* cnt = ((int64_t)CP * E <= SEG_LDS_INTS) ? s_cnt : ws_cnt;
  int nb = 0;
  while ((1 << nb) <= E) ++nb;  // keys 0..E (E = "no token")

  // a wave's first KEEP chunks stay in registers from the counting pass to the scatter pass
  constexpr int KEEP = 4;
  int keep_key[KEEP];
  uint64_t keep_m[KEEP];
#pragma unroll
  for (int i = 0; i < KEEP; ++i) {
    const int t = (wave + i * nwaves) * 64 + lane;
    keep_key[i] = t < T ? min(max(expert_idx[t], 0), E - 1) : E;  // asked for before the table is cleared
  }
  for (int i = tid; i < CP * E; i += nthreads) cnt[i] = 0;
  __syncthreads();

#pragma unroll
  for (int i = 0; i < KEEP; ++i) {
    const int c = wave + i * nwaves;
    const int key = keep_key[i];
    const uint64_t m = match_any(key, nb);  // (chunks past the end: all lanes hold E, nothing written)
    keep_m[i] = m;
    const bool leader = (__ffsll((long long)m) - 1) == lane;
    if (key < E && leader) cnt[key * CP + c] = __popcll(m);
  }
  for (int c = wave + KEEP * nwaves; c < nchunks; c += nwaves) {
    int t = c * 64 + lane;
    bool valid = t < T;
    int key = valid ? min(max(expert_idx[t], 0), E - 1) : E;  // (an index outside [0, E) cannot come from the
                                                                // scoring kernels; a caller's own must not write wild)
    uint64_t m = match_any(key, nb);
    bool leader = (__ffsll((long long)m) - 1) == lane;
    if (valid && leader) cnt[key * CP + c] = __popcll(m);
  }
  __syncthreads();

  // per expert: exclusive running sum over chunks, a wave per expert, a lane per chunk
  for (int e = wave; e < E; e += nwaves) {
    int carry = 0;
    for (int c0 = 0; c0 < nchunks; c0 += 64) {
      const int c = c0 + lane;
      const int v = (c < nchunks) ? cnt[e * CP + c] : 0;
      int inc = v;
      for (int off = 1; off < 64; off <<= 1) {
        int o = __shfl_up(inc, off, 64);
        if (lane >= off) inc += o;
      }
      if (c < nchunks) cnt[e * CP + c] = carry + inc - v;
      carry += __shfl(inc, 63, 64);
    }
    if (lane == 0) s_off[e] = carry;
  }
  __syncthreads();

  // exclusive scan over experts (wave 0, groups of 64 with a carry)
  if (wave == 0) {
    int carry = 0;
    for (int eg = 0; eg < E; eg += 64) {
      int e = eg + lane;
      int v = (e < E) ? s_off[e] : 0;
      int inc = v;
      for (int off = 1; off < 64; off <<= 1) {
        int o = __shfl_up(inc, off, 64);
        if (lane >= off) inc += o;
      }
      if (e < E) {
        int ex = carry + inc - v;
        s_off[e] = ex;
        seg_offsets[e] = ex;
      }
      carry += __shfl(inc, 63, 64);
    }
    if (lane == 0) seg_offsets[E] = T;
  }
  __syncthreads();

#pragma unroll
  for (int i = 0; i < KEEP; ++i) {
    const int c = wave + i * nwaves;
    const int key = keep_key[i];
    if (key < E) {
      const int rank = __popcll(keep_m[i] & ((1ull << lane) - 1ull));
      perm[s_off[key] + cnt[key * CP + c] + rank] = c * 64 + lane;
    }
  }
  for (int c = wave + KEEP * nwaves; c < nchunks; c += nwaves) {
    int t = c * 64 + lane;
    bool valid = t < T;
    int key = valid ? min(max(expert_idx[t], 0), E - 1) : E;
    uint64_t m = match_any(key, nb);
    if (valid) {
      int rank = __popcll(m & ((1ull << lane) - 1ull));
      perm[s_off[key] + cnt[key * CP + c] + rank] = t;
    }
  }
}


// ---------------------------------------------------------------------------
// Decode-sized batches (T <= 64): the whole router in ONE workgroup and one launch.
// One workgroup has one CU's instruction issue (a vector instruction of a wave takes four
// cycles of its SIMD), and at this size that, not memory, is what the router's phases cost:
// every phase is laid out for few instructions per wave.
//   scores  the logits are a small MFMA GEMM (token tiles x expert tiles of 16 x 16, 32 rows of
//           d per step), d split over the 16 waves; a wave asks for the operands of two steps
//           at once, so d = 1024 is one round trip to memory;
//   sum     the waves' partial tiles meet in LDS and are summed in a fixed order, four values
//           (one MFMA result register quad) per thread;
//   pick    a token's row of E logits is scanned by 16 neighbouring lanes (E / 16 experts each,
//           then four DPP steps), four tokens per wave, all waves at once;
//   tables  wave 0: equal-key masks by ballots, counts, a DPP scan, the stable permutation.
// NT = E / 16 expert tiles, MT = token tiles kept per wave (4, or 2 for 128 experts).
// ---------------------------------------------------------------------------
constexpr int small_waves(int nt) { return nt >= 8 ? 8 : 16; }

// NT neighbouring fp16 values of a row of W_g as one load.
template <int NT>
struct GateRow {
  typedef _Float16 type __attribute__((ext_vector_type(NT)));
  static __device__ inline _Float16 at(const type& v, int i) { return v[i]; }
};
template <>
struct GateRow<1> {
  typedef _Float16 type;
  static __device__ inline _Float16 at(const type& v, int) { return v; }
};

// TABLES = false: the same scoring for any number of tokens (T_total), one workgroup per
// 16 tokens, top-1 and gate only; route_segments_kernel follows.
template <int NT, bool TABLES>
__global__ __launch_bounds__(64 * small_waves(NT)) void route_small_kernel(const half_t* __restrict__ x,
                                                                           const half_t* __restrict__ wg, int T_total,
                                                                           int d, int* __restrict__ expert_idx,
                                                                           float* __restrict__ gate,
                                                                           int* __restrict__ seg_offsets,
                                                                           int* __restrict__ perm) {
  constexpr int MT = !TABLES ? 1 : NT >= 8 ? 2 : 4;
  constexpr int E = 16 * NT;
  constexpr int WAVES = small_waves(NT), THREADS = 64 * WAVES;
  // this workgroup's tokens
  const int t_base = TABLES ? 0 : (int)blockIdx.x * 16 * MT;
  const int T = TABLES ? T_total : min(16 * MT, T_total - t_base);
  x += (int64_t)t_base * d;
  expert_idx += t_base;
  gate += t_base;
  // 16 x 16 result tiles the partial-sum buffer holds per wave, token tiles summed per pass
  constexpr int PART_TILES = MT * NT > 8 ? 8 : MT * NT;
  constexpr int MT_PASS = PART_TILES / NT;
  constexpr int LROW = E + 16;  // row of logits; the pad sends neighbouring tokens to different banks
  __shared__ float4_t s_part[WAVES][PART_TILES][64];
  __shared__ __align__(16) float s_logit[MT * 16 * LROW];
  __shared__ int s_idx[64];
  __shared__ int s_seg[E + 1];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 4, j = lane & 15;
  const int mt = (T + 15) >> 4;
  const int steps = d / 32;  // 32-row steps of d, dealt round-robin to the waves

  float4_t acc[MT][NT];
#pragma unroll
  for (int mi = 0; mi < MT; ++mi)
#pragma unroll
    for (int ni = 0; ni < NT; ++ni) acc[mi][ni] = float4_t{0, 0, 0, 0};

  // Lane (g, j) holds, as the A operand, token row j of each token tile (rows past the last
  // token repeat it: their logits are never looked at) over rows 8 g .. 8 g + 7 of a step, and,
  // as the B operand of expert tile ni, column j of that tile.  Which experts make up a tile is
  // free: tile ni takes the experts NT j + ni, so that the NT values a lane needs from one row
  // of W_g are neighbours and come with one load (eight loads per step whatever E is; one CU's
  // memory pipeline takes a wave's load every 16 cycles or so whatever its width, and with two
  // bytes per lane that, not latency, would set the time of this phase).
  using Row = GateRow<NT>;
  const half_t* xrow[MT];
#pragma unroll
  for (int mi = 0; mi < MT; ++mi) xrow[mi] = x + (int64_t)min(16 * mi + j, T - 1) * d + 8 * g;
  const half_t* const wcol = wg + (int64_t)(8 * g) * E + NT * j;
  // Up to 32 experts: two steps per trip, all their operands asked for before the first is
  // used (a wave without a second step repeats the first and leaves its product out).  More
  // expert tiles fill the registers with one step's operands.
  constexpr int PER_TRIP = NT <= 2 ? 2 : 1;
  for (int s = wave; s < steps; s += PER_TRIP * WAVES) {
    const bool two = PER_TRIP == 2 && s + WAVES < steps;  // (uniform)
    const int sb = two ? s + WAVES : s;
    half8_t a0[MT], a1[PER_TRIP == 2 ? MT : 1];
    typename Row::type w0[8], w1[PER_TRIP == 2 ? 8 : 1];
#pragma unroll
    for (int mi = 0; mi < MT; ++mi) {
      a0[mi] = *(const half8_t*)(xrow[mi] + s * 32);
      if constexpr (PER_TRIP == 2) a1[mi] = *(const half8_t*)(xrow[mi] + sb * 32);
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      w0[q] = *(const typename Row::type*)(wcol + (int64_t)s * 32 * E + q * E);
      if constexpr (PER_TRIP == 2) w1[q] = *(const typename Row::type*)(wcol + (int64_t)sb * 32 * E + q * E);
    }
#pragma unroll
    for (int ni = 0; ni < NT; ++ni) {
      half8_t b;
#pragma unroll
      for (int q = 0; q < 8; ++q) b[q] = Row::at(w0[q], ni);
#pragma unroll
      for (int mi = 0; mi < MT; ++mi)
        if (mi < mt) acc[mi][ni] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0[mi], b, acc[mi][ni], 0, 0, 0);
    }
    if constexpr (PER_TRIP == 2) {
      if (two) {
#pragma unroll
        for (int ni = 0; ni < NT; ++ni) {
          half8_t b;
#pragma unroll
          for (int q = 0; q < 8; ++q) b[q] = Row::at(w1[q], ni);
#pragma unroll
          for (int mi = 0; mi < MT; ++mi)
            if (mi < mt) acc[mi][ni] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1[mi], b, acc[mi][ni], 0, 0, 0);
        }
      }
    }
  }
  // D layout of a tile: lane (g, j), register r holds token row 4 g + r, expert NT j + ni.
  // The waves' partial tiles meet in LDS and are summed in a fixed order (wave 0, 1, ...), as
  // many token tiles per pass as the buffer holds.
  for (int m0 = 0; m0 < mt; m0 += MT_PASS) {  // (uniform)
    if (m0 > 0) __syncthreads();
#pragma unroll
    for (int mi = 0; mi < MT; ++mi) {
      if (mi < m0 || mi >= m0 + MT_PASS || mi >= mt) continue;
#pragma unroll
      for (int ni = 0; ni < NT; ++ni) s_part[wave][(mi - m0) * NT + ni][lane] = acc[mi][ni];
    }
    __syncthreads();
    const int n_out = min(MT_PASS, mt - m0) * NT * 64;
    for (int o = tid; o < n_out; o += THREADS) {
      const int slot = o >> 6, l = o & 63;
      float4_t sum = s_part[0][slot][l];
#pragma unroll
      for (int w = 1; w < WAVES; ++w) sum = sum + s_part[w][slot][l];
      const int mo = m0 + slot / NT, ni = slot % NT;
      float* const out = &s_logit[(16 * mo + 4 * (l >> 4)) * LROW + NT * (l & 15) + ni];
#pragma unroll
      for (int r = 0; r < 4; ++r) out[r * LROW] = sum[r];
    }
  }
  __syncthreads();

  // top-1 and gate: a row of 16 lanes per token, four tokens per wave
  for (int t0 = 4 * wave; t0 < T; t0 += 4 * WAVES) {  // (uniform)
    const int t = t0 + g;
    const float* const row = &s_logit[min(t, T - 1) * LROW];
    int idx;
    float gt;
    row16_pick<NT>([row](int e) { return row[e]; }, j, E, &idx, &gt);
    if (j == 0 && t < T) {
      expert_idx[t] = idx;
      gate[t] = gt;
      s_idx[t] = idx;
    }
  }
  if constexpr (!TABLES) return;
  __syncthreads();
  if (wave == 0) {
    const bool valid = lane < T;
    const int key = valid ? min(max(s_idx[lane], 0), E - 1) : E;
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
      const int inc = wave_inclusive_scan(v);
      __builtin_amdgcn_wave_barrier();
      if (e < E) {
        s_seg[e] = carry + inc - v;
        seg_offsets[e] = carry + inc - v;
      }
      carry += __builtin_amdgcn_readlane(inc, 63);
    }
    if (lane == 0) seg_offsets[E] = T;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    if (valid) perm[s_seg[key] + rank] = lane;
  }
}

// One expert (a dense FFN run through the same calls): every token goes to expert 0 with the
// softmax probability of a single logit, 1.
__global__ __launch_bounds__(256) void route_single_expert_kernel(int T, int* __restrict__ expert_idx,
                                                                   float* __restrict__ gate,
                                                                   int* __restrict__ seg_offsets,
                                                                   int* __restrict__ perm) {
  const int t = (int)(blockIdx.x * blockDim.x + threadIdx.x);
  if (t < T) {
    expert_idx[t] = 0;
    gate[t] = 1.0f;
    perm[t] = t;
  }
  if (t == 0) {
    seg_offsets[0] = 0;
    seg_offsets[1] = T;
  }
}

// True when route_small_kernel can take the call.
static bool small_route_fits(int T, int d, int E) {
  if (T < 1 || T > 64 || d < 32 || (d % 32) != 0) return false;
  const int mt = (T + 15) / 16;
  switch (E) {
    case 16: return mt <= 4;
    case 32: return mt <= 4;
    case 64: return mt <= 4;
    case 128: return mt <= 2;
    default: return false;
  }
}

}  // namespace

size_t moqe_route_ws_bytes(int64_t T, int64_t E) {
  int64_t nchunks = (T + 63) / 64;
  int64_t ints = (nchunks | 1) * E;
  size_t b = ints > SEG_LDS_INTS ? (size_t)ints * 4 : 0;
  return b < 256 ? 256 : ((b + 255) & ~(size_t)255);
}

static int pow2_ceil(int v) {
  int p = 1;
  while (p < v) p <<= 1;
  return p;
}

hipError_t moqe_launch_route(const uint16_t* x, const uint16_t* wg, const float* logits, int T, int d, int E,
                             int* expert_idx, float* gate, int* seg_offsets, int* perm, void* ws,
                             hipStream_t stream) {
  if (E == 1) {
    // (also with given logits: the argmax over one column is 0 and its softmax 1 whatever it holds)
    hipLaunchKernelGGL(route_single_expert_kernel, dim3((unsigned)((T + 255) / 256 > 0 ? (T + 255) / 256 : 1)),
                       dim3(256), 0, stream, T, expert_idx, gate, seg_offsets, perm);
    return hipGetLastError();
  }
  if (T > 0 && !logits && small_route_fits(T, d, E)) {
    const half_t* xh = (const half_t*)x;
    const half_t* wh = (const half_t*)wg;
    switch (E) {
      case 16: hipLaunchKernelGGL((route_small_kernel<1, true>), dim3(1), dim3(64 * small_waves(1)), 0, stream, xh, wh, T, d, expert_idx, gate, seg_offsets, perm); break;
      case 32: hipLaunchKernelGGL((route_small_kernel<2, true>), dim3(1), dim3(64 * small_waves(2)), 0, stream, xh, wh, T, d, expert_idx, gate, seg_offsets, perm); break;
      case 64: hipLaunchKernelGGL((route_small_kernel<4, true>), dim3(1), dim3(64 * small_waves(4)), 0, stream, xh, wh, T, d, expert_idx, gate, seg_offsets, perm); break;
      default: hipLaunchKernelGGL((route_small_kernel<8, true>), dim3(1), dim3(64 * small_waves(8)), 0, stream, xh, wh, T, d, expert_idx, gate, seg_offsets, perm); break;
    }
    return hipGetLastError();
  }
  if (T > 0 && !logits && d >= 32 && (d % 32) == 0 && (E == 16 || E == 32 || E == 64 || E == 128)) {
    // more tokens than one workgroup takes: MFMA scoring, one workgroup per 16 tokens
    const half_t* xh = (const half_t*)x;
    const half_t* wh = (const half_t*)wg;
    const int per_wg = 16;
    const dim3 grid((unsigned)((T + per_wg - 1) / per_wg));
    switch (E) {
      case 16: hipLaunchKernelGGL((route_small_kernel<1, false>), grid, dim3(64 * small_waves(1)), 0, stream, xh, wh, T, d, expert_idx, gate, seg_offsets, perm); break;
      case 32: hipLaunchKernelGGL((route_small_kernel<2, false>), grid, dim3(64 * small_waves(2)), 0, stream, xh, wh, T, d, expert_idx, gate, seg_offsets, perm); break;
      case 64: hipLaunchKernelGGL((route_small_kernel<4, false>), grid, dim3(64 * small_waves(4)), 0, stream, xh, wh, T, d, expert_idx, gate, seg_offsets, perm); break;
      default: hipLaunchKernelGGL((route_small_kernel<8, false>), grid, dim3(64 * small_waves(8)), 0, stream, xh, wh, T, d, expert_idx, gate, seg_offsets, perm); break;
    }
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    const int seg_threads = T <= 256 ? 256 : SEG_THREADS;
    hipLaunchKernelGGL(route_segments_kernel, dim3(1), dim3(seg_threads), 0, stream, expert_idx, T, E, seg_offsets, perm,
                       (int*)ws);
    return hipGetLastError();
  }
  if (T > 0) {
    if (logits) {
      hipLaunchKernelGGL(route_pick_kernel, dim3((T + 3) / 4), dim3(256), 0, stream, logits, T, E, expert_idx, gate);
    } else {
      int EP = pow2_ceil(E);
      if (EP > SCORE_THREADS) EP = SCORE_THREADS;
      // 8 tokens per block once there are enough tokens to fill the chip, else 1
      if (T >= 2048) {
        constexpr int TB = 8;
        size_t sm = (((size_t)TB * d * 2 + 15) & ~(size_t)15) + (size_t)SCORE_THREADS * TB * 4 + (size_t)TB * E * 4;
        hipLaunchKernelGGL(route_score_kernel<TB>, dim3((T + TB - 1) / TB), dim3(SCORE_THREADS), sm, stream,
                           (const half_t*)x, (const half_t*)wg, T, d, E, EP, expert_idx, gate);
      } else if ((E % 8) == 0 && E <= 256) {
        int EGP = pow2_ceil(E / 8);
        hipLaunchKernelGGL(route_score8_kernel, dim3(T), dim3(SCORE_THREADS), 0, stream, (const half_t*)x,
                           (const half_t*)wg, T, d, E, EGP, expert_idx, gate);
      } else {
        constexpr int TB = 1;
        size_t sm = (((size_t)TB * d * 2 + 15) & ~(size_t)15) + (size_t)SCORE_THREADS * TB * 4 + (size_t)TB * E * 4;
        hipLaunchKernelGGL(route_score_kernel<TB>, dim3((T + TB - 1) / TB), dim3(SCORE_THREADS), sm, stream,
                           (const half_t*)x, (const half_t*)wg, T, d, E, EP, expert_idx, gate);
      }
    }
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
  }
  // one wave per 64-token chunk, up to the full block
  const int seg_threads = T <= 64 ? 64 : T <= 256 ? 256 : SEG_THREADS;
  hipLaunchKernelGGL(route_segments_kernel, dim3(1), dim3(seg_threads), 0, stream, expert_idx, T, E, seg_offsets, perm,
                     (int*)ws);
  return hipGetLastError();
}
