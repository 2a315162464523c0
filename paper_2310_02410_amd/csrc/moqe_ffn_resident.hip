// Expert FFN contraction for segments with many tokens when a tile's token rows fit in LDS
// whole: 64 tokens where K <= 1024 (FFN1 of the paper's layers), 16 tokens where K <= 4096
// (their FFN2) - Sec. 2.1 two-layer FFN, App. A A' = Q s.
//
//   out[rows of expert e, n] = epilogue( sum_k a[row, k] * (Q_e[k, n] * s_e[n]) + b_e[n] )
//
// Work decomposition
//   pair = (expert e, tile of TM = 64 or 16 of its tokens), found on device from seg_offsets
//   unit = (pair, group of NT column tiles of 16 channels).  A unit costs 8 + 10 (token tiles
//          of the pair) - the unpack does not shrink with a ragged pair, the matrix-core work and
//          the epilogue do -, taking up a pair costs about eight units of a full pair of 64 at
//          K = 1024, and the units of the whole launch, in pair-major order, are cut into one
//          contiguous range of equal cost per workgroup (one workgroup of WAVES waves per compute
//          unit): every workgroup gets the same work whatever the number of pairs is, and a range
//          touches as few pairs as possible
//   per pair of its range a workgroup
//     - stages the pair's TM x K token rows in LDS ONCE (128 KiB at most; loads that go from
//       global memory straight into LDS, a row's 16-byte pieces XOR-swizzled by the row number so
//       that the fragment reads are conflict-free without padding), one barrier; the row numbers
//       (FFN1: through perm) were asked for while the pair before was being worked on;
//     - takes the constants' share out of the K-sums (see "unpack" below), one more barrier;
//     - then every wave works through units with no further barrier - its first one by its
//       number, the following ones handed out through a counter in LDS, because the two waves
//       of a SIMD do not advance at the same rate: the packed chunks of the unit's column
//       tiles stream from global memory into a rolling window of registers (the packed layout
//       already is the matrix-core operand order), are dequantized in registers and multiplied
//       with the fragments read from LDS a step ahead (v_mfma_f32_16x16x32_f16, weights as
//       first operand, tokens as second, fp32 accumulate); the window runs on across the end of
//       a unit, so a unit's first chunks arrive during the previous unit's epilogue.
//   Token tiles a ragged pair does not have are neither staged nor multiplied (the loop is
//   instantiated for 1 to 4 token tiles).  With one token tile a step is two MFMAs and too short
//   to hide an LDS read: the fragments are then read a whole chunk ahead.
//   Pairs of 16 tokens read an expert's weights once per 16 of its tokens instead of once per 64:
//   they serve batches with few tokens per expert (most experts fill one such pair at most),
//   where staging K in blocks costs a barrier every 128 rows of K for a tile that is mostly
//   padding; launches with so few pairs that units of two column tiles would leave waves idle use
//   units of one.
//   Unpack: linear codes become (code + a constant per position in the step) with the unpack
//   of the decode kernels (moqe_unpack.h), a packed subtract per register less than the exact
//   one; sum_k a[token, k] c[k] does not depend on the channel, is computed once per pair on
//   the matrix cores and is what the accumulators start from (negated).  The constants (at most
//   132 per weight) cost no accuracy that shows against the fp16 rounding of the outputs, also
//   over K = 4096 of all-positive rows (tested).  With four token tiles the loop issues 2.5 vector
//   instructions per MFMA; a vector instruction takes the SIMD's issue port for 4 cycles, an MFMA
//   for 8 of its 16, so at 8 MFMAs and 12 to 20 vector instructions a step the matrix cores, not
//   the issue port, bound the loop.
// Compared with staging K in blocks through LDS (moqe_ffn_prefill.hip, which serves longer K and
// K > 1024 at many tokens per expert) the token rows are fetched once per pair and workgroup
// instead of once per block of output channels, and the main loop has no barrier and no wait
// that the compiler cannot see.
#include "moqe_dev.h"
#include "moqe_kernels.h"
#include "moqe_unpack.h"

#include <type_traits>

namespace {

constexpr int RS_LDS_ELEMS = 64 * 1024;  // token-row elements resident per workgroup: 128 KiB of LDS
constexpr int RS_MAX_K = 4096;           // (pairs of 16 tokens; pairs of 64 up to K = 1024)
constexpr int RS_MAX_E = 1024;
// Cost model of the work split, fitted to time stamps of the 4096-token and the 1536-token
// layers (int2 and int4, uniform and Zipf load): eight units (of two column tiles, 32 K steps per
// 1024 of K) of a pair with m token tiles take 1.9 / 2.6-3.0 / 3.8-4.2 / 5.2-5.3 us for m = 1 .. 4
// on a workgroup's eight waves - the unpack does not shrink with a ragged pair, the matrix-core
// work and the epilogue do - and taking up a pair (staging its rows, the offset sums) about as
// long as eight units of a full pair.  RS_SWITCH: a pair's start, in the scale of
// rs_cost_of_8_units.
constexpr int RS_SWITCH = 44;
__host__ __device__ constexpr int rs_cost_of_8_units(int token_tiles) { return 8 + 10 * token_tiles; }

struct RsPair {
  int e, row0, rows;
};
struct RsJob {
  RsPair t;
  int g0, g1;  // the pair's units for this workgroup; g0 >= g1: no further pair
};
// (members, not an array: they stay in registers across a pair)
struct RsRows {
  uint32_t r0, r1, r2, r3;
};

// NT: column tiles per unit; WAVES: waves per workgroup (8: two per SIMD, up to 256 registers
// each); W: packed chunks in flight per wave and column tile (the chunk count of a column tile
// must be a multiple of W); MODE 0: FFN1 (rows of `a` by token through perm, ReLU, output by sorted
// position), MODE 1: FFN2 (rows by sorted position, gate and residual, output by token); TM: tokens
// per pair, 64 (K <= 1024) or 16 (K <= 4096)
template <int BITS, int NT, int WAVES, int W, int MODE, int TM>
__global__ __launch_bounds__(64 * WAVES) void moe_resident_kernel(PrefillArgs A) {
  static_assert(TM == 64 || TM == 16, "pairs of 64 or 16 tokens");
  constexpr int SEG = TM * 32;               // 16-byte pieces of the pair's rows per 256 of K
  constexpr int FB = moqe_field_bits(BITS);  // stored bits per weight
  static_assert(FB == 2 || FB == 3 || FB == 4, "2- to 4-bit codes");
  constexpr int SC = FB == 4 ? 4 : 8;        // steps of 32 rows per packed chunk
  constexpr int LO_BITS = FB == 3 ? 2 : FB;
  constexpr int LW = SC * LO_BITS / 4;       // main-plane words per lane per chunk (4)
  constexpr int HW = FB == 3 ? SC / 4 : 0;   // 1-bit-plane words per lane per chunk
  constexpr int CHUNK_BYTES = 64 * SC * FB;
  // an offset beyond every descriptor (a matrix has at most 2^29 bytes): the load returns zero
  constexpr uint32_t NOWHERE = 0x80000000u;

  // K is cut into segments of 256 (32 pieces of 16 bytes per row); piece p of row r of segment
  // sg lives at s_a[(sg * TM + r) * 32 + (p ^ (r & 15))]
  __shared__ uint4_t s_a[RS_LDS_ELEMS / 8];
  __shared__ int s_cost[RS_MAX_E];     // inclusive prefix of the experts' costs
  __shared__ int s_seg[RS_MAX_E + 1];  // seg_offsets
  // The constants' share of the K-sums is taken out per slab of 512 along K where K can exceed
  // 1024 (one slab for the whole K otherwise), so that the running sums never carry more than one
  // slab's share.
  constexpr int NSLAB = TM == 64 ? 1 : 8;
  constexpr int SLAB_STEPS = TM == 64 ? 32 : 16;  // steps of 32 rows per slab
  constexpr int CPS = SLAB_STEPS / SC;            // packed chunks per slab
  __shared__ float s_corr[WAVES][NSLAB][TM];
  __shared__ int s_next;               // the next unit of the pair nobody has taken yet

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = uniform_i32(tid >> 6);
  const int g = lane >> 4, j = lane & 15;
  const int E = A.E, K = A.K, N = A.N;
  const int G = (int)gridDim.x, bid = (int)blockIdx.x;

  const int CT = N >> 4;
  const int NG = (CT + NT - 1) / NT;        // units per pair
  // cost of a unit of a pair with m token tiles, and of taking up a pair
  const int Q = K / (32 * SC);              // packed chunks per column tile
  const int NSG = K >> 8;                   // segments of 256 along K
  // (a unit's cost grows with K, taking up a pair - 128 KiB of rows at most - does not; at
  // K = 1024 the two are in the ratio the time stamps gave)
  auto unit_cost = [NSG](int m) { return rs_cost_of_8_units(m) * NT / 2 * NSG; };
  constexpr int SWITCH = RS_SWITCH * WAVES * 4;

  // ---- cost of every expert's pairs, inclusive prefix ----
  if (wave == 0) {
    int carry = 0;
    for (int eg = 0; eg < E; eg += 64) {
      const int e = eg + lane;
      int v = 0;
      if (e < E) {
        const int s0 = A.seg_offsets[e];
        const int n = A.seg_offsets[e + 1] - s0;
        s_seg[e] = s0;
        if (e == E - 1) s_seg[E] = s0 + n;
        if (n >= A.min_tokens)
          v = (n / TM) * (SWITCH + NG * unit_cost(TM / 16)) + ((n % TM) ? SWITCH + NG * unit_cost(((n % TM) + 15) >> 4) : 0);
      }
      v = wave_inclusive_scan(v);
      if (e < E) s_cost[e] = carry + v;
      carry += __builtin_amdgcn_readlane(v, 63);
    }
  }
  __syncthreads();

  // Workgroups are dealt to the 8 XCDs round-robin by their index: XCD x takes the x-th eighth
  // of the ranges, so neighbouring ranges (one pair's, one expert's) share an L2.
  const int64_t C = s_cost[E - 1];
  const int widx = (bid & 7) * (G >> 3) + (bid >> 3);
  const int c_lo = (int)(C * widx / G), c_hi = (int)(C * (widx + 1) / G);
  if (c_lo >= c_hi) return;

  const int64_t matrix_bytes = (int64_t)K * N * FB / 8;
  const uint32_t lane_lo = (uint32_t)lane * LW * 4, lane_hi = (64u * LW + (uint32_t)lane * HW) * 4;
  UnpackConsts<BITS> uc;
  uc.init();
  const rsrc_t a_rsrc = make_rsrc(A.a, (uint32_t)((int64_t)A.T * K * 2));
  const uint32_t out_bytes = (uint32_t)((int64_t)A.T * N * 2);
  const rsrc_t out_rsrc = make_rsrc(A.out, out_bytes);
  const rsrc_t res_rsrc = make_rsrc(A.residual, A.residual ? out_bytes : 0u);

  // This lane's piece of a fragment in step s of a segment (s = 0 .. 7): logical piece 4 s + g
  // of a row with (row & 15) == j, stored at (4 s + g) ^ j = (4 s) ^ (g ^ j) = 16 (s >> 2) +
  // ((4 (s & 3)) ^ (g ^ j)): four per-lane values (in units of 16 bytes, row j of a token tile
  // included), everything else is uniform or an immediate.
  const int fb = g ^ j;
  const int ab0 = j * 32 + fb, ab1 = j * 32 + (4 ^ fb), ab2 = j * 32 + (8 ^ fb), ab3 = j * 32 + (12 ^ fb);

  // load n of a staging pass: 64 pieces from the lanes' byte offsets in `a` to s_a[64 n ..]
  // (kept out of the generic lambda below: the builtin is only known to the device pass)
  auto stage_load = [&](int n, uint32_t off) {
    typedef __attribute__((address_space(3))) void* lds_ptr;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, (lds_ptr)&s_a[64 * n], 16, off, 0, 0, 0);
  };

  // Byte offsets in `a` of the pieces this lane stages for pair t: row 2 rr + (lane >> 5) of the
  // pair for the wave's row pairs rr = wave, wave + WAVES, ... (FFN1: through perm, a global read,
  // which is why this is asked for a pair ahead); piece (lane & 31) of each 512-byte segment of
  // the row, swizzled.
  constexpr int RPW = (TM / 2) / WAVES;
  static_assert((TM / 2) % WAVES == 0 && RPW >= 1, "a wave stages whole pairs of rows");
  static_assert(RPW <= 4, "RsRows holds four row pairs");
  auto row_offsets = [&](const RsPair t) -> RsRows {
    uint32_t o[4] = {0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < RPW; ++i) {
      const int r = 2 * (wave + i * WAVES) + (lane >> 5);
      const int sr = t.row0 + min(r, t.rows - 1);
      const uint32_t arow = MODE == 0 ? (uint32_t)A.perm[sr] : (uint32_t)sr;
      o[i] = arow * (uint32_t)K * 2u + (uint32_t)((((lane & 31) ^ (r & 15))) * 16);
    }
    return RsRows{o[0], o[1], o[2], o[3]};
  };

  // ---- this workgroup's units: those whose first unit of cost lies in [c_lo, c_hi) ----
  // next_job walks through the pairs that have such units, in order.
  int it_e = E, it_ti = -1;
  for (int eg = 0; eg < E; eg += 64) {  // the first expert whose cost range ends beyond c_lo
    const bool beyond = eg + lane < E && s_cost[eg + lane] > c_lo;
    const unsigned long long m = __ballot(beyond);
    if (m) {
      it_e = uniform_i32(eg + (int)__builtin_ctzll(m));
      break;
    }
  }
  auto next_job = [&]() -> RsJob {
    for (; it_e < E; ++it_e, it_ti = -1) {
      const int base = it_e > 0 ? s_cost[it_e - 1] : 0;
      if (base >= c_hi) break;
      if (s_cost[it_e] == base) continue;  // no pairs
      const int seg0 = s_seg[it_e], n = s_seg[it_e + 1] - seg0;
      const int full = n / TM, rem = n % TM;
      const int npairs = full + (rem ? 1 : 0);
      const int pair_cost = SWITCH + NG * unit_cost(TM / 16);
      if (it_ti < 0) {
        it_ti = c_lo > base ? (c_lo - base) / pair_cost : 0;
        if (it_ti > full) it_ti = full;
      }
      for (; it_ti < npairs; ++it_ti) {
        const int S = base + it_ti * pair_cost + SWITCH;  // cost at the pair's first unit
        if (S - SWITCH >= c_hi) break;
        const int rows = it_ti < full ? TM : rem;
        const int w = unit_cost((rows + 15) >> 4);
        const int u0 = c_lo > S ? (c_lo - S + w - 1) / w : 0;
        int u1 = c_hi > S ? (c_hi - S + w - 1) / w : 0;
        if (u1 > NG) u1 = NG;
        if (u0 >= u1) continue;
        RsJob jb;
        jb.t = RsPair{uniform_i32(it_e), uniform_i32(seg0 + TM * it_ti), uniform_i32(rows)};
        jb.g0 = uniform_i32(u0);
        jb.g1 = uniform_i32(u1);
        ++it_ti;
        return jb;
      }
    }
    return RsJob{RsPair{0, 0, 1}, 0, 0};
  };

  // The units [g0, g1) of pair t for this workgroup
  auto run_pair = [&](const RsPair t, const int g0, const int g1, const RsRows rows_off, RsJob* job_next,
                      RsRows* rows_next, auto MTC) {
    constexpr int MT = decltype(MTC)::value;  // token tiles of 16 the pair has
    const rsrc_t b_rsrc = make_rsrc((const char*)A.codes + (int64_t)t.e * matrix_bytes, (uint32_t)matrix_bytes);
    uint32_t b_lo[W][NT][LW];
    uint32_t b_hi[W][NT][HW > 0 ? HW : 1];
    float4_t acc[MT][NT];

    // byte offset of the first chunk of column tile ni of unit grp (NOWHERE if there is none)
    auto unit_base = [&](int grp, uint32_t (&base)[NT]) {
#pragma unroll
      for (int ni = 0; ni < NT; ++ni) {
        const int ct = grp * NT + ni;
        const bool ok = (grp < g1) & (ct < CT);
        base[ni] = uniform_u32(ok ? (uint32_t)ct * (uint32_t)Q * CHUNK_BYTES : NOWHERE);
      }
    };
    // chunk c of a unit's column tiles into window slot SLOT
    auto load_chunk = [&](auto SLOT, const uint32_t (&base)[NT], int c) {
      constexpr int slot = decltype(SLOT)::value;
#pragma unroll
      for (int ni = 0; ni < NT; ++ni) {
        const uint32_t off = base[ni] + (uint32_t)c * CHUNK_BYTES;
        load_words<LW, 0>(b_rsrc, off + lane_lo, b_lo[slot][ni]);
        if constexpr (FB == 3) load_words<HW, 0>(b_rsrc, off + lane_hi, b_hi[slot][ni]);
      }
    };

    // ---- stage the pair's token rows ----
    // Load n = (TM / 2) sg + rr brings the rows 2 rr and 2 rr + 1 of segment sg (32 pieces each) to
    // s_a[64 n ..]; wave w issues the loads of the row pairs rr = w, w + WAVES, ... < TM / 2 of
    // every segment: the caller has their offsets in `a` ready
    // (row_offsets).  Row pairs of token tiles the pair does not have are left out; the rows a
    // ragged tile lacks repeat its last row (never stored).
    {
      const uint32_t rowoff[4] = {rows_off.r0, rows_off.r1, rows_off.r2, rows_off.r3};
      for (int sg = 0; sg < NSG; ++sg) {
#pragma unroll
        for (int i = 0; i < RPW; ++i) {
          const int rr = wave + i * WAVES;
          if (rr < 8 * MT) stage_load((TM / 2) * sg + rr, rowoff[i] + (uint32_t)sg * 512u);
        }
      }
    }
    // the workgroup's next pair and the rows it will stage, found and asked for now: the search
    // and the trip through perm are over long before that pair is taken up
    *job_next = next_job();
    *rows_next = row_offsets(job_next->t);
    // FFN2 writes by token, times the token's gate.  Byte offset of this lane's output rows
    // (T N < 2^31: checked by the caller); rows a ragged tile lacks get an offset beyond the
    // descriptor, so that their stores (and residual loads) touch no memory.
    float gt[MT];
    uint32_t out_off[MT];
#pragma unroll
    for (int mi = 0; mi < MT; ++mi) {
      const int row = 16 * mi + j;
      const bool have = row < t.rows;
      int orow = t.row0 + row;
      gt[mi] = 1.0f;
      if constexpr (MODE != 0) {
        orow = have ? A.perm[t.row0 + row] : 0;
        gt[mi] = A.gate[orow];
      }
      out_off[mi] = have ? (uint32_t)orow * (uint32_t)N * 2u : NOWHERE;
    }

    // Every wave starts with unit g0 + wave; further units are handed out as waves ask for
    // them (the two waves of a SIMD do not advance at the same rate: the older one is served
    // first, and with fixed shares the younger one would finish a third later).
    int grp = g0 + wave;
    if (tid == 0) s_next = g0 + WAVES;  // (read after the barrier below)
    uint32_t cur[NT], nxt[NT];
    unit_base(grp, cur);
    {
      // the first W chunks of this wave's first unit
      auto first = [&](auto SLOT) { load_chunk(SLOT, cur, decltype(SLOT)::value); };
      first(std::integral_constant<int, 0>{});
      if constexpr (W > 1) first(std::integral_constant<int, 1>{});
      if constexpr (W > 2) first(std::integral_constant<int, 2>{});
      if constexpr (W > 3) first(std::integral_constant<int, 3>{});
      if constexpr (W > 4) first(std::integral_constant<int, 4>{});
      if constexpr (W > 5) first(std::integral_constant<int, 5>{});
      if constexpr (W > 6) first(std::integral_constant<int, 6>{});
      if constexpr (W > 7) first(std::integral_constant<int, 7>{});
    }
    // loads into LDS are invisible to the compiler's wait insertion
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    __syncthreads();

    // Linear codes are unpacked to (code + a constant per position in the step) - a packed
    // subtract per register less than the exact unpack - and the constants' share of the K-sum,
    // sum_k a[token, k] c[k], is taken out once per pair (the accumulators start at minus that
    // sum): it does not depend on the channel.
    // Every wave multiplies the steps wave, wave + WAVES, ... of the pair's rows with the
    // constants, the partial sums meet in LDS and are added in a fixed order.
    // Over a long K of all-positive rows that sum is thousands of times the signal and its fp32
    // rounding would show: it is taken out slab by slab (512 of K each), the accumulators start
    // at minus the first slab's sum and the next slab's is subtracted when its first chunk is due.
    float corr[MT][NSLAB];
#pragma unroll
    for (int mi = 0; mi < MT; ++mi)
#pragma unroll
      for (int sl = 0; sl < NSLAB; ++sl) corr[mi][sl] = 0.0f;
    if constexpr (!moqe_is_log(BITS)) {
      float4_t cacc[MT][NSLAB];
      const half8_t c_even = bias_frag<BITS>(0), c_odd = bias_frag<BITS>(1);
#pragma unroll
      for (int sl = 0; sl < NSLAB; ++sl) {
#pragma unroll
        for (int mi = 0; mi < MT; ++mi) cacc[mi][sl] = float4_t{0, 0, 0, 0};
        const int st_end = min(SLAB_STEPS * (sl + 1), 8 * NSG);
        for (int st = SLAB_STEPS * sl + wave; st < st_end; st += WAVES) {
          const int within = st & 7;
          const int ab = (within & 3) == 0 ? ab0 : (within & 3) == 1 ? ab1 : (within & 3) == 2 ? ab2 : ab3;
          const uint4_t* ps = s_a + (st >> 3) * SEG + (within >> 2) * 16 + ab;
          const half8_t cf = (st & 1) ? c_odd : c_even;
#pragma unroll
          for (int mi = 0; mi < MT; ++mi)
            cacc[mi][sl] = __builtin_amdgcn_mfma_f32_16x16x32_f16(cf, __builtin_bit_cast(half8_t, ps[mi * (16 * 32)]), cacc[mi][sl], 0, 0, 0);
        }
      }
      if (g == 0) {
#pragma unroll
        for (int mi = 0; mi < MT; ++mi)
#pragma unroll
          for (int sl = 0; sl < NSLAB; ++sl) s_corr[wave][sl][16 * mi + j] = cacc[mi][sl][0];
      }
      __syncthreads();
#pragma unroll
      for (int mi = 0; mi < MT; ++mi) {
#pragma unroll
        for (int sl = 0; sl < NSLAB; ++sl) {
#pragma unroll
          for (int w = 0; w < WAVES; ++w) corr[mi][sl] += s_corr[w][sl][16 * mi + j];
        }
      }
    }

    // a chunk's first piece: segment c (8 steps per chunk) or half of segment c / 2 (4 steps)
    auto chunk_ofs = [&](int c) { return SC == 8 ? c * SEG : (c >> 1) * SEG + (c & 1) * 16; };
    // With a single token tile a step is too short to hide the LDS read of the next step's
    // fragment: the fragments are then read a whole chunk ahead, step s of chunk c + 1 as soon as
    // step s of chunk c has been issued (the rows do not depend on the unit: after a unit's last
    // chunk comes the next unit's first).
    half8_t afr[MT == 1 ? SC : 1];
    if constexpr (MT == 1) {
      const uint4_t* q = s_a + chunk_ofs(0);
#pragma unroll
      for (int st = 0; st < SC; ++st) {
        const int ab = (st & 3) == 0 ? ab0 : (st & 3) == 1 ? ab1 : (st & 3) == 2 ? ab2 : ab3;
        afr[st] = __builtin_bit_cast(half8_t, q[ab + (st >> 2) * 16]);
      }
    }
    // chunk c (of the unit in flight) from window slot SLOT
    auto compute_chunk = [&](auto SLOT, int c) {
      constexpr int slot = decltype(SLOT)::value;
      const int cofs = MT == 1 ? chunk_ofs(c + 1 < Q ? c + 1 : 0) : chunk_ofs(c);
      const uint4_t* p0 = s_a + cofs + ab0;
      const uint4_t* p1 = s_a + cofs + ab1;
      const uint4_t* p2 = s_a + cofs + ab2;
      const uint4_t* p3 = s_a + cofs + ab3;
      if constexpr (NSLAB > 1 && !moqe_is_log(BITS)) {
        // The first chunk of a further slab: its offset sum goes out now.  No branch (behind one
        // the compiler waits for every load in flight, which empties the window): where the
        // window is a multiple of a slab's chunks the slot says whether this chunk starts a slab,
        // elsewhere a select does; slab 0's sum is what the accumulators started from.
        constexpr bool by_slot = (W % CPS) == 0;
        if constexpr (!by_slot || (slot % CPS) == 0) {
          const int sl = c / CPS;
          const bool starts = by_slot || (c & (CPS - 1)) == 0;
#pragma unroll
          for (int mi = 0; mi < MT; ++mi) {
            float cs = 0.0f;
#pragma unroll
            for (int q = 1; q < NSLAB; ++q) cs = (starts && sl == q) ? corr[mi][q] : cs;
#pragma unroll
            for (int ni = 0; ni < NT; ++ni) acc[mi][ni] -= float4_t{cs, cs, cs, cs};
          }
        }
      }
      // the fragments of step s + 1 are read while step s is multiplied; nothing moves across
      // a step's end (without the fence the scheduler hoists a whole chunk's fragment reads to
      // its start, which costs more registers than there are)
      auto read_frags = [&](int s, half8_t (&a)[MT]) {
        const uint4_t* ps = (s & 3) == 0 ? p0 : (s & 3) == 1 ? p1 : (s & 3) == 2 ? p2 : p3;
#pragma unroll
        for (int mi = 0; mi < MT; ++mi) a[mi] = __builtin_bit_cast(half8_t, ps[mi * (16 * 32) + (s >> 2) * 16]);
      };
      half8_t a[2][MT];
      if constexpr (MT > 1) read_frags(0, a[0]);
#pragma unroll
      for (int s = 0; s < SC; ++s) {
        if constexpr (MT == 1) {
          a[s & 1][0] = afr[s];
          half8_t ahead[MT];
          read_frags(s, ahead);
          afr[s] = ahead[0];
        } else {
          if (s + 1 < SC) read_frags(s + 1, a[(s + 1) & 1]);
        }
#pragma unroll
        for (int ni = 0; ni < NT; ++ni) {
          half8_t w;
          if constexpr (BITS == 4) {
            w = unpack4(b_lo[slot][ni][s], uc);
          } else if constexpr (BITS == MOQE_LOG4) {
            w = unpack4_log(b_lo[slot][ni][s], uc);
          } else if constexpr (BITS == MOQE_LOG2) {
            const uint32_t d = b_lo[slot][ni][s >> 1];
            w = (s & 1) ? unpack2_log<1>(d, uc) : unpack2_log<0>(d, uc);
          } else if constexpr (BITS == MOQE_LOG3) {
            const uint32_t d = b_lo[slot][ni][s >> 1], hd = b_hi[slot][ni][s >> 2];
            w = (s & 3) == 0 ? unpack3_log<0>(d, hd, uc) : (s & 3) == 1 ? unpack3_log<1>(d, hd, uc)
              : (s & 3) == 2 ? unpack3_log<2>(d, hd, uc) : unpack3_log<3>(d, hd, uc);
          } else if constexpr (BITS == 2) {
            const uint32_t d = b_lo[slot][ni][s >> 1];
            w = (s & 1) ? unpack2<1>(d, uc) : unpack2<0>(d, uc);
          } else {
            const uint32_t d = b_lo[slot][ni][s >> 1], hd = b_hi[slot][ni][s >> 2];
            w = (s & 3) == 0 ? unpack3_sum<0>(d, hd, uc) : (s & 3) == 1 ? unpack3_sum<1>(d, hd, uc)
              : (s & 3) == 2 ? unpack3_sum<2>(d, hd, uc) : unpack3_sum<3>(d, hd, uc);
          }
#pragma unroll
          for (int mi = 0; mi < MT; ++mi)
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_16x16x32_f16(w, a[s & 1][mi], acc[mi][ni], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    // W chunks from cq on, each slot refilled as soon as it is used up: with chunk c + W of the
    // unit in flight, or (LAST) with one of the first W chunks of the wave's next unit
    auto window = [&](int cq, auto LASTC) {
      constexpr bool LAST = decltype(LASTC)::value;
      auto one = [&](auto SLOT) {
        constexpr int slot = decltype(SLOT)::value;
        compute_chunk(SLOT, cq + slot);
        if constexpr (LAST) load_chunk(SLOT, nxt, slot);
        else load_chunk(SLOT, cur, cq + slot + W);
      };
      one(std::integral_constant<int, 0>{});
      if constexpr (W > 1) one(std::integral_constant<int, 1>{});
      if constexpr (W > 2) one(std::integral_constant<int, 2>{});
      if constexpr (W > 3) one(std::integral_constant<int, 3>{});
      if constexpr (W > 4) one(std::integral_constant<int, 4>{});
      if constexpr (W > 5) one(std::integral_constant<int, 5>{});
      if constexpr (W > 6) one(std::integral_constant<int, 6>{});
      if constexpr (W > 7) one(std::integral_constant<int, 7>{});
    };

    while (grp < g1) {
      // the unit after this one, asked for now: its first chunks are requested while this
      // unit's last ones are multiplied
      int taken = 0;
      if (lane == 0) taken = __hip_atomic_fetch_add(&s_next, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      const int ng = uniform_i32(taken);
      unit_base(ng, nxt);
      // scales and biases of the unit's channels (4 per lane and column tile), used in the epilogue
      uint2_t sc2[NT], bi2[NT];
#pragma unroll
      for (int ni = 0; ni < NT; ++ni) {
        const int ct = grp * NT + ni;
        const int c0 = 16 * (ct < CT ? ct : 0) + 4 * g;
        sc2[ni] = *(const uint2_t*)(A.scales + (int64_t)t.e * N + c0);
        bi2[ni] = *(const uint2_t*)(A.bias + (int64_t)t.e * N + c0);
      }
#pragma unroll
      for (int mi = 0; mi < MT; ++mi)
#pragma unroll
        for (int ni = 0; ni < NT; ++ni) acc[mi][ni] = float4_t{-corr[mi][0], -corr[mi][0], -corr[mi][0], -corr[mi][0]};

      for (int cq = 0; cq < Q - W; cq += W) window(cq, std::false_type{});
      window(Q - W, std::true_type{});

      // ---- epilogue ----
      // The result tile is channels x tokens: lane (g, j) holds channels 4 g .. 4 g + 3 of the
      // column tile for token j of the token tile: four neighbouring fp16 outputs, one 8-byte
      // store, through a descriptor (no branch around a memory operation).
#pragma unroll
      for (int ni = 0; ni < NT; ++ni) {
        const int ct = grp * NT + ni;
        // (a column tile beyond the matrix: nowhere)
        const uint32_t c_off = ct < CT ? (uint32_t)(16 * ct + 4 * g) * 2u : NOWHERE;
        const float sc[4] = {(float)half_from_bits((uint16_t)sc2[ni].x), (float)half_from_bits((uint16_t)(sc2[ni].x >> 16)),
                             (float)half_from_bits((uint16_t)sc2[ni].y), (float)half_from_bits((uint16_t)(sc2[ni].y >> 16))};
        const float bi[4] = {(float)half_from_bits((uint16_t)bi2[ni].x), (float)half_from_bits((uint16_t)(bi2[ni].x >> 16)),
                             (float)half_from_bits((uint16_t)bi2[ni].y), (float)half_from_bits((uint16_t)(bi2[ni].y >> 16))};
#pragma unroll
        for (int mi = 0; mi < MT; ++mi) {
          const uint32_t off = (out_off[mi] | c_off) >= NOWHERE ? NOWHERE : out_off[mi] + c_off;
          float o[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) o[r] = fmaf(acc[mi][ni][r], sc[r], bi[r]);
          if constexpr (MODE == 0) {
            // max(0, .) as the median of (., 0, +inf): one operation
#pragma unroll
            for (int r = 0; r < 4; ++r) o[r] = __builtin_amdgcn_fmed3f(o[r], 0.0f, __builtin_inff());
          } else {
#pragma unroll
            for (int r = 0; r < 4; ++r) o[r] *= gt[mi];
            if (A.residual) {
              const uint2_t rs = __builtin_amdgcn_raw_buffer_load_b64(res_rsrc, off, 0, 0);
              o[0] += (float)half_from_bits((uint16_t)rs.x);
              o[1] += (float)half_from_bits((uint16_t)(rs.x >> 16));
              o[2] += (float)half_from_bits((uint16_t)rs.y);
              o[3] += (float)half_from_bits((uint16_t)(rs.y >> 16));
            }
          }
          uint2_t pk;
          pk.x = (uint32_t)half_to_bits((half_t)o[0]) | ((uint32_t)half_to_bits((half_t)o[1]) << 16);
          pk.y = (uint32_t)half_to_bits((half_t)o[2]) | ((uint32_t)half_to_bits((half_t)o[3]) << 16);
          __builtin_amdgcn_raw_buffer_store_b64(pk, out_rsrc, off, 0, 0);
        }
      }
      grp = ng;
#pragma unroll
      for (int ni = 0; ni < NT; ++ni) cur[ni] = nxt[ni];
    }
  };

  RsJob cur = next_job();
  RsRows cur_rows = row_offsets(cur.t);
  bool first_pair = true;
  while (cur.g0 < cur.g1) {
    RsJob nxt;
    RsRows nxt_rows;
    if (!first_pair) __syncthreads();  // every wave is done with the previous pair's rows
    first_pair = false;
    if constexpr (TM == 64) {
      const int mt = (cur.t.rows + 15) >> 4;
      if (mt == 4) run_pair(cur.t, cur.g0, cur.g1, cur_rows, &nxt, &nxt_rows, std::integral_constant<int, 4>{});
      else if (mt == 3) run_pair(cur.t, cur.g0, cur.g1, cur_rows, &nxt, &nxt_rows, std::integral_constant<int, 3>{});
      else if (mt == 2) run_pair(cur.t, cur.g0, cur.g1, cur_rows, &nxt, &nxt_rows, std::integral_constant<int, 2>{});
      else run_pair(cur.t, cur.g0, cur.g1, cur_rows, &nxt, &nxt_rows, std::integral_constant<int, 1>{});
    } else {
      run_pair(cur.t, cur.g0, cur.g1, cur_rows, &nxt, &nxt_rows, std::integral_constant<int, 1>{});
    }
    cur = nxt;
    cur_rows = nxt_rows;
  }
}

}  // namespace

// Two column tiles per unit and 8 waves (two per SIMD, up to 256 registers each) measured
// fastest for pairs of 64: 4 column tiles per unit, or 12 or 16 waves with a window of two chunks,
// were 5 to 15 % slower on the 4096-token layers (4 column tiles per unit also with the units
// handed out one by one: 46.7 against 44.6 us, so the LDS reads are not what the loop waits for).
template <int BITS, int W, int TM, int NT>
static void launch_shape(const PrefillArgs& a, int grid, hipStream_t stream) {
  constexpr int WAVES = 8;
  if (a.mode == 0)
    hipLaunchKernelGGL((moe_resident_kernel<BITS, NT, WAVES, W, 0, TM>), dim3((unsigned)grid), dim3(64 * WAVES), 0, stream, a);
  else
    hipLaunchKernelGGL((moe_resident_kernel<BITS, NT, WAVES, W, 1, TM>), dim3((unsigned)grid), dim3(64 * WAVES), 0, stream, a);
}

template <int BITS>
static void launch_bits(const PrefillArgs& a, int grid, hipStream_t stream) {
  constexpr int FB = moqe_field_bits(BITS);
  const int Q = a.K / (32 * (FB == 4 ? 4 : 8));
  if (a.K * 64 <= RS_LDS_ELEMS) {
    if (Q % 4 == 0) launch_shape<BITS, 4, 64, 2>(a, grid, stream);
    else launch_shape<BITS, 2, 64, 2>(a, grid, stream);
  } else {
    // (one token tile per pair leaves registers for a window twice as deep)
    // Units of a single column tile where units of two would leave waves without one: there are at
    // most T / 16 + E pairs (and at most T), each with N / 32 units of two column tiles.
    const int64_t pairs_max = a.T < a.T / 16 + a.E ? a.T : a.T / 16 + a.E;
    const bool narrow = pairs_max * ((a.N + 31) / 32) < (int64_t)grid * 8;
    if (Q % 8 == 0) {
      if (narrow) launch_shape<BITS, 8, 16, 1>(a, grid, stream);
      else launch_shape<BITS, 8, 16, 2>(a, grid, stream);
    } else if (Q % 4 == 0) {
      launch_shape<BITS, 4, 16, 2>(a, grid, stream);
    } else {
      launch_shape<BITS, 2, 16, 2>(a, grid, stream);
    }
  }
}

bool moqe_resident_supported(int bits, int64_t K, int64_t N) {
  const int fb = moqe_field_bits(bits);
  if (fb != 2 && fb != 3 && fb != 4) return false;
  const int kc = fb == 4 ? 128 : 256;
  // an even number of packed chunks per column tile: the window holds two or four
  return K >= 256 && K <= RS_MAX_K && (K % (2 * kc)) == 0 && N >= 16 && (N % 16) == 0;
}

hipError_t moqe_launch_resident(const PrefillArgs& a, int num_cus, hipStream_t stream) {
  // (byte offsets of the output rows are 32-bit, and offsets from 2^31 on mean "nowhere")
  if (a.E > RS_MAX_E || (int64_t)a.T * a.N * 2 >= (1ll << 31)) return hipErrorInvalidValue;
  int grid = num_cus & ~7;  // one workgroup per compute unit, a multiple of the 8 XCDs
  if (grid < 8) grid = 8;
  switch (a.bits) {
    case 4: launch_bits<4>(a, grid, stream); break;
    case 3: launch_bits<3>(a, grid, stream); break;
    case 2: launch_bits<2>(a, grid, stream); break;
    case MOQE_LOG4: launch_bits<MOQE_LOG4>(a, grid, stream); break;
    case MOQE_LOG3: launch_bits<MOQE_LOG3>(a, grid, stream); break;
    case MOQE_LOG2: launch_bits<MOQE_LOG2>(a, grid, stream); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}
