// One expert contraction of a decode-sized batch (at most 64 tokens - 128 in pairs of 8 - and at
// most 128 experts) as a fused dequantize-in-register grouped GEMM, bound by the packed weight
// bytes it reads:
//
//   out[rows of expert e, n] = epilogue( sum_k a[row, k] * (Q_e[k, n] * s_e[n]) + b_e[n] )
// (paper Sec. 2.1 two-layer FFN, App. A dequantization A' = Q s; the per-channel scale
// multiplies the finished K-sum because it does not depend on k).
//
// A step of this size moves a few tens of MB and lasts microseconds, so the kernel is built
// around the latencies in front of and behind the weight stream rather than around throughput:
//   * every wave reads the routing tables itself, with a few loads into registers (one round
//     trip, no LDS staging, no workgroup barrier: lane t holds token t, and token t + 64 in the
//     instantiations for 65 to 128 tokens), and finds its work with ballots;
//   * a workgroup serves ONE pair (expert, tile of up to 4 - or, from 33 tokens on, 8 - of its
//     tokens): the persistent grid is split into as many equal groups as there are pairs and a
//     group's workgroups share the pair's column tiles, so a wave needs one set of token rows
//     for all its units;
//   * the token rows ride along with the weights: a CU's (and the memory fabric's) requests are
//     served in order, so rows asked for on their own arrive behind whatever weights other waves
//     asked for a moment earlier - measured: microseconds late, with all arithmetic left for the
//     end.  Instead a wave's first unit asks for the rows in blocks of 128 columns, each block
//     directly in front of the weight chunk that meets it (one 16-byte load per lane brings the
//     block of all four rows), parks a block in LDS when its chunk is due, and folds the K-sum of
//     the code offsets into the same steps; later units find the rows in LDS;
//   * a wave keeps a window of four chunks (4 KiB of packed codes) in flight and refills a slot
//     as soon as its chunk is unpacked.  A wave issues in order: while it is still queueing
//     requests it cannot start on data that has already arrived, and a CU takes only so many
//     requests at a time, so asking for a unit or two up front (measured) held every wave in the
//     request queue for microseconds and left the arithmetic for the end;
//   * from the first request to the last store the code is free of branches that hold memory
//     operations: loads and stores take an empty buffer descriptor or an out-of-range offset
//     where a unit, a row or a lane has nothing to do.  Loads return in order under one counter,
//     and only in such code does the compiler wait for exactly the chunk it is about to unpack
//     while the younger ones stay in flight.
//
// Work decomposition: unit = (pair, column tile of 16 channels); `R` waves of a workgroup share a
// unit along K (each owns 32*KS rows, partial sums meet in LDS), 4/R teams per workgroup.  Codes go
// straight from registers into v_mfma_f32_16x16x32_f16 as the B operand (see moqe_unpack.h), the
// token rows are the A operand (the rows of a fragment beyond the pair's 4 or 8 read a row of zeros).
#include <type_traits>

#include "moqe_dev.h"
#include "moqe_kernels.h"
#include "moqe_unpack.h"

namespace {

constexpr int WG_THREADS = 256;
constexpr int WG_WAVES = 4;
// Workgroups (of 4 waves) per CU.  Measured on the benchmark layer at 24 tokens, FFN1 / FFN2 /
// whole step: two 8.1 / 8.7 / 24.9 us at int4 (8.8 / 9.4 / 26.8 at int3, 7.1 / 7.3 / 21.8 at int2),
// three 8.7 / 10.2 / 25.9 (9.6 / 11.3 / 27.5, 7.4 / 8.5 / 22.1), four slower still: eight waves per CU
// with four chunks in flight each already cover the latency, and every further wave asks for
// its token rows and first chunks in the same opening burst.
#ifndef MOQE_SMALL_WG_PER_CU
#define MOQE_SMALL_WG_PER_CU 2
#endif
constexpr int MIN_WAVES = MOQE_SMALL_WG_PER_CU;  // workgroups per CU the register and LDS budgets are sized for
#ifndef MOQE_SMALL_WINDOW
#define MOQE_SMALL_WINDOW 4
#endif
// Chunks (1 KiB of packed codes, 1.5 KiB for 3-bit codes) a wave has in flight at most.  A wave
// issues in order: while it is still queueing requests it cannot start on data that is already
// there, so asking for everything up front leaves the arithmetic for the end; a window that
// just covers the latency keeps request and arithmetic going side by side.
constexpr int MAX_WINDOW = MOQE_SMALL_WINDOW;
// (the window divides the chunks of a unit, so that a chunk's slot is known at compile time)
// (3-bit codes: a chunk is two loads, 1.5 KiB, and covers 8 steps with two MFMAs each - a window
// of two measured faster than four: C1 FFN1 8.55 against 8.85 us, FFN2 8.7 against 9.45)
constexpr int window_chunks(int nch, int field_bits) {
  const int most = field_bits == 3 ? (MAX_WINDOW < 2 ? MAX_WINDOW : 2) : MAX_WINDOW;
  int w = nch < most ? nch : most;
  while (nch % w) --w;
  return w;
}
constexpr uint32_t NOWHERE = 0x80000000u;  // a buffer offset beyond every descriptor: loads give 0, stores vanish

__device__ inline int read_lane(int v, int l) { return __builtin_amdgcn_readlane(v, l); }
__device__ inline float read_lane(float v, int l) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), l));
}

// Packed words of the chunks in flight (WIN slots) as one lane holds them.
template <int BITS, int KS, int WIN>
struct WindowWords {
  using S = Shape<BITS, KS>;
  uint32_t lo[WIN * S::LW];
  uint32_t hi[S::FB == 3 ? WIN * S::HW : 1];
};

// What a wave knows about a unit besides its packed words.
struct Unit {
  bool active;       // (wave-uniform) an inactive unit loads nothing and stores nothing
  int col;           // column tile
  rsrc_t codes;      // this wave's K-slice of the unit's packed words (empty when inactive)
  uint16_t sc, bi;   // fp16 scale and bias of the lane's channel
  uint16_t res[4];   // MODE 1: residual of the lane's channel for the lane's four rows of the pair (0 without one)
};

// MODE 0: rows of `a` by token (through perm), out = relu(.) by sorted position (FFN1 -> h)
// MODE 1: rows of `a` by sorted position, out = gate * (.) (+ residual) by token (FFN2 -> y)
// TR: token rows of a pair, 4 or 8.  With 8 an expert's weights are streamed once per eight of
// its tokens instead of once per four; the parked rows then take twice the LDS, which leaves
// room for two workgroups per CU instead of three.
// XT: tokens the routing tables in registers cover, 64 (one register per table) or 128 (two).
template <int BITS, int KS, int MODE, int TR, int XT = 64>
__global__ __launch_bounds__(WG_THREADS, TR == 4 ? MIN_WAVES : 2) void moe_decode_small_kernel(SmallDecodeArgs A) {
  static_assert(XT == 64 || XT == 128, "one or two registers per routing table");
  constexpr int TILE_ROWS = TR;
  constexpr int RQ = TR / 4;  // row quads: lanes 16 q .. 16 q + 15 hold the results of rows 4 q .. 4 q + 3
  using S = Shape<BITS, KS>;
  constexpr int WIN = window_chunks(S::NCH, S::FB);  // chunks in flight
  using Words = WindowWords<BITS, KS, WIN>;
  constexpr int PIECES = KS * 4;          // 16-byte pieces of a row slice (8 columns each)
  constexpr int ROW_PIECES = PIECES + 4;  // parked row, padded by 64 bytes against bank conflicts
  constexpr int ZERO_ROW = WG_WAVES * TILE_ROWS;
  // token rows travel in blocks of (up to) 4 steps = 128 columns of all four rows: 16 lanes per row
  constexpr int BLK_PER_CHUNK = S::SC >= 4 ? S::SC / 4 : 1;
  constexpr int BLK_STEPS = S::SC / BLK_PER_CHUNK;
  constexpr int BLK_PIECES = BLK_STEPS * 4;  // pieces of one row in a block
  constexpr int NBLK = S::NCH * BLK_PER_CHUNK;
  constexpr uint32_t UNIT_BYTES = S::NCH * S::CHUNK_WORDS * 4;

  __shared__ uint4_t s_x[WG_WAVES * TILE_ROWS + 1][ROW_PIECES];
  __shared__ float4_t s_red[2][WG_WAVES][16 * RQ];

  UnpackConsts<BITS> uc;
  uc.init();
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = uniform_i32(tid >> 6);
  const int grp = lane >> 4;  // MFMA row group (k sub-block for A/B, token quad for D)
  const int j = lane & 15;    // token row for A, channel for B and D
  const int E = A.E, T = A.T, N = A.N, R = A.ksplit;
  const int K = 32 * KS * R;
  const int G = (int)gridDim.x, bid = (int)blockIdx.x;

  // ---- one round trip: the routing tables into registers (lane e: expert e and e + 64; lane t: token t) ----
  const rsrc_t seg_rs = make_rsrc(A.seg_offsets, (uint32_t)(E + 1) * 4u);
  const rsrc_t tok_rs = make_rsrc(A.perm, (uint32_t)T * 4u);
  const uint32_t l4 = (uint32_t)lane * 4u;
  int s0 = (int)__builtin_amdgcn_raw_buffer_load_b32(seg_rs, l4, 0, 0);
  int s1 = (int)__builtin_amdgcn_raw_buffer_load_b32(seg_rs, l4 + 4u, 0, 0);
  int s2 = (int)__builtin_amdgcn_raw_buffer_load_b32(seg_rs, l4 + 256u, 0, 0);
  int s3 = (int)__builtin_amdgcn_raw_buffer_load_b32(seg_rs, l4 + 260u, 0, 0);
  int pm = (int)__builtin_amdgcn_raw_buffer_load_b32(tok_rs, l4, 0, 0);
  int pm_hi = 0;  // (XT = 128: tokens 64 .. 127; past the batch the descriptor gives zeros)
  if constexpr (XT == 128) pm_hi = (int)__builtin_amdgcn_raw_buffer_load_b32(tok_rs, l4 + 256u, 0, 0);
  float gt = 0.0f, gt_hi = 0.0f;
  if constexpr (MODE == 1) {
    const rsrc_t gate_rs = make_rsrc(A.gate, (uint32_t)T * 4u);
    gt = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(gate_rs, l4, 0, 0));
    if constexpr (XT == 128) gt_hi = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(gate_rs, l4 + 256u, 0, 0));
  }
  // the zero row, while the tables travel (every wave writes the same zeros and reads only after
  // its own writes)
  {
#pragma unroll
    for (int i = 0; i < (PIECES + 63) / 64; ++i)
      if (64 * i + lane < PIECES) s_x[ZERO_ROW][64 * i + lane] = uint4_t{0, 0, 0, 0};
  }
  // (tables a caller made up are clamped into range: a wild row or token index must not become
  // a wild address)
  s0 = min(max(s0, 0), T);
  s2 = min(max(s2, 0), T);
  const int n0 = lane < E ? min(max(s1 - s0, 0), T - s0) : 0;
  const int n1 = lane + 64 < E ? min(max(s3 - s2, 0), T - s2) : 0;
  pm = min(max(pm, 0), T - 1);
  pm_hi = min(max(pm_hi, 0), T - 1);

  // ---- token tiles per expert, their prefix, the pair this workgroup serves ----
  const int t0 = (n0 >= A.min_tokens && n0 < A.max_tokens) ? (n0 + TILE_ROWS - 1) / TILE_ROWS : 0;
  const int t1 = (n1 >= A.min_tokens && n1 < A.max_tokens) ? (n1 + TILE_ROWS - 1) / TILE_ROWS : 0;
  const int incl0 = wave_inclusive_scan(t0);
  const int tot0 = read_lane(incl0, 63);
  int incl1 = tot0, P = tot0;
  if (E > 64) {  // (uniform)
    incl1 = tot0 + wave_inclusive_scan(t1);
    P = read_lane(incl1, 63);
  }
  if (P <= 0) return;
  const int wpp = max(1, G / P);  // workgroups per pair
  const int pair = bid / wpp, slot = bid - pair * wpp;
  if (pair >= P) return;
  // (lanes past the last expert hold the total, which no pair index reaches)
  int e = __popcll(__ballot(incl0 <= pair));
  if (E > 64) e += __popcll(__ballot(incl1 <= pair));
  e = uniform_i32(min(e, E - 1));
  const bool upper = e >= 64;
  const int el = e & 63;
  const int first = read_lane(upper ? incl1 - t1 : incl0 - t0, el);
  const int seg0 = read_lane(upper ? s2 : s0, el);
  const int n_e = read_lane(upper ? n1 : n0, el);
  const int m = pair - first;
  const int row0 = seg0 + TILE_ROWS * m;  // sorted position of the pair's first token
  const int rows_valid = min(TILE_ROWS, n_e - TILE_ROWS * m);
  int tk[TILE_ROWS];  // the pair's tokens
#pragma unroll
  for (int r = 0; r < TILE_ROWS; ++r) {
    // (rows past the pair's last one may read any lane: their token is never used)
    const int pos = row0 + r;
    tk[r] = read_lane(pm, pos & 63);
    if constexpr (XT == 128) tk[r] = (pos & 64) ? read_lane(pm_hi, pos & 63) : tk[r];
  }

  // ---- this workgroup's column tiles, this wave's place in it ----
  const int CT = N >> 4;
  const int cbase = CT / wpp, crem = CT - cbase * wpp;
  const int c_begin = slot * cbase + min(slot, crem);
  const int c_end = c_begin + cbase + (slot < crem ? 1 : 0);
  const int teams = WG_WAVES / R, team = wave / R, ks = wave - team * R;
  const int nl = (c_end - c_begin + teams - 1) / teams;  // units per team, the same for every wave
  if (nl <= 0) return;

  const int Q = K / (32 * S::SC);  // chunks per column tile
  const int64_t matrix_words = (int64_t)K * N * S::FB / 32;
  const uint32_t* const codes_e = A.codes + (int64_t)e * matrix_words + (int64_t)ks * S::NCH * S::CHUNK_WORDS;
  const rsrc_t scale_rs = make_rsrc((const uint16_t*)A.scales + (int64_t)e * N, (uint32_t)N * 2u);
  const rsrc_t bias_rs = make_rsrc((const uint16_t*)A.bias + (int64_t)e * N, (uint32_t)N * 2u);
  const rsrc_t res_rs = make_rsrc(A.residual, (MODE == 1 && A.residual) ? (uint32_t)T * (uint32_t)N * 2u : 0u);
  const rsrc_t out_rs = make_rsrc(A.out, (uint32_t)T * (uint32_t)N * 2u);

  auto make_unit = [&](int it) -> Unit {
    Unit u;
    u.col = c_begin + team + it * teams;
    u.active = it < nl && u.col < c_end;
    u.codes = make_rsrc(codes_e + (int64_t)u.col * Q * S::CHUNK_WORDS, u.active ? UNIT_BYTES : 0u);
    const uint32_t unit_nowhere = u.active ? 0u : NOWHERE;
    const uint32_t ch = ((uint32_t)(16 * u.col + j) * 2u) | unit_nowhere;
    u.sc = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(scale_rs, ch, 0, 0);
    u.bi = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(bias_rs, ch, 0, 0);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      u.res[r] = 0;
      if constexpr (MODE == 1) {
        int tok = tk[r];
        if constexpr (RQ == 2) tok = grp == 1 ? tk[4 + r] : tok;
        const uint32_t at = (((uint32_t)tok * (uint32_t)N + (uint32_t)(16 * u.col + j)) * 2u) | unit_nowhere |
                            ((grp < RQ && 4 * grp + r < rows_valid) ? 0u : NOWHERE);
        u.res[r] = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(res_rs, at, 0, 0);
      }
    }
    return u;
  };
  const uint32_t lane_lo = (uint32_t)lane * S::LW * 4, lane_hi = (64u * S::LW + (uint32_t)lane * S::HW) * 4;
  // chunk ch of a unit into window slot ch % WIN
  auto issue_chunk = [&](Words& b, rsrc_t r, int ch) {
    const int slot = ch % WIN;
    load_words<S::LW>(r, lane_lo + ch * S::CHUNK_WORDS * 4, &b.lo[slot * S::LW]);
    if constexpr (S::FB == 3) load_words<S::HW>(r, lane_hi + ch * S::CHUNK_WORDS * 4, &b.hi[slot * S::HW]);
  };

  // ---- the first requests: the first WIN chunks of the first unit, the token rows woven in ----
  // row block b: lane (r, p) = (lane / 16, lane % 16) asks for piece p of the block of row r; rows
  // the pair does not have and pieces past the block read as zeros
  const rsrc_t a_rs = make_rsrc(A.a, (uint32_t)T * (uint32_t)K * 2u);
  const int rr = lane >> 4, rp = lane & 15;
  uint32_t row_off[RQ];  // byte offset of this lane's piece of block 0, rows rr and (TR = 8) rr + 4
#pragma unroll
  for (int q = 0; q < RQ; ++q) {
    const int r = rr + 4 * q;
    int tok = tk[0];
#pragma unroll
    for (int i = 1; i < TILE_ROWS; ++i) tok = r == i ? tk[i] : tok;
    const uint32_t arow = MODE == 0 ? (uint32_t)tok : (uint32_t)(row0 + r);
    row_off[q] = (r < rows_valid && rp < BLK_PIECES) ? (arow * (uint32_t)K + (uint32_t)ks * (KS * 32) + (uint32_t)rp * 8u) * 2u
                                                      : NOWHERE;
  }
  uint4_t rows[WIN * BLK_PER_CHUNK * RQ];  // row blocks in flight, slot as for the chunks
  auto issue_rows = [&](int ch) {
#pragma unroll
    for (int bi = 0; bi < BLK_PER_CHUNK; ++bi) {
      const int b = ch * BLK_PER_CHUNK + bi;
#pragma unroll
      for (int q = 0; q < RQ; ++q)
        rows[((ch % WIN) * BLK_PER_CHUNK + bi) * RQ + q] =
            __builtin_amdgcn_raw_buffer_load_b128(a_rs, row_off[q] + (uint32_t)(b * BLK_STEPS * 64), 0, 0);
    }
  };
  // (the scheduling fences keep the requests in this order: the scale and bias, which the first
  // store waits for, in front of everything, each row block in front of its chunk)
  Unit uA = make_unit(0);
  __builtin_amdgcn_sched_barrier(0);
  Words wA;
#pragma unroll
  for (int ch = 0; ch < WIN; ++ch) {
    issue_rows(ch);
    issue_chunk(wA, uA.codes, ch);
    __builtin_amdgcn_sched_barrier(0);
  }

  // where the rows are parked: lane (grp, j) reads row j, k = 32 s + 8 grp .. +7 of this wave's slice
  uint4_t(*patch)[ROW_PIECES] = &s_x[wave * TILE_ROWS];
  const uint4_t* const afrag = j < TILE_ROWS ? &patch[j][grp] : &s_x[ZERO_ROW][grp];
  // offsets the unpacked values carry (exponent bias + zero point), summed against the rows by
  // the first unit (log-scale codes unpack to their exact values: nothing to remove)
  float4_t corr = {0, 0, 0, 0};

  // The lane's four result rows are rows 4 grp + r of the pair (lanes from 16 RQ on hold none):
  // their tokens and, MODE 1, gates
  int tkl[4];
  float g[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    tkl[r] = tk[r];
    if constexpr (RQ == 2) tkl[r] = grp == 1 ? tk[4 + r] : tk[r];
    g[r] = 1.0f;
    if constexpr (MODE == 1) {
      auto gate_of = [&](int tok) {  // (tok is uniform)
        float v = read_lane(gt, tok & 63);
        if constexpr (XT == 128) v = (tok & 64) ? read_lane(gt_hi, tok & 63) : v;
        return v;
      };
      g[r] = gate_of(tk[r]);
      if constexpr (RQ == 2) g[r] = grp == 1 ? gate_of(tk[4 + r]) : g[r];
    }
  }

  // Consumes unit `u` chunk by chunk; as soon as a chunk's words are unpacked its slot is
  // refilled with the chunk WIN further on, of this unit or of the next one, `nx`.  The wave's
  // first unit (FIRST) also parks the row blocks as they arrive, asks for the later ones in
  // front of their chunks, and accumulates `corr`.
  auto compute_unit = [&](auto first_tag, Words& b, const Unit& u, const Unit& nx) -> float4_t {
    constexpr bool FIRST = decltype(first_tag)::value;
    float4_t acc0 = {0, 0, 0, 0}, acc1 = {0, 0, 0, 0};
    float4_t c0 = {0, 0, 0, 0}, c1 = {0, 0, 0, 0};
#pragma unroll
    for (int ch = 0; ch < S::NCH; ++ch) {
      // A wave without this unit skips the arithmetic and nothing else: the reloads below are
      // issued on every path, so that all paths have the same history of memory operations.
      // (The flag is made opaque per chunk: were the chunks' tests merged into one, the
      // compiler would lay the unit out as two separate sequences of loads again.)
      int act = uniform_i32((int)u.active);
      asm volatile("" : "+s"(act));
      if constexpr (FIRST) {
#pragma unroll
        for (int bi = 0; bi < BLK_PER_CHUNK; ++bi) {
          const int blk = ch * BLK_PER_CHUNK + bi;
          if (rp < BLK_PIECES) {
#pragma unroll
            for (int q = 0; q < RQ; ++q)
              patch[rr + 4 * q][blk * BLK_PIECES + rp] = rows[((ch % WIN) * BLK_PER_CHUNK + bi) * RQ + q];
          }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      }
      if (act) {
#pragma unroll
        for (int s1 = 0; s1 < S::SC; ++s1) {
          const int s = ch * S::SC + s1;
          half8_t w;
          if constexpr (BITS == 4) {
            w = unpack4(b.lo[(ch % WIN) * S::LW + s1], uc);
          } else if constexpr (BITS == MOQE_LOG4) {
            w = unpack4_log(b.lo[(ch % WIN) * S::LW + s1], uc);
          } else if constexpr (BITS == MOQE_LOG3) {
            const uint32_t d = b.lo[(ch % WIN) * S::LW + (s1 >> 1)], hd = b.hi[(ch % WIN) * S::HW + (s1 >> 2)];
            w = (s1 & 3) == 0 ? unpack3_log<0>(d, hd, uc) : (s1 & 3) == 1 ? unpack3_log<1>(d, hd, uc)
              : (s1 & 3) == 2 ? unpack3_log<2>(d, hd, uc) : unpack3_log<3>(d, hd, uc);
          } else if constexpr (BITS == MOQE_LOG2) {
            const uint32_t d = b.lo[(ch % WIN) * S::LW + (s1 >> 1)];
            w = (s1 & 1) ? unpack2_log<1>(d, uc) : unpack2_log<0>(d, uc);
          } else {
            const uint32_t d = b.lo[(ch % WIN) * S::LW + (s1 >> 1)];
            w = (s1 & 1) ? unpack2<1>(d, uc) : unpack2<0>(d, uc);
          }
          const half8_t a = __builtin_bit_cast(half8_t, afrag[4 * s]);
          acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, w, acc0, 0, 0, 0);
          if constexpr (FIRST && !moqe_is_log(BITS)) {
            if (s & 1) c1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, bias_frag<BITS>(1), c1, 0, 0, 0);
            else c0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, bias_frag<BITS>(0), c0, 0, 0, 0);
          }
          if constexpr (BITS == 3) {  // the 1-bit plane as a second MFMA
            const uint32_t hd = b.hi[(ch % WIN) * S::HW + (s1 >> 2)];
            const half8_t wh = (s1 & 3) == 0 ? unpack1x4<0>(hd, uc) : (s1 & 3) == 1 ? unpack1x4<1>(hd, uc)
                             : (s1 & 3) == 2 ? unpack1x4<2>(hd, uc) : unpack1x4<3>(hd, uc);
            acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, wh, acc1, 0, 0, 0);
          }
        }
      }
      // the chunk's words are consumed: refill its slot WIN chunks ahead
      if (ch + WIN < S::NCH) {
        if constexpr (FIRST) issue_rows(ch + WIN);
        issue_chunk(b, u.codes, ch + WIN);
      } else {
        issue_chunk(b, nx.codes, ch + WIN - S::NCH);
      }
    }
    if constexpr (FIRST) corr = c0 + c1;
    return acc0 + acc1 - corr;
  };

  // where the pair's output rows start (bytes), and the top bit for rows the pair does not have
  // and for lanes that hold no result
  uint32_t out_row[4], out_row_nowhere[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    out_row[r] = (uint32_t)(MODE == 0 ? row0 + 4 * min(grp, RQ - 1) + r : tkl[r]) * (uint32_t)N * 2u;
    out_row_nowhere[r] = (grp < RQ && 4 * grp + r < rows_valid) ? 0u : NOWHERE;
  }
  const uint32_t lane_nowhere = (ks == 0 && lane < 16 * RQ) ? 0u : NOWHERE;

  int par = 0;
  auto finish_unit = [&](const Unit& u, float4_t part) {
    // the pair's rows are rows 0 .. TR - 1 of the MFMA tile: lanes 0 .. 16 RQ - 1 hold them, four
    // rows of one channel each
    if (R > 1) {  // (uniform; every wave of the workgroup runs the same number of units)
      if (lane < 16 * RQ) s_red[par][wave][lane] = part;
      __syncthreads();
      if (ks == 0 && lane < 16 * RQ) {
        for (int q = 1; q < R; ++q) part = part + s_red[par][wave + q][lane];
      }
      par ^= 1;
    }
    const float sc = (float)half_from_bits(u.sc);
    const float bi = (float)half_from_bits(u.bi);
    // one 2-byte store per row from the lanes of the team's first wave that hold rows; everything else is
    // sent NOWHERE by or-ing the top bit into the offset (the sums stay below 2^31)
    const uint32_t unit_off = ((uint32_t)(16 * u.col + j) * 2u) | (u.active ? lane_nowhere : NOWHERE);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      float o = fmaf(part[r], sc, bi);
      if constexpr (MODE == 0) {
        o = fmaxf(o, 0.0f);  // ReLU
      } else {
        o = fmaf(g[r], o, (float)half_from_bits(u.res[r]));
      }
      const uint16_t hb = half_to_bits((half_t)o);
      __builtin_amdgcn_raw_buffer_store_b16(hb, out_rs, (out_row[r] + unit_off) | out_row_nowhere[r], 0, 0);
    }
  };

  {
    const Unit nA = make_unit(1);
    const float4_t part = compute_unit(std::true_type{}, wA, uA, nA);
    finish_unit(uA, part);
    uA = nA;
  }
  for (int it = 1; it < nl; ++it) {
    const Unit nA = make_unit(it + 1);
    const float4_t part = compute_unit(std::false_type{}, wA, uA, nA);
    finish_unit(uA, part);
    uA = nA;
  }
}

// Workgroups per CU of one instantiation on the current device (asked once per device).
template <int BITS, int KS, int MODE, int TR, int XT>
int resident_per_cu() {
  static int cache[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 1;
  if (cache[dev] == 0) {
    constexpr int want = TR == 4 ? MIN_WAVES : 2;
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, moe_decode_small_kernel<BITS, KS, MODE, TR, XT>, WG_THREADS, 0) != hipSuccess ||
        n < 1)
      n = 1;
    cache[dev] = n > want ? want : n;
  }
  return cache[dev];
}

template <int BITS, int KS, int MODE, int TR, int XT = 64>
void launch_rows(const SmallDecodeArgs& a, int num_cus, hipStream_t stream) {
  hipLaunchKernelGGL((moe_decode_small_kernel<BITS, KS, MODE, TR, XT>), dim3(resident_per_cu<BITS, KS, MODE, TR, XT>() * num_cus),
                     dim3(WG_THREADS), 0, stream, a);
}

template <int BITS, int KS>
hipError_t launch_mode(const SmallDecodeArgs& a, int num_cus, hipStream_t stream) {
  // A persistent grid split evenly over the pairs.  (A grid sized for the largest possible number
  // of pairs with one unit per wave, handed out by the hardware as slots become free, measured
  // 1.5 us slower: every late workgroup pays the table round trip again.)
  // (pairs of 8 rows: slices of 32 steps only - the sizes the batches that gain from them have)
  if constexpr (KS == 32) {
    if (a.rows == 8 && a.T > 64) {
      if (a.mode == 0) launch_rows<BITS, KS, 0, 8, 128>(a, num_cus, stream);
      else launch_rows<BITS, KS, 1, 8, 128>(a, num_cus, stream);
      return hipGetLastError();
    }
    if (a.rows == 8) {
      if (a.mode == 0) launch_rows<BITS, KS, 0, 8>(a, num_cus, stream);
      else launch_rows<BITS, KS, 1, 8>(a, num_cus, stream);
      return hipGetLastError();
    }
  }
  if (a.T > 64) return hipErrorInvalidValue;  // (65 to 128 tokens: pairs of 8 rows only)
  if (a.mode == 0) launch_rows<BITS, KS, 0, 4>(a, num_cus, stream);
  else launch_rows<BITS, KS, 1, 4>(a, num_cus, stream);
  return hipGetLastError();
}

template <int BITS>
hipError_t launch_bits(const SmallDecodeArgs& a, int num_cus, hipStream_t stream) {
  switch (a.ksteps) {
    case 32: return launch_mode<BITS, 32>(a, num_cus, stream);
    case 24: return launch_mode<BITS, 24>(a, num_cus, stream);
    case 16: return launch_mode<BITS, 16>(a, num_cus, stream);
    case 8: return launch_mode<BITS, 8>(a, num_cus, stream);
    case 4: return launch_mode<BITS, 4>(a, num_cus, stream);
    case 2:
      if constexpr (moqe_field_bits(BITS) != 3) return launch_mode<BITS, 2>(a, num_cus, stream);
      return hipErrorInvalidValue;
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

bool moqe_decode_small_supported(int bits, int64_t T, int64_t E, int64_t K, int64_t N, int grid_min, int rows) {
  const int fb = moqe_field_bits(bits);
  if (fb != 2 && fb != 3 && fb != 4) return false;
  // (every pair needs a workgroup of its own, and there are at most T pairs)
  if (T < 1 || T > 128 || T > grid_min || E < 1 || E > 128) return false;
  // rows and outputs are addressed with 32-bit byte offsets inside their buffers
  if (T * K * 2 >= (1ll << 31) || T * N * 2 >= (1ll << 31)) return false;
  int ks = 0, r = 0;
  if (!moqe_pick_ksplit(bits > 100 ? fb : bits, K, &ks, &r)) return false;
  // (65 to 128 tokens: in pairs of 8 rows, which exist for wave slices of 32 steps)
  return T <= 64 || (rows == 8 && ks == 32);
}

hipError_t moqe_launch_decode_small(const SmallDecodeArgs& a, int num_cus, hipStream_t stream) {
  switch (a.bits) {
    case 4: return launch_bits<4>(a, num_cus, stream);
    case 3: return launch_bits<3>(a, num_cus, stream);
    case 2: return launch_bits<2>(a, num_cus, stream);
    case MOQE_LOG4: return launch_bits<MOQE_LOG4>(a, num_cus, stream);
    case MOQE_LOG3: return launch_bits<MOQE_LOG3>(a, num_cus, stream);
    case MOQE_LOG2: return launch_bits<MOQE_LOG2>(a, num_cus, stream);
    default: return hipErrorInvalidValue;
  }
}
