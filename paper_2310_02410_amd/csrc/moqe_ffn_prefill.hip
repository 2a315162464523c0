// Expert FFN contraction for segments with many tokens: a dense tiled contraction on the
// matrix cores (paper Sec. 2.1 two-layer FFN, App. A dequantization A' = Q s), used where
// an expert has enough tokens for the arithmetic, not the weight bytes, to set the time.
//
//   out[rows of expert e, n] = epilogue( sum_k a[row, k] * (Q_e[k, n] * s_e[n]) + b_e[n] )
//
// Work decomposition
//   pair = (expert e, tile of 64 of its tokens), found on device from seg_offsets; only
//          experts with at least min_tokens tokens have pairs (the decode kernel takes the rest)
//   workgroup = (pair, block of output channels), 4 waves side by side along the channels;
//          every wave owns all 64 tokens of the tile, so a weight fragment is unpacked once
//          for four token tiles.  Two shapes:
//          PF_NT = 4: 256 channels, 64 per wave (4 x 4 accumulator tiles of
//                  v_mfma_f32_16x16x32_f16), 2 workgroups per compute unit - launches with
//                  enough tiles for several full rounds
//          PF_NT = 2: 128 channels, 32 per wave (4 x 2 tiles), 3 workgroups per compute unit -
//                  narrow matrices and smaller launches, so that the grid still fills the chip
//          PF_NT = 1: 64 channels, 16 per wave - launches with fewer 64 x 128 tiles than the
//                  chip has places
//   The grid is persistent; a workgroup walks over its share of the tiles.
//   K runs in staged blocks of 128 rows:
//     - the block's 64 token rows are staged in LDS by loads that go from global memory
//       straight into LDS (buffer_load ... lds, 16 bytes per lane, no registers in between),
//       three buffers deep and two blocks ahead; a row's 16-byte pieces are stored XOR-swizzled
//       by the row number, so that the fragment reads are conflict-free without padding; every
//       wave reads its A fragments from there;
//     - each wave loads the packed chunk (128 rows for int4, 256 for int2/int3) of each of its
//       column tiles with one 16-byte load per lane (the packed layout is already in B-operand
//       order), one chunk ahead, and dequantizes in registers: the unpack of one B fragment is
//       amortized over the wave's token tiles, and the fragment never has to travel through LDS
//       because no other wave needs it;
//     - the stream of blocks runs on across tile boundaries, so a tile's first operands arrive
//       while the previous tile's results are being written.
//   The unpack brings every field down to the signed code exactly (one packed subtract per
//   register more than the decode kernel's unpack, which leaves exponent and zero-point offsets
//   in the K-sum and removes them afterwards: over a whole K of all-positive activations that
//   costs accuracy, and here the unpack is shared by several token tiles anyway).  The scale
//   multiplies the finished sum (see moqe_unpack.h).
#include "moqe_dev.h"
#include "moqe_kernels.h"
#include "moqe_unpack.h"

#include <type_traits>


namespace {

constexpr int PF_THREADS = 256;
constexpr int PF_TILE_M = 64;    // tokens per workgroup tile
constexpr int PF_KB = 128;       // rows of K staged in LDS at a time
constexpr int PF_WG_PER_CU = 3;  // persistent workgroups per compute unit
constexpr int PF_MAX_E = 1024;
// An expert's packed weights are read once per 64-token tile of that expert, by workgroups of
// one XCD: ordinary cached loads (the decode kernel's weights are read once and stream past L2).
constexpr int PF_B_NT = 0;
constexpr int PF_SEG_LDS = 128;  // segment starts are kept in LDS for up to this many experts

// The four token rows a lane stages per block: first their row numbers in `a`, then their byte
// offsets (members, not an array: they must stay in registers; a reload from scratch in front
// of every load would also wait for all loads in flight).
struct PfRowOff {
  uint32_t r0, r1, r2, r3;
};

struct PfTile {
  int e, cb, row0, rows;
  bool valid;
};

// PF_NT: column tiles (of 16 channels) per wave: 4, 2 or 1
template <int BITS, int PF_NT>
__global__ __launch_bounds__(PF_THREADS, (PF_NT == 4 || BITS == 16) ? 2 : PF_WG_PER_CU) void moe_prefill_kernel(PrefillArgs A) {
  constexpr int PF_MT = PF_TILE_M / 16;       // token tiles per wave: all of the tile's
  constexpr int PF_TILE_CT = 4 * PF_NT;       // column tiles per workgroup tile
  // A chunk here is what a wave fetches at a time for one column tile: one packed chunk (128
  // rows for int4, 256 for int2 / int3) or, where packed chunks are shorter (64 rows for int8,
  // 32 for unquantized fp16 weights, BITS = 16), the packed chunks of a staged block.
  constexpr int FB = moqe_field_bits(BITS);   // stored bits per weight (4-bit log-scale codes: 4)
  constexpr int SC = (FB == 4 || FB == 8 || FB == 16) ? 4 : 8;  // steps of 32 rows per chunk
  constexpr int PCH = FB == 16 ? 4 : FB == 8 ? 2 : 1;  // packed chunks per chunk
  constexpr int SUB = SC / 4;                 // staged K blocks per chunk
  constexpr int LO_BITS = FB == 3 ? 2 : FB;
  constexpr int LWC = (SC / PCH) * LO_BITS / 4;  // main-plane words per lane per packed chunk (4)
  constexpr int LW = LWC * PCH;               // ... per chunk
  constexpr int HW = FB == 3 ? SC / 4 : 0;    // 1-bit-plane words per lane per chunk
  constexpr int CHUNK_BYTES = 64 * SC * FB;
  constexpr int ROW_PIECES = PF_KB / 8;       // 16-byte pieces per staged row (256 bytes, no padding)
  constexpr int NBUF = 3;                     // staged blocks in LDS: one in use, two on their way
  constexpr int NLD = 4;                      // LDS-direct loads per wave and block (4 rows each)

  // piece p of row r lives at s_a[.][r][p ^ (r & 15)]
  __shared__ uint4_t s_a[NBUF][PF_TILE_M][ROW_PIECES];
  __shared__ int s_incl[PF_MAX_E];
  __shared__ int s_seg[PF_SEG_LDS];  // seg_offsets[0 .. E - 1] when E <= PF_SEG_LDS

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = uniform_i32(tid >> 6);
  const int wn = wave;  // this wave's place along the channels
  const int g = lane >> 4, j = lane & 15;
  const int E = A.E, K = A.K, N = A.N;
  const int G = (int)gridDim.x, bid = (int)blockIdx.x;

  // ---- inclusive prefix of token tiles per expert: pair index -> expert ----
  if (wave == 0) {
    int carry = 0;
    for (int eg = 0; eg < E; eg += 64) {
      const int e = eg + lane;
      int v = 0;
      if (e < E) {
        const int s0 = A.seg_offsets[e];
        const int n = A.seg_offsets[e + 1] - s0;
        v = n >= A.min_tokens ? (n + PF_TILE_M - 1) / PF_TILE_M : 0;
        if (E <= PF_SEG_LDS) s_seg[e] = s0;
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
  // Tiles are numbered pair-major (a pair's column blocks are consecutive).  Workgroups are
  // dealt to the 8 XCDs round-robin by their index, so workgroups bid = x (mod 8) share XCD x's
  // L2: XCD x takes the x-th eighth of the tiles, its workgroups walk through it side by side.
  // A pair's token rows and an expert's weights are then fetched into one L2 only, and are
  // still there when the neighbouring tiles ask for them.
  const int n_tiles = s_incl[E - 1] * A.n_cblocks;
  const int xcd = bid & 7, GX = G >> 3;
  const int t_begin = (int)((int64_t)n_tiles * xcd / 8), t_end = (int)((int64_t)n_tiles * (xcd + 1) / 8);
  const int t_first = t_begin + (bid >> 3);
  if (t_first >= t_end) return;

  const int CT = N >> 4;
  const int Q = K / (32 * SC);   // packed chunks per column tile
  const int TB = Q * SUB;        // staged blocks per tile
  const int64_t matrix_bytes = (int64_t)K * N * FB / 8;
  const uint32_t lane_lo = (uint32_t)lane * LWC * 4, lane_hi = (64u * LWC + (uint32_t)lane * HW) * 4;
  UnpackConsts<BITS> uc;
  uc.init();

  // Finds tile `tile` (pair, column block): all of it is uniform over the workgroup and, with
  // the segment starts in LDS, needs no global read.
  auto find = [&](int tile) -> PfTile {
    PfTile t;
    t.valid = tile < t_end;
    t.e = 0; t.cb = 0; t.row0 = 0; t.rows = 1;
    if (!t.valid) return t;
    const int p = tile / A.n_cblocks;
    t.cb = tile - p * A.n_cblocks;
    int lo = 0, hi = E - 1;
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (s_incl[mid] > p) hi = mid; else lo = mid + 1;
    }
    t.e = uniform_i32(lo);
    const int first = t.e > 0 ? s_incl[t.e - 1] : 0;
    int seg0, seg1;
    if (E <= PF_SEG_LDS) {
      seg0 = s_seg[t.e];
      seg1 = t.e + 1 < E ? s_seg[t.e + 1] : A.seg_offsets[E];
    } else {
      seg0 = A.seg_offsets[t.e];
      seg1 = A.seg_offsets[t.e + 1];
    }
    t.row0 = uniform_i32(seg0 + PF_TILE_M * (p - first));
    t.rows = uniform_i32(min(PF_TILE_M, seg1 - seg0 - PF_TILE_M * (p - first)));
    return t;
  };
  // descriptors of a tile's column tiles for this wave; past the matrix (or no tile): empty
  auto make_brs = [&](const PfTile& t, rsrc_t (&brs)[PF_NT]) {
#pragma unroll
    for (int ni = 0; ni < PF_NT; ++ni) {
      const int ct = t.cb * PF_TILE_CT + wn * PF_NT + ni;
      const bool ok = t.valid && ct < CT;
      const char* base = (const char*)A.codes + (int64_t)t.e * matrix_bytes + (int64_t)(ok ? ct : 0) * Q * CHUNK_BYTES;
      brs[ni] = make_rsrc(base, ok ? (uint32_t)Q * CHUNK_BYTES : 0u);
    }
  };

  uint32_t b_lo[2][PF_NT][LW];
  uint32_t b_hi[2][PF_NT][HW > 0 ? HW : 1];
  float4_t acc[PF_MT][PF_NT];

  auto load_b = [&](auto BUF, const rsrc_t (&brs)[PF_NT], int c) {
    constexpr int buf = decltype(BUF)::value;
#pragma unroll
    for (int ni = 0; ni < PF_NT; ++ni) {
#pragma unroll
      for (int pc = 0; pc < PCH; ++pc)
        load_words<LWC, PF_B_NT>(brs[ni], (uint32_t)c * CHUNK_BYTES + pc * (CHUNK_BYTES / PCH) + lane_lo,
                                 &b_lo[buf][ni][LWC * pc]);
      if constexpr (FB == 3) load_words<HW, PF_B_NT>(brs[ni], (uint32_t)c * CHUNK_BYTES + lane_hi, b_hi[buf][ni]);
    }
  };

  // Token rows: wave w stages rows 16 w .. 16 w + 15 of the tile with NLD loads of 4 rows each;
  // lane l of load i writes LDS piece (l & 15) of row 16 w + 4 i + (l >> 4), which under the
  // swizzle holds the row's piece (l & 15) ^ (row & 15).
  const rsrc_t a_rsrc = make_rsrc(A.a, (uint32_t)((int64_t)A.T * K * 2));
  static_assert(NLD == 4, "PfRowOff holds four rows");
  // Row numbers in `a` of the four rows this lane stages for tile t (FFN1: through perm, a
  // global read that is asked for at the start of the tile before, blocks before its first
  // use); the rows a ragged tile lacks repeat its last row (never stored).
  auto stage_row = [&](const PfTile& t, int i) -> uint32_t {
    const int sr = t.row0 + min(16 * wave + 4 * i + (lane >> 4), t.rows - 1);
    if (A.mode != 0) return (uint32_t)sr;
    return t.valid ? (uint32_t)A.perm[sr] : 0u;
  };
  auto stage_rows = [&](const PfTile& t) -> PfRowOff {
    return PfRowOff{stage_row(t, 0), stage_row(t, 1), stage_row(t, 2), stage_row(t, 3)};
  };
  auto row_offset = [&](uint32_t arow, int i) -> uint32_t {
    const int row = 4 * i + (lane >> 4);  // 16 wave + row is the row of the tile
    return arow * (uint32_t)K * 2u + (uint32_t)(((lane & 15) ^ (row & 15)) * 16);
  };
  auto row_offsets = [&](const PfRowOff r) -> PfRowOff {
    return PfRowOff{row_offset(r.r0, 0), row_offset(r.r1, 1), row_offset(r.r2, 2), row_offset(r.r3, 3)};
  };
  auto load_a = [&](const PfRowOff off, int blk, int buf) {
    const uint32_t kb = (uint32_t)blk * (PF_KB * 2);
    typedef __attribute__((address_space(3))) void* lds_ptr;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, (lds_ptr)&s_a[buf][16 * wave + 0][0], 16, off.r0 + kb, 0, 0, 0);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, (lds_ptr)&s_a[buf][16 * wave + 4][0], 16, off.r1 + kb, 0, 0, 0);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, (lds_ptr)&s_a[buf][16 * wave + 8][0], 16, off.r2 + kb, 0, 0, 0);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, (lds_ptr)&s_a[buf][16 * wave + 12][0], 16, off.r3 + kb, 0, 0, 0);
  };
  // this lane's fragment piece per step of a block: logical piece 4 s + g of a row with (row & 15) == j
  // = frag_base ^ (4 s): 4 s only has bits that g has not
  const int frag_base = g ^ j;

  // the four steps of staged block `sub` of the chunk held in B buffer BUF
  auto compute = [&](int abuf, auto BUF, auto SUBI) {
    constexpr int bbuf = decltype(BUF)::value;
    constexpr int sub = decltype(SUBI)::value;
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
      constexpr int s0 = 4 * sub;
      const int s = s0 + s4;  // step within the chunk (compile-time after unrolling)
      half8_t a[PF_MT];
#pragma unroll
      for (int mi = 0; mi < PF_MT; ++mi)
        a[mi] = __builtin_bit_cast(half8_t, s_a[abuf][16 * mi + j][frag_base ^ (4 * s4)]);
#pragma unroll
      for (int ni = 0; ni < PF_NT; ++ni) {
        half8_t w;
        if constexpr (BITS == 16) {
          w = frag_from_words(b_lo[bbuf][ni][4 * s], b_lo[bbuf][ni][4 * s + 1], b_lo[bbuf][ni][4 * s + 2],
                              b_lo[bbuf][ni][4 * s + 3]);
        } else if constexpr (BITS == 8) {
          w = unpack8_exact(b_lo[bbuf][ni][2 * s], b_lo[bbuf][ni][2 * s + 1], uc);
        } else if constexpr (BITS == 4) {
          w = unpack4_exact(b_lo[bbuf][ni][s], uc);
        } else if constexpr (BITS == MOQE_LOG4) {
          w = unpack4_log(b_lo[bbuf][ni][s], uc);
        } else if constexpr (BITS == MOQE_LOG2) {
          const uint32_t d = b_lo[bbuf][ni][s >> 1];
          w = (s & 1) ? unpack2_log<1>(d, uc) : unpack2_log<0>(d, uc);
        } else if constexpr (BITS == MOQE_LOG3) {
          const uint32_t d = b_lo[bbuf][ni][s >> 1], hd = b_hi[bbuf][ni][s >> 2];
          w = (s & 3) == 0 ? unpack3_log<0>(d, hd, uc) : (s & 3) == 1 ? unpack3_log<1>(d, hd, uc)
            : (s & 3) == 2 ? unpack3_log<2>(d, hd, uc) : unpack3_log<3>(d, hd, uc);
        } else if constexpr (BITS == 2) {
          const uint32_t d = b_lo[bbuf][ni][s >> 1];
          w = (s & 1) ? unpack2_exact<1>(d, uc) : unpack2_exact<0>(d, uc);
        } else {
          const uint32_t d = b_lo[bbuf][ni][s >> 1], hd = b_hi[bbuf][ni][s >> 2];
          w = (s & 3) == 0 ? unpack3_exact<0>(d, hd, uc) : (s & 3) == 1 ? unpack3_exact<1>(d, hd, uc)
            : (s & 3) == 2 ? unpack3_exact<2>(d, hd, uc) : unpack3_exact<3>(d, hd, uc);
        }
#pragma unroll
        for (int mi = 0; mi < PF_MT; ++mi)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_16x16x32_f16(w, a[mi], acc[mi][ni], 0, 0, 0);
      }
    }
  };

  // ---- the workgroup's tiles, as one continuous stream of staged blocks ----
  // While block t is multiplied, blocks t + 1 and t + 2 are on their way into the other two LDS
  // buffers and the next packed chunk into the other register buffer - also across the end of
  // a tile, so that the next tile's first operands arrive during this tile's epilogue.
  // LDS-direct loads are invisible to the compiler's wait insertion: the waits on them are
  // explicit.  Loads complete in order, so "all but the youngest NLD" means block t + 1 is in.
  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;
  constexpr int WAIT_ALL = 0x0F70;                 // s_waitcnt vmcnt(0)
  constexpr int WAIT_BUT_NLD = 0x0F70 | NLD;       // s_waitcnt vmcnt(NLD)
  PfTile cur = find(t_first);
  rsrc_t cur_brs[PF_NT], nxt_brs[PF_NT];
  make_brs(cur, cur_brs);
  PfRowOff cur_off = row_offsets(stage_rows(cur));
  load_b(I0{}, cur_brs, 0);
  load_a(cur_off, 0, 0);
  load_a(cur_off, 1, 1);
  __builtin_amdgcn_s_waitcnt(WAIT_ALL);
  __syncthreads();
  int gb = 0;                       // blocks done so far: block t of the stream lives in buffer t % NBUF
  const bool cross = (Q & 1) == 0;  // with an even chunk count the chunk stream crosses tiles too

  for (int it = 0; cur.valid; ++it) {
    const PfTile nxt = find(t_first + (it + 1) * GX);
    make_brs(nxt, nxt_brs);
    const PfRowOff nxt_rows = stage_rows(nxt);  // first needed two blocks before the tile's end
    // FFN2 writes by token, times the token's gate: the tokens of the rows this lane writes
    // are asked for now, their gates after the first chunk, both used in the epilogue
    int cur_tk[PF_MT];
    float cur_gt[PF_MT];
#pragma unroll
    for (int mi = 0; mi < PF_MT; ++mi) {
      const int row = 16 * mi + j;
      cur_tk[mi] = (A.mode != 0 && row < cur.rows) ? A.perm[cur.row0 + row] : 0;
      cur_gt[mi] = 1.0f;
    }
    // scales and biases of this tile's channels (4 per lane and column tile), asked for now and
    // used in the epilogue, by when they have long arrived
    uint2_t sc2[PF_NT], bi2[PF_NT];
#pragma unroll
    for (int ni = 0; ni < PF_NT; ++ni) {
      const int ct = cur.cb * PF_TILE_CT + wn * PF_NT + ni;
      const int c0 = 16 * (ct < CT ? ct : 0) + 4 * g;
      sc2[ni] = *(const uint2_t*)(A.scales + (int64_t)cur.e * N + c0);
      bi2[ni] = *(const uint2_t*)(A.bias + (int64_t)cur.e * N + c0);
    }
#pragma unroll
    for (int mi = 0; mi < PF_MT; ++mi)
#pragma unroll
      for (int ni = 0; ni < PF_NT; ++ni) acc[mi][ni] = float4_t{0, 0, 0, 0};

    auto do_chunk = [&](int c, auto BUF) {
      constexpr int bbuf = decltype(BUF)::value;
      using OTHER = std::integral_constant<int, 1 - bbuf>;
      if (c + 1 < Q) {
        load_b(OTHER{}, cur_brs, c + 1);
      } else if (bbuf == 1) {
        load_b(OTHER{}, nxt_brs, 0);  // first chunk of the next tile (empty descriptors if none)
      }
      auto do_block = [&](auto SUBI) {
        constexpr int sub = decltype(SUBI)::value;
        const int blk = c * SUB + sub;
        // block blk + 2 of the stream: this tile's, or the next tile's first or second block
        const int ahead = blk + 2;
        bool issued = true;
        if (ahead < TB) load_a(cur_off, ahead, (gb + 2) % NBUF);
        else if (nxt.valid) load_a(row_offsets(nxt_rows), ahead - TB, (gb + 2) % NBUF);
        else issued = false;
        compute(gb % NBUF, BUF, SUBI);
        if (issued) __builtin_amdgcn_s_waitcnt(WAIT_BUT_NLD);
        else __builtin_amdgcn_s_waitcnt(WAIT_ALL);
        __syncthreads();
        ++gb;
      };
      do_block(I0{});
      if constexpr (SUB == 2) do_block(I1{});
    };
    for (int c = 0; c < Q; c += 2) {
      do_chunk(c, I0{});
      if (c == 0 && A.mode != 0) {
#pragma unroll
        for (int mi = 0; mi < PF_MT; ++mi) cur_gt[mi] = A.gate[cur_tk[mi]];
      }
      if (c + 1 < Q) do_chunk(c + 1, I1{});
    }
    if (!cross && nxt.valid) load_b(I0{}, nxt_brs, 0);

    // ---- epilogue ----
    // The weights are the MFMA's first operand and the tokens its second, so the result tile is
    // channels x tokens: lane (g, j) holds channels 4 g .. 4 g + 3 of the column tile for token
    // j of the token tile - four neighbouring fp16 outputs, written with one 8-byte store.
    // element offset of this lane's output rows (T N < 2^31: checked by the caller); -1: no row
    int out_row[PF_MT];
#pragma unroll
    for (int mi = 0; mi < PF_MT; ++mi) {
      const int row = 16 * mi + j;
      out_row[mi] = row < cur.rows ? (A.mode == 0 ? cur.row0 + row : cur_tk[mi]) * N : -1;
    }
#pragma unroll
    for (int ni = 0; ni < PF_NT; ++ni) {
      const int ct = cur.cb * PF_TILE_CT + wn * PF_NT + ni;
      if (ct >= CT) continue;
      const int c0 = 16 * ct + 4 * g;
      const float sc[4] = {(float)half_from_bits((uint16_t)sc2[ni].x), (float)half_from_bits((uint16_t)(sc2[ni].x >> 16)),
                           (float)half_from_bits((uint16_t)sc2[ni].y), (float)half_from_bits((uint16_t)(sc2[ni].y >> 16))};
      const float bi[4] = {(float)half_from_bits((uint16_t)bi2[ni].x), (float)half_from_bits((uint16_t)(bi2[ni].x >> 16)),
                           (float)half_from_bits((uint16_t)bi2[ni].y), (float)half_from_bits((uint16_t)(bi2[ni].y >> 16))};
#pragma unroll
      for (int mi = 0; mi < PF_MT; ++mi) {
        if (out_row[mi] < 0) continue;
        float o[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) o[r] = fmaf(acc[mi][ni][r], sc[r], bi[r]);
        if (A.mode == 0) {
#pragma unroll
          for (int r = 0; r < 4; ++r) o[r] = fmaxf(o[r], 0.0f);
        } else {
#pragma unroll
          for (int r = 0; r < 4; ++r) o[r] *= cur_gt[mi];
          if (A.residual) {
            const uint2_t rs = *(const uint2_t*)(A.residual + out_row[mi] + c0);
            o[0] += (float)half_from_bits((uint16_t)rs.x);
            o[1] += (float)half_from_bits((uint16_t)(rs.x >> 16));
            o[2] += (float)half_from_bits((uint16_t)rs.y);
            o[3] += (float)half_from_bits((uint16_t)(rs.y >> 16));
          }
        }
        uint2_t pk;
        pk.x = (uint32_t)half_to_bits((half_t)o[0]) | ((uint32_t)half_to_bits((half_t)o[1]) << 16);
        pk.y = (uint32_t)half_to_bits((half_t)o[2]) | ((uint32_t)half_to_bits((half_t)o[3]) << 16);
        *(uint2_t*)(A.out + out_row[mi] + c0) = pk;
      }
    }
    cur = nxt;
#pragma unroll
    for (int ni = 0; ni < PF_NT; ++ni) cur_brs[ni] = nxt_brs[ni];
    cur_off = row_offsets(nxt_rows);
  }
}

}  // namespace

bool moqe_prefill_supported(int bits, int64_t K, int64_t N) {
  const int fb = moqe_field_bits(bits);
  const int kc = (fb == 4 || fb == 8 || fb == 16) ? 128 : 256;
  return (fb == 2 || fb == 3 || fb == 4 || fb == 8 || fb == 16) && K >= 256 && (K % kc) == 0 && N >= 16 && (N % 16) == 0;
}

template <int BITS>
static void launch_bits(const PrefillArgs& a, int64_t pairs, int num_cus, hipStream_t stream) {
  PrefillArgs args = a;
  const int CT = a.N / 16;
  // Both shapes give every wave all 64 tokens, so a weight fragment is unpacked once for four
  // token tiles.  64 x 256 tiles (64 channels per wave, two workgroups per compute unit: the
  // 4 x 4 accumulator tiles need the registers) halve the token-row traffic per flop; 64 x 128
  // tiles (32 channels per wave, three workgroups per compute unit) make twice as many,
  // half-sized tiles.  The big shape pays once a launch has at least three full rounds of its
  // tiles (measured: +7 % at 8192 tokens, -10 % at 1536); below that the last, partly filled
  // round costs more than the traffic saves.
  // (fp16 weights hold 16 words per chunk and column tile: only the narrow shape has the registers)
  const bool wide = BITS != 16 && CT >= 128 && pairs * ((CT + 15) / 16) >= 3ll * 2 * num_cus;
  const int per_cu = (wide || BITS == 16) ? 2 : PF_WG_PER_CU;
  // A launch that cannot even fill the chip once with 64 x 128 tiles takes 64 x 64 ones (16
  // channels per wave): twice the workgroups to share the weight stream (fp16 experts at batch
  // 24, FFN2: 44.7 -> 34.2 us; no change where the launch was not short of workgroups).
  const bool small = !wide && pairs * ((CT + 7) / 8) < (int64_t)per_cu * num_cus;
  args.n_cblocks = wide ? (CT + 15) / 16 : small ? (CT + 3) / 4 : (CT + 7) / 8;
  int64_t grid = pairs * args.n_cblocks;  // upper bound on the tiles
  if (grid > (int64_t)per_cu * num_cus) grid = (int64_t)per_cu * num_cus;
  grid = grid < 8 ? 8 : (grid & ~(int64_t)7);  // a multiple of the 8 XCDs
  if constexpr (BITS != 16) {
    if (wide) {
      hipLaunchKernelGGL((moe_prefill_kernel<BITS, 4>), dim3((unsigned)grid), dim3(PF_THREADS), 0, stream, args);
      return;
    }
  }
  if (small)
    hipLaunchKernelGGL((moe_prefill_kernel<BITS, 1>), dim3((unsigned)grid), dim3(PF_THREADS), 0, stream, args);
  else
    hipLaunchKernelGGL((moe_prefill_kernel<BITS, 2>), dim3((unsigned)grid), dim3(PF_THREADS), 0, stream, args);
}

hipError_t moqe_launch_prefill(const PrefillArgs& a, int num_cus, hipStream_t stream) {
  // upper bound on the number of (expert, 64-token tile) pairs
  const int64_t with_pairs = a.min_tokens > 0 ? a.T / a.min_tokens : a.E;
  const int64_t pairs = a.T / PF_TILE_M + (with_pairs < a.E ? with_pairs : a.E);
  if (pairs <= 0) return hipSuccess;
  if (pairs * ((a.N / 16 + 3) / 4) >= (1ll << 31)) return hipErrorInvalidValue;
  switch (a.bits) {
    case 16: launch_bits<16>(a, pairs, num_cus, stream); break;
    case 8: launch_bits<8>(a, pairs, num_cus, stream); break;
    case 4: launch_bits<4>(a, pairs, num_cus, stream); break;
    case MOQE_LOG4: launch_bits<MOQE_LOG4>(a, pairs, num_cus, stream); break;
    case MOQE_LOG3: launch_bits<MOQE_LOG3>(a, pairs, num_cus, stream); break;
    case MOQE_LOG2: launch_bits<MOQE_LOG2>(a, pairs, num_cus, stream); break;
    case 3: launch_bits<3>(a, pairs, num_cus, stream); break;
    case 2: launch_bits<2>(a, pairs, num_cus, stream); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}
