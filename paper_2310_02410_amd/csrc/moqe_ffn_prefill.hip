// Expert FFN contraction for segments with many tokens: a dense tiled contraction on the
// matrix cores (paper Sec. 2.1 two-layer FFN, App. A dequantization A' = Q s), used where
// an expert has enough tokens for the arithmetic, not the weight bytes, to set the time.
//
//   out[rows of expert e, n] = epilogue( sum_k a[row, k] * (Q_e[k, n] * s_e[n]) + b_e[n] )
//
// Work decomposition
//   pair = (expert e, tile of 64 of its tokens), found on device from seg_offsets; only
//          experts with at least min_tokens tokens have pairs (the decode kernel takes the rest)
//   workgroup = (pair, block of 8 column tiles = 128 output channels), 4 waves as
//          2 token halves x 2 channel halves: a wave owns 32 tokens x 64 channels,
//          2 x 4 accumulator tiles of v_mfma_f32_16x16x32_f16
//   K runs in blocks of one packed chunk (128 rows for int4, 256 for int2/int3):
//     - the block's 64 token rows are staged in LDS (double buffered, loaded one block ahead
//       through registers) and every wave reads its A fragments from there;
//     - each wave loads the chunk of each of its 4 column tiles with one 16-byte load per lane
//       (the packed layout is already in B-operand order), one block ahead, and dequantizes in
//       registers: the unpack of one B fragment is amortized over the 2 token tiles, and the
//       fragment never has to travel through LDS because no other wave needs it.
//   The exponent / zero-point offsets the unpack leaves in the values are removed after the
//   K-sum through one extra MFMA per token tile and step against a constant fragment, the
//   scale multiplies the finished sum (see moqe_unpack.h).
#include "moqe_dev.h"
#include "moqe_kernels.h"
#include "moqe_unpack.h"

namespace {

constexpr int PF_THREADS = 256;
constexpr int PF_TILE_M = 64;   // tokens per workgroup
constexpr int PF_TILE_CT = 8;   // column tiles (of 16 channels) per workgroup
constexpr int PF_MT = 2;        // token tiles per wave
constexpr int PF_NT = 4;        // column tiles per wave
constexpr int PF_MAX_E = 1024;

template <int BITS>
__global__ __launch_bounds__(PF_THREADS, 2) void moe_prefill_kernel(PrefillArgs A) {
  constexpr int SC = BITS == 4 ? 4 : 8;       // steps of 32 rows per K block (= one packed chunk)
  constexpr int KC = 32 * SC;                 // rows of K per block
  constexpr int LO_BITS = BITS == 3 ? 2 : BITS;
  constexpr int LW = SC * LO_BITS / 4;        // main-plane words per lane per chunk (4)
  constexpr int HW = BITS == 3 ? SC / 4 : 0;  // 1-bit-plane words per lane per chunk
  constexpr int CHUNK_BYTES = 64 * SC * BITS;
  constexpr int ROW_PIECES = KC / 8 + 4;      // 16-byte pieces per staged row: data + 64 bytes of padding
  constexpr int NP = PF_TILE_M * (KC / 8) / PF_THREADS;  // pieces each thread moves per block

  __shared__ uint4_t s_a[2][PF_TILE_M][ROW_PIECES];
  __shared__ int s_incl[PF_MAX_E];
  __shared__ long long s_rowoff[PF_TILE_M];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = uniform_i32(tid >> 6);
  const int wm = wave & 1, wn = wave >> 1;
  const int g = lane >> 4, j = lane & 15;
  const int E = A.E, K = A.K, N = A.N;

  // ---- which pair is this workgroup's?  inclusive prefix of token tiles per expert ----
  if (wave == 0) {
    int carry = 0;
    for (int eg = 0; eg < E; eg += 64) {
      const int e = eg + lane;
      int v = 0;
      if (e < E) {
        const int n = A.seg_offsets[e + 1] - A.seg_offsets[e];
        v = n >= A.min_tokens ? (n + PF_TILE_M - 1) / PF_TILE_M : 0;
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
  const int P = s_incl[E - 1];
  const int p = (int)(blockIdx.x / (unsigned)A.n_cblocks);
  const int cb = (int)(blockIdx.x % (unsigned)A.n_cblocks);
  if (p >= P) return;  // the grid is an upper bound on the number of pairs
  int lo = 0, hi = E - 1;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (s_incl[mid] > p) hi = mid; else lo = mid + 1;
  }
  const int e = uniform_i32(lo);
  const int first = e > 0 ? s_incl[e - 1] : 0;
  const int seg0 = A.seg_offsets[e];
  const int n_e = A.seg_offsets[e + 1] - seg0;
  const int row0 = seg0 + PF_TILE_M * (p - first);
  const int rows = min(PF_TILE_M, n_e - PF_TILE_M * (p - first));

  // element offset of each token row in `a` (-1: no such row, reads as zero)
  if (tid < PF_TILE_M) {
    long long off = -1;
    if (tid < rows) off = (long long)(A.mode == 0 ? A.perm[row0 + tid] : row0 + tid) * K;
    s_rowoff[tid] = off;
  }
  __syncthreads();

  UnpackConsts<BITS> uc;
  uc.init();
  const int CT = N >> 4;
  const int Q = K / KC;  // K blocks = chunks per column tile
  const int64_t matrix_bytes = (int64_t)K * N * BITS / 8;
  // this wave's column tiles; a tile past the matrix gets an empty descriptor and loads nothing
  rsrc_t brs[PF_NT];
#pragma unroll
  for (int ni = 0; ni < PF_NT; ++ni) {
    const int ct = cb * PF_TILE_CT + wn * PF_NT + ni;
    const bool ok = ct < CT;
    const char* base = (const char*)A.codes + (int64_t)e * matrix_bytes + (int64_t)(ok ? ct : 0) * Q * CHUNK_BYTES;
    brs[ni] = make_rsrc(base, ok ? (uint32_t)Q * CHUNK_BYTES : 0u);
  }
  const uint32_t lane_lo = (uint32_t)lane * LW * 4, lane_hi = (64u * LW + (uint32_t)lane * HW) * 4;

  uint32_t b_lo[2][PF_NT][LW];
  uint32_t b_hi[2][PF_NT][HW > 0 ? HW : 1];
  uint4_t a_next[NP];

  auto load_b = [&](int buf, int kb) {
#pragma unroll
    for (int ni = 0; ni < PF_NT; ++ni) {
      load_words<LW>(brs[ni], (uint32_t)kb * CHUNK_BYTES + lane_lo, b_lo[buf][ni]);
      if constexpr (BITS == 3) load_words<HW>(brs[ni], (uint32_t)kb * CHUNK_BYTES + lane_hi, b_hi[buf][ni]);
    }
  };
  auto load_a = [&](int kb) {
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      const int q = tid + PF_THREADS * i;
      const int row = q / (KC / 8), pc = q % (KC / 8);
      const long long off = s_rowoff[row];
      a_next[i] = uint4_t{0, 0, 0, 0};
      if (off >= 0) a_next[i] = *(const uint4_t*)((const half_t*)A.a + off + (int64_t)kb * KC + pc * 8);
    }
  };
  auto store_a = [&](int buf) {
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      const int q = tid + PF_THREADS * i;
      s_a[buf][q / (KC / 8)][q % (KC / 8)] = a_next[i];
    }
  };

  float4_t acc[PF_MT][PF_NT];
  float4_t corr[PF_MT];
#pragma unroll
  for (int mi = 0; mi < PF_MT; ++mi) {
    corr[mi] = float4_t{0, 0, 0, 0};
#pragma unroll
    for (int ni = 0; ni < PF_NT; ++ni) acc[mi][ni] = float4_t{0, 0, 0, 0};
  }

  auto compute = [&](int abuf, int bbuf) {
#pragma unroll
    for (int s = 0; s < SC; ++s) {
      half8_t a[PF_MT];
#pragma unroll
      for (int mi = 0; mi < PF_MT; ++mi)
        a[mi] = __builtin_bit_cast(half8_t, s_a[abuf][32 * wm + 16 * mi + j][4 * s + g]);
#pragma unroll
      for (int ni = 0; ni < PF_NT; ++ni) {
        half8_t w;
        if constexpr (BITS == 4) {
          w = unpack4(b_lo[bbuf][ni][s], uc);
        } else {
          const uint32_t d = b_lo[bbuf][ni][s >> 1];
          w = (s & 1) ? unpack2<1>(d, uc) : unpack2<0>(d, uc);
        }
#pragma unroll
        for (int mi = 0; mi < PF_MT; ++mi)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[mi], w, acc[mi][ni], 0, 0, 0);
        if constexpr (BITS == 3) {
          const uint32_t hd = b_hi[bbuf][ni][s >> 2];
          const half8_t wh = (s & 3) == 0 ? unpack1x4<0>(hd, uc) : (s & 3) == 1 ? unpack1x4<1>(hd, uc)
                           : (s & 3) == 2 ? unpack1x4<2>(hd, uc) : unpack1x4<3>(hd, uc);
#pragma unroll
          for (int mi = 0; mi < PF_MT; ++mi)
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[mi], wh, acc[mi][ni], 0, 0, 0);
        }
      }
      // what the unpacked values carry besides the code: exponent bias and zero point
#pragma unroll
      for (int mi = 0; mi < PF_MT; ++mi)
        corr[mi] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[mi], bias_frag<BITS>(s & 1), corr[mi], 0, 0, 0);
    }
  };

  // ---- K loop: block kb + 1 is fetched while block kb is multiplied ----
  load_a(0);
  load_b(0, 0);
  store_a(0);
  __syncthreads();
  for (int kb = 0; kb < Q; kb += 2) {
    // even block: A buffer 0, B buffer 0; fetch into 1
    const bool more1 = kb + 1 < Q;
    if (more1) {
      load_a(kb + 1);
      load_b(1, kb + 1);
    }
    compute(0, 0);
    if (more1) store_a(1);
    __syncthreads();
    if (!more1) break;
    // odd block
    const bool more2 = kb + 2 < Q;
    if (more2) {
      load_a(kb + 2);
      load_b(0, kb + 2);
    }
    compute(1, 1);
    if (more2) store_a(0);
    __syncthreads();
  }

  // ---- epilogue: D lane (g, j), register r = token row 4 g + r of the tile, channel j ----
#pragma unroll
  for (int ni = 0; ni < PF_NT; ++ni) {
    const int ct = cb * PF_TILE_CT + wn * PF_NT + ni;
    if (ct >= CT) continue;
    const int col = 16 * ct + j;
    const float sc = (float)half_from_bits(A.scales[(int64_t)e * N + col]);
    const float bi = (float)half_from_bits(A.bias[(int64_t)e * N + col]);
#pragma unroll
    for (int mi = 0; mi < PF_MT; ++mi) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int row = 32 * wm + 16 * mi + 4 * g + r;
        if (row >= rows) continue;
        float o = fmaf(acc[mi][ni][r] - corr[mi][r], sc, bi);
        const int srow = row0 + row;
        if (A.mode == 0) {
          o = fmaxf(o, 0.0f);
          ((half_t*)A.out)[(int64_t)srow * N + col] = (half_t)o;
        } else {
          const int tk = A.perm[srow];
          float v = A.gate[tk] * o;
          const int64_t at = (int64_t)tk * N + col;
          if (A.residual) v += (float)((const half_t*)A.residual)[at];
          ((half_t*)A.out)[at] = (half_t)v;
        }
      }
    }
  }
}

}  // namespace

bool moqe_prefill_supported(int bits, int64_t K, int64_t N) {
  const int kc = bits == 4 ? 128 : 256;
  return (bits == 2 || bits == 3 || bits == 4) && K >= kc && (K % kc) == 0 && N >= 16 && (N % 16) == 0;
}

hipError_t moqe_launch_prefill(const PrefillArgs& a, hipStream_t stream) {
  PrefillArgs args = a;
  args.n_cblocks = (a.N / 16 + PF_TILE_CT - 1) / PF_TILE_CT;
  // upper bound on the number of (expert, 64-token tile) pairs
  const int64_t with_pairs = a.min_tokens > 0 ? a.T / a.min_tokens : a.E;
  const int64_t pairs = a.T / PF_TILE_M + (with_pairs < a.E ? with_pairs : a.E);
  const int64_t grid = pairs * args.n_cblocks;
  if (grid <= 0) return hipSuccess;
  if (grid >= (1ll << 31)) return hipErrorInvalidValue;
  switch (a.bits) {
    case 4: hipLaunchKernelGGL(moe_prefill_kernel<4>, dim3((unsigned)grid), dim3(PF_THREADS), 0, stream, args); break;
    case 3: hipLaunchKernelGGL(moe_prefill_kernel<3>, dim3((unsigned)grid), dim3(PF_THREADS), 0, stream, args); break;
    case 2: hipLaunchKernelGGL(moe_prefill_kernel<2>, dim3((unsigned)grid), dim3(PF_THREADS), 0, stream, args); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}
