// Offline channel-wise absmax quantization and dense bit packing
// (paper App. A "Linear quantization with absolute maximum", App. C fp16 scales; also App. A's
// "Log-scale quantization" as a second codec), plus the inverse of the packing for tests.
#include "moqe_dev.h"
#include "moqe_kernels.h"

namespace {

// Smallest fp16 bit pattern whose value is >= v (v finite, >= 0).  One rounding,
// toward +inf, done in exact fp64 steps (scaling by powers of two, ceil).
__device__ inline uint16_t half_bits_round_up(double v) {
  if (!(v > 0.0)) return 0;
  if (v > 65504.0) return 0x7BFF;  // beyond fp16: undefined input, saturate
  const double two24 = 16777216.0;
  if (v < 6.103515625e-05) {  // below 2^-14: subnormal grid of 2^-24
    double n = ceil(v * two24);
    return (uint16_t)n;  // n == 1024 is exactly the smallest normal's pattern
  }
  int e = ilogb(v);  // v = f * 2^e, f in [1,2)
  double f = scalbn(v, -e);
  int mant = (int)ceil((f - 1.0) * 1024.0);
  if (mant == 1024) {
    mant = 0;
    e += 1;
  }
  int be = e + 15;
  if (be >= 31) return 0x7BFF;
  return (uint16_t)((be << 10) | mant);
}

__device__ inline int quantize_one(float w, double s, int lo, int hi) {
  if (!(s > 0.0)) return 0;
  double r = rint((double)w / s);  // IEEE fp64 divide, ties to even
  r = r < (double)lo ? (double)lo : r;
  r = r > (double)hi ? (double)hi : r;
  return (int)r;
}

// Log-scale code of one weight (App. A): sign bit, then the exponent Q = ceil(log2(2T/3)) of
// T = clip(|w|/s, 2^(1-2^(b-1)), 1) counted from its lowest value.  Q is the smallest integer
// with |w| <= 1.5 * 2^Q * s; the right-hand side is exact in fp64 (s is an fp16 number), so
// no quotient or logarithm is rounded.  The printed clip bounds are read as that interval.
__device__ inline uint32_t log_code_one(float w, double s, int bits) {
  if (!(s > 0.0)) return 0u;
  const int half = 1 << (bits - 1), q_lo = 1 - half;
  const double mag = fabs((double)w);
  int expo = 0;
  while (expo > q_lo && mag <= 1.5 * scalbn(s, expo - 1)) --expo;
  return (uint32_t)((w < 0.0f ? half : 0) + (expo - q_lo));
}

// s = 2 max|A_:,n| / (2^b - 1) (log-scale codec: s = max|A_:,n|), stored fp16 rounded up.  A workgroup takes 256 neighbouring
// channels of one expert: a lane owns 4 of them (16-byte loads, a wave reads 1 KiB per row), the
// 4 waves split the K rows and keep 8 loads in flight each; the partial maxima meet in LDS.
__global__ __launch_bounds__(256) void scale_kernel(const float* __restrict__ w, int64_t E, int K, int N, int bits,
                                                     int codec, uint16_t* __restrict__ scales) {
  __shared__ float4_t s_max[4][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nblocks = (N + 255) / 256;
  const int64_t e = blockIdx.x / nblocks;
  const int n0 = (int)(blockIdx.x % nblocks) * 256 + 4 * lane;
  float4_t m = {0.0f, 0.0f, 0.0f, 0.0f};
  if (n0 < N) {  // N is a multiple of 16, so the lane's 4 channels are all there
    const float* col = w + e * (int64_t)K * N + n0;
    const int k_begin = (int)((int64_t)K * wave / 4), k_end = (int)((int64_t)K * (wave + 1) / 4);
    int k = k_begin;
    for (; k + 8 <= k_end; k += 8) {
      float4_t v[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = __builtin_nontemporal_load((const float4_t*)(col + (int64_t)(k + i) * N));
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        m.x = fmaxf(m.x, fabsf(v[i].x));
        m.y = fmaxf(m.y, fabsf(v[i].y));
        m.z = fmaxf(m.z, fabsf(v[i].z));
        m.w = fmaxf(m.w, fabsf(v[i].w));
      }
    }
    for (; k < k_end; ++k) {
      const float4_t v = *(const float4_t*)(col + (int64_t)k * N);
      m.x = fmaxf(m.x, fabsf(v.x));
      m.y = fmaxf(m.y, fabsf(v.y));
      m.z = fmaxf(m.z, fabsf(v.z));
      m.w = fmaxf(m.w, fabsf(v.w));
    }
  }
  s_max[wave][lane] = m;
  __syncthreads();
  if (wave == 0 && n0 < N) {
    for (int q = 1; q < 4; ++q) {
      const float4_t o = s_max[q][lane];
      m.x = fmaxf(m.x, o.x);
      m.y = fmaxf(m.y, o.y);
      m.z = fmaxf(m.z, o.z);
      m.w = fmaxf(m.w, o.w);
    }
    uint16_t* out = scales + e * N + n0;
    if (bits == 16) {  // unquantized: the stored values are the weights themselves, scale 1
      out[0] = out[1] = out[2] = out[3] = 0x3C00;
      return;
    }
    if (codec == MOQE_CODEC_LOG) {
      out[0] = half_bits_round_up((double)m.x);
      out[1] = half_bits_round_up((double)m.y);
      out[2] = half_bits_round_up((double)m.z);
      out[3] = half_bits_round_up((double)m.w);
      return;
    }
    const double den = (double)((1 << bits) - 1);
    out[0] = half_bits_round_up((2.0 * (double)m.x) / den);
    out[1] = half_bits_round_up((2.0 * (double)m.y) / den);
    out[2] = half_bits_round_up((2.0 * (double)m.z) / den);
    out[3] = half_bits_round_up((2.0 * (double)m.w) / den);
  }
}

// Tensor-wise scale: every channel of a matrix gets the largest channel scale.  The fp16
// round-up is monotone, so the largest stored channel scale is the stored scale of the matrix
// maximum; positive fp16 numbers order like their bit patterns.  One workgroup per matrix.
__global__ __launch_bounds__(256) void tensor_scale_kernel(uint16_t* __restrict__ scales, int N) {
  __shared__ uint16_t s_max[256];
  uint16_t* row = scales + (int64_t)blockIdx.x * N;
  uint16_t m = 0;
  for (int n = threadIdx.x; n < N; n += 256) m = row[n] > m ? row[n] : m;
  s_max[threadIdx.x] = m;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off && s_max[threadIdx.x + off] > s_max[threadIdx.x]) s_max[threadIdx.x] = s_max[threadIdx.x + off];
    __syncthreads();
  }
  m = s_max[0];
  for (int n = threadIdx.x; n < N; n += 256) row[n] = m;
}

// One thread per packed 32-bit word.
__global__ __launch_bounds__(256) void pack_kernel(const float* __restrict__ w, const uint16_t* __restrict__ scales,
                                                    PackGeom g, int codec, int64_t E, uint32_t* __restrict__ codes) {
  const int64_t words_per_matrix = g.matrix_bytes / 4;
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= E * words_per_matrix) return;
  int64_t e = idx / words_per_matrix;
  int64_t D = idx % words_per_matrix;
  const int chunk_words = g.chunk_bytes / 4;
  int ci = (int)(D / chunk_words);
  int r = (int)(D % chunk_words);
  int c = ci / g.Q, p = ci % g.Q;
  int fbits = g.bits, vshift = 0, lane_words = g.lo_lane_bytes / 4;
  if (g.bits == 3) {
    fbits = 2;
    int lo_words = 64 * lane_words;
    if (r >= lo_words) {
      r -= lo_words;
      fbits = 1;
      vshift = 2;
      lane_words = g.hi_lane_bytes / 4;
    }
  }
  const int vmask = (1 << fbits) - 1;
  int slot = r / lane_words, word = r % lane_words;
  int grp = slot / 16, j = slot % 16;
  int n = 16 * c + j;
  const int per = 32 / fbits;
  const int z = 1 << (g.bits - 1);
  const int lo = -z, hi = z - 1;
  double s = (double)(float)half_from_bits(scales[e * g.N + n]);
  const float* wm = w + e * (int64_t)g.K * g.N;
  uint32_t val = 0;
  for (int t = 0; t < per; ++t) {
    int m = word * per + t;
    int s1 = m >> 3, i = m & 7;
    int k = 32 * (p * g.SC + s1) + 8 * grp + i;
    uint32_t u;
    if (g.bits == 16) {
      u = half_to_bits((half_t)wm[(int64_t)k * g.N + n]);  // one rounding, to nearest even
    } else if (codec == MOQE_CODEC_LOG) {
      u = log_code_one(wm[(int64_t)k * g.N + n], s, g.bits);
    } else {
      u = (uint32_t)(quantize_one(wm[(int64_t)k * g.N + n], s, lo, hi) + z);
    }
    val |= ((u >> vshift) & vmask) << (16 * (t & 1) + fbits * (t >> 1));
  }
  codes[idx] = val;
}

// The stored field u of code (k, n) of matrix e.
__device__ inline uint32_t stored_field(const uint32_t* __restrict__ codes, const PackGeom& g, int64_t e, int k, int n) {
  int c = n / 16, j = n % 16;
  int s = k / 32, grp = (k % 32) / 8, i = k % 8;
  int slot = 16 * grp + j;
  int p = s / g.SC, s1 = s % g.SC;
  int m = 8 * s1 + i;
  const uint32_t* base = codes + e * (g.matrix_bytes / 4) + (int64_t)(c * g.Q + p) * (g.chunk_bytes / 4);
  uint32_t u;
  if (g.bits != 3) {
    int per = 32 / g.bits;
    int word = m / per, t = m % per;
    uint32_t d = base[slot * (g.lo_lane_bytes / 4) + word];
    u = (d >> (16 * (t & 1) + g.bits * (t >> 1))) & ((1u << g.bits) - 1);
  } else {
    int word = m / 16, t = m % 16;
    uint32_t d = base[slot * (g.lo_lane_bytes / 4) + word];
    u = (d >> (16 * (t & 1) + 2 * (t >> 1))) & 3u;
    int hword = m / 32, ht = m % 32;
    uint32_t hd = base[64 * (g.lo_lane_bytes / 4) + slot * (g.hi_lane_bytes / 4) + hword];
    u |= ((hd >> (16 * (ht & 1) + (ht >> 1))) & 1u) << 2;
  }
  return u;
}

// One thread per code: packed layout -> int8 [E,K,N].
__global__ __launch_bounds__(256) void unpack_kernel(const uint32_t* __restrict__ codes, PackGeom g, int64_t E,
                                                      int8_t* __restrict__ q_out) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t per_matrix = (int64_t)g.K * g.N;
  if (idx >= E * per_matrix) return;
  int64_t e = idx / per_matrix;
  int64_t rem = idx % per_matrix;
  const uint32_t u = stored_field(codes, g, e, (int)(rem / g.N), (int)(rem % g.N));
  q_out[idx] = (int8_t)((int)u - (1 << (g.bits - 1)));
}

// One thread per code: A' = P s 2^Q of a log-scale code as fp32, by adding Q to the exponent
// field of s (an fp16 number is a normal fp32 number, and Q >= -7 keeps it one) and setting
// the sign bit.  s = 0 stays 0.
__global__ __launch_bounds__(256) void dequantize_log_kernel(const uint32_t* __restrict__ codes,
                                                              const uint16_t* __restrict__ scales, PackGeom g,
                                                              int64_t E, float* __restrict__ w_out) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t per_matrix = (int64_t)g.K * g.N;
  if (idx >= E * per_matrix) return;
  int64_t e = idx / per_matrix;
  int64_t rem = idx % per_matrix;
  const int n = (int)(rem % g.N);
  const uint32_t u = stored_field(codes, g, e, (int)(rem / g.N), n);
  const int half = 1 << (g.bits - 1);
  const int expo = (int)(u & (uint32_t)(half - 1)) + 1 - half;  // Q <= 0
  uint32_t v = __builtin_bit_cast(uint32_t, (float)half_from_bits(scales[e * g.N + n]));
  if (v != 0u) v = (v - ((uint32_t)(-expo) << 23)) | ((u & (uint32_t)half) ? 0x80000000u : 0u);
  w_out[idx] = __builtin_bit_cast(float, v);
}

}  // namespace

hipError_t moqe_launch_quantize(const float* w, int64_t E, const PackGeom& g, void* codes, uint16_t* scales,
                                bool tensor_scale, int codec, hipStream_t stream) {
  const int64_t blocks = E * ((g.N + 255) / 256);
  hipLaunchKernelGGL(scale_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, w, E, g.K, g.N, g.bits, codec, scales);
  if (tensor_scale && g.bits != 16)
    hipLaunchKernelGGL(tensor_scale_kernel, dim3((unsigned)E), dim3(256), 0, stream, scales, g.N);
  int64_t words = E * (g.matrix_bytes / 4);
  hipLaunchKernelGGL(pack_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, stream, w, scales, g, codec,
                     E, (uint32_t*)codes);
  return hipGetLastError();
}

hipError_t moqe_launch_unpack(const void* codes, int64_t E, const PackGeom& g, int8_t* q_out, hipStream_t stream) {
  int64_t n = E * (int64_t)g.K * g.N;
  hipLaunchKernelGGL(unpack_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, (const uint32_t*)codes, g,
                     E, q_out);
  return hipGetLastError();
}

hipError_t moqe_launch_dequantize_log(const void* codes, const uint16_t* scales, int64_t E, const PackGeom& g,
                                      float* w_out, hipStream_t stream) {
  int64_t n = E * (int64_t)g.K * g.N;
  hipLaunchKernelGGL(dequantize_log_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream,
                     (const uint32_t*)codes, scales, g, E, w_out);
  return hipGetLastError();
}
