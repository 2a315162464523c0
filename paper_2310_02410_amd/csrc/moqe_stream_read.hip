// A plain streaming read: what this machine delivers for a launch that does nothing but pull a
// given number of bytes from HBM with 16-byte loads.  The expert kernels' achieved rate is
// reported next to this measured ceiling (and next to the nominal HBM peak).  Same launch shape
// as the decode kernels: a grid of three 4-wave workgroups per CU, every wave asking for its
// share in 1 KiB wave-loads, 12 in flight.
#include "moqe_dev.h"
#include "moqe_kernels.h"

namespace {

constexpr int IN_FLIGHT = 12;

__global__ __launch_bounds__(256) void stream_read_kernel(const uint4_t* __restrict__ src, uint32_t bytes,
                                                          uint32_t* __restrict__ sink) {
  // row = 1 KiB = one wave-load; wave q takes rows q, q + nwaves, ...; rows past the end fall
  // outside the buffer descriptor and read as zeros without touching memory
  const uint32_t nwaves = gridDim.x * 4u, q = blockIdx.x * 4u + (threadIdx.x >> 6);
  const uint32_t lane = threadIdx.x & 63u, n_rows = bytes >> 10;
  const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint4_t*>(src), 0, bytes, 0x00020000);
  uint4_t acc = {0, 0, 0, 0};
  for (uint32_t r = q; r < n_rows; r += IN_FLIGHT * nwaves) {
    uint4_t v[IN_FLIGHT];
#pragma unroll
    for (int i = 0; i < IN_FLIGHT; ++i) {
      const uint32_t row = r + i * nwaves;
      v[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, row < n_rows ? (row << 10) + lane * 16u : 0x80000000u, 0, 2);
    }
#pragma unroll
    for (int i = 0; i < IN_FLIGHT; ++i) acc ^= v[i];
  }
  // fold to one word per wave; the result only exists so that the loads cannot be dropped
  uint32_t x = acc.x ^ acc.y ^ acc.z ^ acc.w;
  for (int off = 32; off >= 1; off >>= 1) x ^= __shfl_xor(x, off, 64);
  if (lane == 0 && x == 0x9E3779B9u) sink[0] = x;
}

}  // namespace

hipError_t moqe_launch_stream_read(const void* src, size_t bytes, uint32_t* sink, int num_cus, hipStream_t stream) {
  hipLaunchKernelGGL(stream_read_kernel, dim3(3 * num_cus), dim3(256), 0, stream, (const uint4_t*)src, (uint32_t)bytes, sink);
  return hipGetLastError();
}
