// Internal launchers behind the C ABI (host side).  Shapes are validated by the
// callers in moqe_api.hip before any of these is reached.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "moqe.h"
#include "moqe_dev.h"

// tensor_scale: one scale per matrix (the largest channel scale) instead of one per channel
// codec: MOQE_CODEC_LINEAR or MOQE_CODEC_LOG of moqe.h
hipError_t moqe_launch_quantize(const float* w, int64_t E, const PackGeom& g, void* codes, uint16_t* scales,
                                bool tensor_scale, int codec, hipStream_t stream);
hipError_t moqe_launch_dequantize_log(const void* codes, const uint16_t* scales, int64_t E, const PackGeom& g,
                                      float* w_out, hipStream_t stream);
hipError_t moqe_launch_unpack(const void* codes, int64_t E, const PackGeom& g, int8_t* q_out, hipStream_t stream);

// Plain read of `bytes` (a multiple of 1024) from src; sink receives at most one word.
hipError_t moqe_launch_stream_read(const void* src, size_t bytes, uint32_t* sink, int num_cus, hipStream_t stream);

size_t moqe_route_ws_bytes(int64_t T, int64_t E);
// logits != NULL: start from given logits (x, wg, d unused).
hipError_t moqe_launch_route(const uint16_t* x, const uint16_t* wg, const float* logits, int T, int d, int E,
                             int* expert_idx, float* gate, int* seg_offsets, int* perm, void* ws, hipStream_t stream);

// One contraction of the expert FFN over the routed segments.
struct PhaseArgs {
  // weights of this contraction: K inputs -> N outputs
  const uint32_t* codes;
  const uint16_t* scales;  // [E,N] fp16
  const uint16_t* bias;    // [E,N] fp16
  int K, N;
  int ksplit;  // waves sharing one output tile along K (K = 32 * ksteps * ksplit)
  int mode;    // 0: rows of `a` by token through perm, out = relu(.) by sorted position
               // 1: rows of `a` by sorted position, out = gate * (.) (+ residual) by token
  const uint16_t* a;
  uint16_t* out;
  const uint16_t* residual;  // mode 1, may be NULL
};

// One launch of the decode-step kernel: any of router / FFN1 / FFN2, in that order.
struct DecodeArgs {
  int bits, ksteps;  // 32-row steps one wave keeps in registers (same for both contractions)
  int E, T;
  int phase_mask;  // bit 0: router, bit 1: FFN1 (ph[0]), bit 2: FFN2 (ph[1])
  // router inputs (bit 0): x [T,d_route], w_gate [d_route,E]
  const uint16_t* x;
  const uint16_t* w_gate;
  int d_route;
  // routing tables: written by the router phase, read otherwise
  int* expert_idx;   // [T]
  float* gate;       // [T] by token (may be NULL when only FFN1 runs)
  int* seg_offsets;  // [E+1]
  int* perm;         // [T] sorted position -> token
  PhaseArgs ph[2];
  // expert segments with min_tokens <= n < max_tokens are handled, the rest skipped
  int min_tokens, max_tokens;
  // Multi-phase launches.  sync: 1024 bytes, zero before the first launch: launch epoch,
  // start counter, error flag (one word per 128-byte line).  route_entries: two 64-bit words
  // per token for the router phase.  h_base: two buffers of h_stride fp16 elements each,
  // zero before the first launch; FFN1 fills one (ph[0].out / ph[1].a are then ignored).
  unsigned* sync;
  unsigned long long* route_entries;
  uint16_t* h_base;
  size_t h_stride;
  unsigned h_bytes;  // bytes of h this launch writes (T * f * 2)
};

// One contraction over the expert segments with at least min_tokens tokens: tiled MFMA
// contraction with the token rows staged in LDS (many tokens per expert).
struct PrefillArgs {
  int bits, E, T;
  int K, N;
  int mode;  // as in PhaseArgs
  int min_tokens;
  int n_cblocks;  // set by the launcher
  const uint32_t* codes;
  const uint16_t* scales;
  const uint16_t* bias;
  const uint16_t* a;
  uint16_t* out;
  const uint16_t* residual;
  const int* seg_offsets;
  const int* perm;
  const float* gate;
};
bool moqe_prefill_supported(int bits, int64_t K, int64_t N);
hipError_t moqe_launch_prefill(const PrefillArgs& a, int num_cus, hipStream_t stream);
// The same contraction with a tile's token rows resident in LDS for the whole K (K <= 1024,
// 2- to 4-bit codes, T N < 2^30).
bool moqe_resident_supported(int bits, int64_t K, int64_t N);
hipError_t moqe_launch_resident(const PrefillArgs& a, int num_cus, hipStream_t stream);

// One contraction of a decode-sized batch (T <= 64, E <= 128, 2- to 4-bit codes): the lean
// dequantize-in-register kernel, one pair (expert, 4 tokens) per workgroup.
struct SmallDecodeArgs {
  int bits, ksteps, ksplit;  // K = 32 * ksteps * ksplit
  int rows;                  // token rows of a pair: 4, or 8 (slices of 32 steps only)
  int mode;                  // as in PhaseArgs
  int E, T, N;
  int min_tokens, max_tokens;  // expert segments with min_tokens <= n < max_tokens are handled
  const uint32_t* codes;
  const uint16_t* scales;
  const uint16_t* bias;
  const uint16_t* a;
  uint16_t* out;
  const uint16_t* residual;  // mode 1, may be NULL
  const float* gate;         // mode 1
  const int* seg_offsets;
  const int* perm;
};
// (bits as the kernels are instantiated: 2, 3, 4 or MOQE_LOG2..4; grid_min = workgroups the
// launch will have at least: one per CU)
bool moqe_decode_small_supported(int bits, int64_t T, int64_t E, int64_t K, int64_t N, int grid_min, int rows);
hipError_t moqe_launch_decode_small(const SmallDecodeArgs& a, int num_cus, hipStream_t stream);

// Dequantize-in-register path for few tokens per expert (tiles of 4 tokens), any batch size.
hipError_t moqe_launch_decode(const DecodeArgs& a, int num_cus, hipStream_t stream);
// Picks (ksteps, ksplit) for a contraction length K; false if unsupported.
bool moqe_pick_ksplit(int bits, int64_t K, int* ksteps, int* ksplit);
// Whether the decode kernel's own router phase can serve these sizes.
bool moqe_decode_can_route(int64_t T, int64_t d, int64_t E);
