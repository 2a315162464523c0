// Internal launchers behind the C ABI (host side).  Shapes are validated by the
// callers in moqe_api.hip before any of these is reached.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "moqe_dev.h"

hipError_t moqe_launch_quantize(const float* w, int64_t E, const PackGeom& g, void* codes, uint16_t* scales,
                                hipStream_t stream);
hipError_t moqe_launch_unpack(const void* codes, int64_t E, const PackGeom& g, int8_t* q_out, hipStream_t stream);

size_t moqe_route_ws_bytes(int64_t T, int64_t E);
// logits != NULL: start from given logits (x, wg, d unused).
hipError_t moqe_launch_route(const uint16_t* x, const uint16_t* wg, const float* logits, int T, int d, int E,
                             int* expert_idx, float* gate, int* seg_offsets, int* perm, void* ws, hipStream_t stream);

// One contraction of the expert FFN over the routed segments.
struct FfnArgs {
  // weights of this contraction: K inputs -> N outputs, E experts
  const uint32_t* codes;
  const uint16_t* scales;  // [E,N] fp16
  const uint16_t* bias;    // [E,N] fp16
  int bits, E, K, N;
  int ksteps;  // 32-row steps one wave keeps in registers
  int ksplit;  // waves sharing one output tile along K (K = 32 * ksteps * ksplit)
  // routing
  const int* seg_offsets;  // [E+1]
  const int* perm;         // [T] sorted position -> token
  const float* gate;       // [T] by token
  int T;
  // operands
  const uint16_t* a;  // mode 0: x [T,K] by token; mode 1: h [T,K] by sorted position
  uint16_t* h_out;    // mode 0: relu(a W + b) -> [T,N] by sorted position
  uint16_t* y_out;    // mode 1: gate * (a W + b) (+ residual) -> [T,N] by token
  const uint16_t* residual;  // mode 1, may be NULL
  int mode;
  // expert segments with min_tokens <= n < max_tokens are handled, the rest skipped
  int min_tokens, max_tokens;
  // debug builds (-DMOQE_PHASE_TRACE): 8 wall-clock stamps per workgroup, else unused
  long long* trace;
};

// Register-resident dequantize + 16-token MFMA path (few tokens per expert).
hipError_t moqe_launch_ffn_decode(const FfnArgs& a, int num_cus, hipStream_t stream);
// Picks (ksteps, ksplit) for a contraction length K; false if unsupported.
bool moqe_pick_ksplit(int bits, int64_t K, int* ksteps, int* ksplit);
