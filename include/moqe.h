/*
 * moqe.h - C ABI of the MI355X (gfx950) MoQE hot path.
 *
 * MoQE (Mixture of Quantized Experts) keeps the expert weights of a top-1
 * routed MoE FFN as weight-only, per-output-channel, linearly quantized
 * int4 / int3 / int2 codes with fp16 scales and runs them against fp16
 * activations (paper: abstract; Sec. 3 "Experiments"; App. A "Quantization
 * algorithms"; App. B "MoE architecture"; App. C on fp16 channel scales).
 *
 * Conventions shared by every call
 *   - Every pointer is a DEVICE pointer unless its comment says "host".
 *   - The caller owns every buffer.  The library allocates nothing, never frees and
 *     (moqe_workspace_status apart) never synchronises: each call validates its
 *     arguments on the host, enqueues kernels on `stream` (a hipStream_t passed as
 *     void*, NULL = the null stream) and returns.
 *   - State the library keeps between calls: four process-wide tuning settings
 *     (moqe_set_launch_mode, moqe_set_decode_kernel, moqe_set_tiled_kernel,
 *     moqe_set_prefill_policy; plain atomics, results do not depend on them), per-device cached device properties,
 *     and the array behind moqe_moe_layer_static.  Everything else that survives a
 *     call lives in the caller's FFN / layer workspace (see the *_workspace_bytes
 *     functions below).
 *   - Device buffers must be 16-byte aligned (MOQE_ERR_ALIGN otherwise).
 *   - Argument errors are reported before anything is launched, so a failed
 *     call leaves all outputs untouched.  A failed launch returns
 *     MOQE_ERR_HIP; moqe_last_hip_error() gives the runtime's message.
 *   - T = 0 (no tokens) is valid and a no-op apart from seg_offsets = 0.
 *   - moqe_f16 is the IEEE binary16 bit pattern.
 *
 * Supported shapes: bits in {2,3,4,8} (Table 2's quantized rows) and bits = 16, the unquantized
 * baseline of the same table: moqe_quantize then stores fp16(w) (one rounding, to nearest
 * even) in place of codes, by the layout rule below with a field = the fp16 bit pattern, and
 * scales of 1; such layers run on the tiled kernel at every batch size (K a multiple of 128,
 * at least 256) and moqe_unpack does not apply.  N a multiple of 16; K a multiple of
 * 32 (fp16, int8, int4), 64 (int2), 128 (int3) and, when K/32 exceeds the chunk length
 * SC (1 step for fp16, 2 for int8, 4 for int4, 8 for int2/int3), K/32 a multiple of SC.  The FFN
 * additionally needs K = 32 * KS * R with KS in {2,4,8,16,24,32} and
 * R in {1,2,4} for both of its contractions (K = d and K = f).
 *
 * Packed layout of one [K,N] code matrix (K*N*bits/8 bytes, no padding; the
 * paper's Table 2 size column fixes the density, the arrangement is ours):
 *   column tile c = n / 16, j = n % 16; step s = k / 32, row group
 *   g = (k % 32) / 8, i = k % 8; slot l = 16 g + j; SC = min(SCmax, K/32);
 *   chunk p = s / SC, s' = s % SC, m = 8 s' + i.  Chunks are stored column
 *   tile major: chunk (c, p) starts at byte (c * K/(32 SC) + p) * 64 SC bits.
 *   Stored field value u = q + 2^(bits-1) (offset binary); log-scale codes
 *   (moqe_quantize_log) store u = sign * 2^(bits-1) + exponent code in the same fields.
 *   bits 2,4,8,16: the chunk is 64 slots of SC*bits bytes; inside a slot, 32/bits
 *     codes fill a little-endian 32-bit word: word = m / (32/bits),
 *     t = m % (32/bits), bit position = 16 (t & 1) + bits (t >> 1).
 *   bits 3: the chunk is a 2-bit plane (u & 3, arranged as for bits = 2)
 *     followed by a 1-bit plane (u >> 2): 64 slots of SC bytes, word = m / 32,
 *     t = m % 32, bit position = 16 (t & 1) + (t >> 1).
 *   A slot is what one lane of a 64-wide wavefront loads (16 bytes at full SC)
 *   and is already in the operand order of the 16x16x32 fp16 MFMA.
 *   A stack of E matrices is E such strings back to back.
 */
#ifndef MOQE_H
#define MOQE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef uint16_t moqe_f16;

typedef enum {
  MOQE_OK = 0,
  MOQE_ERR_NULL = 1,      /* a required pointer is NULL */
  MOQE_ERR_BITS = 2,      /* bits not in {2,3,4,8,16}, or not a width the codec has */
  MOQE_ERR_SHAPE = 3,     /* a dimension is negative, zero where it may not be, or unsupported */
  MOQE_ERR_ALIGN = 4,     /* a device pointer is not 16-byte aligned */
  MOQE_ERR_WORKSPACE = 5, /* workspace_bytes is smaller than the matching *_workspace_bytes() */
  MOQE_ERR_HIP = 6,       /* the HIP runtime refused a launch */
  MOQE_ERR_TIMEOUT = 7    /* moqe_workspace_status: a wait inside a single-launch step timed out */
} moqe_status;

/* Human-readable name of a status; static storage, never NULL. */
const char* moqe_status_string(int status);
/* Message of the last HIP error seen by this thread's calls; static storage. */
const char* moqe_last_hip_error(void);
/* ABI version, currently 2 (1: moqe_layer without its codec field). */
int moqe_version(void);

/* How moqe_expert_ffn and moqe_moe_layer issue their work (a process-wide setting, for
 * tuning and tests; results are identical in every mode):
 *   AUTO      whatever measured fastest on the decode workload (currently SEPARATE)
 *   SEPARATE  one launch per step of the path (router scores, router tables, FFN1, FFN2)
 *   FUSED     one launch for as much as the shapes allow: FFN1 + FFN2 when both contractions
 *             use the same wave slice length and h fits the chained buffers (T*f*2 <= 1 MiB),
 *             plus the router in moqe_moe_layer when T <= 64, E <= 256 and E % 8 == 0
 * Returns the previous mode, or -1 (and changes nothing) for an unknown mode. */
enum { MOQE_LAUNCH_AUTO = 0, MOQE_LAUNCH_SEPARATE = 1, MOQE_LAUNCH_FUSED = 2 };
int moqe_set_launch_mode(int mode);

/* Which dequantize-in-register kernel serves decode-sized batches (a process-wide setting, for
 * tests and comparisons; each kernel is deterministic, all run the same sums in the same order
 * and differ only in how the last step, gate times output, is rounded to fp16 - by at most one
 * unit in the last place of a few outputs in ten thousand): AUTO takes the kernel specialised for
 * decode-sized batches (at most 128 experts, 2- to 4-bit codes) where it applies and the general
 * one elsewhere; the specialised kernel works on (expert, 4 of its tokens) up to 32 tokens and on
 * (expert, 8 of its tokens) from 33 tokens on, where experts with more than four tokens are
 * common and their weights are then streamed once per eight (K = 1024 or 4096 only, else 4).  It
 * takes batches of up to 64 tokens, and in groups of 8 up to 128 (measured on the benchmark
 * layer at 128 tokens: 41.6 us per step at int4 and 36.1 at int2, against 51.4 and 42.7 through
 * the tiled kernels); from 65 tokens on only while moqe_set_prefill_policy's min_segment_tokens
 * is at least its default, i.e. no segments are asked onto the tiled kernel explicitly.
 * GENERAL always takes the general kernel; ROWS8 / ROWS4 are AUTO with 8 / 4 tokens at every
 * batch size (bit-identical results; ROWS4 ends at 64 tokens).  Launch mode FUSED uses the
 * general kernel.  Returns the previous setting, or -1 (nothing changed) for an unknown one. */
enum { MOQE_DECODE_AUTO = 0, MOQE_DECODE_GENERAL = 1, MOQE_DECODE_ROWS8 = 2, MOQE_DECODE_ROWS4 = 3 };
int moqe_set_decode_kernel(int which);

/* Which tiled matrix-core kernel serves the expert segments that take one (a process-wide
 * setting, for tests and comparisons; results are within the same tolerance either way).  The
 * resident kernel keeps a tile's token rows in LDS for the whole contraction: tiles of 64 tokens
 * where K <= 1024, of 16 tokens where K <= 4096 (K a multiple of 256 for int4 and of 512 for
 * int3 / int2; 2- to 4-bit codes, at most 1024 experts, T*N < 2^30); the other kernel stages K in
 * blocks for tiles of 64 tokens.  AUTO takes the resident kernel where K <= 1024 and, for longer
 * K, while the batch has at most 16 tokens per expert on average (T <= 16 E: most experts then
 * fill one tile of 16 at most; measured on the benchmark layer's FFN2, K = 4096: 22.3 against
 * 29.4 us at 256 tokens and int4, 17.4 against 27.3 at int2, 24.4 against 29.7 at 512 tokens,
 * 38 against 31 at 1024); STREAMED always stages K in blocks; RESIDENT takes the resident
 * kernel wherever it applies.  Returns the previous setting, or -1 (nothing changed) for an
 * unknown one. */
enum { MOQE_TILED_AUTO = 0, MOQE_TILED_STREAMED = 1, MOQE_TILED_RESIDENT = 2 };
int moqe_set_tiled_kernel(int which);

/* Path choice inside the expert FFN (process-wide, for tuning and tests; results are within
 * the same tolerance either way).  Batches with at least all_tiled_tokens_per_expert tokens per
 * expert on average (T >= that * E; eight times that for 8-bit codes, which have no tiled kernel
 * with resident token rows) and at least min_batch_tokens tokens do not launch the decode kernel:
 * every segment, however small, takes the tiled MFMA kernel (token rows in LDS, tiles of 64 or 16
 * tokens).  Below that, in a batch of at least min_batch_tokens tokens, expert segments with at
 * least min_segment_tokens tokens are computed by the tiled kernel and all other segments by the
 * dequantize-in-register decode kernel; smaller batches do not launch the tiled kernel at all.
 * Defaults below: everything tiled from 65 tokens (129 where the kernel for decode-sized batches
 * applies, see moqe_set_decode_kernel) and 2 tokens per expert on, the decode kernel alone below
 * that - on the benchmark layer (E = 32, d = 1024, f = 4096) the two kernels side by
 * side were never faster than the better of the two alone (65 to 384 tokens: 65-78 us per step
 * side by side against 47-57), and the tiled kernels alone are the faster from 65 tokens on at
 * every width (65 tokens: 46.9 / 52.0 / 40.0 us per step at int4 / int3 / int2 against 50.2 /
 * 52.2 / 42.8 with the decode kernel alone; 160 tokens: 51.3 / 55.4 / 42.1 against 65.0 / 66.3 /
 * 52.2).  A huge min_batch_tokens switches the tiled kernel off, a huge
 * all_tiled_tokens_per_expert the first rule.  The tiled kernel needs K >= 256 and a multiple of
 * 128 (int8, int4) or 256 (int2, int3), T*K*2 < 2^32 and T*N < 2^31; other layers use the decode
 * kernel throughout.  Launch mode FUSED uses the decode kernel for everything it chains.
 * Returns 0, or -1 (nothing changed) if a value < 1. */
#define MOQE_PREFILL_MIN_SEGMENT_DEFAULT 0x40000000
#define MOQE_PREFILL_MIN_BATCH_DEFAULT 65
#define MOQE_PREFILL_ALL_TILED_DEFAULT 2
int moqe_set_prefill_policy(int min_segment_tokens, int min_batch_tokens, int all_tiled_tokens_per_expert);

/* Which kernels one contraction of the expert FFN (moqe_expert_ffn1 / _ffn2, and moqe_expert_ffn /
 * moqe_moe_layer in the launch modes that run one contraction per launch) launches for experts of
 * `bits` bits (2, 3, 4, 8, 16), T tokens, E experts and [K, N] matrices, under the settings above as
 * they stand: the sum of MOQE_PATH_DECODE_SMALL or MOQE_PATH_DECODE (the dequantize-in-register
 * kernel for decode-sized batches, or the general one) and MOQE_PATH_TILED_RESIDENT or
 * MOQE_PATH_TILED_STAGED (the tiled matrix-core kernel with a tile's token rows resident in LDS, or
 * with K staged in blocks) - one of each pair at most, both where segments are shared out by size.
 * Host only, launches nothing; the decode-sized kernel needs a workgroup per (expert, token group)
 * resident at once, so the answer uses the current device's compute unit count (256 without a
 * device).  Returns -1 for sizes or widths the expert FFN does not take. */
enum { MOQE_PATH_DECODE_SMALL = 1, MOQE_PATH_DECODE = 2, MOQE_PATH_TILED_RESIDENT = 4, MOQE_PATH_TILED_STAGED = 8 };
int moqe_contraction_path(int bits, int64_t T, int64_t E, int64_t K, int64_t N);

/* Bytes of one packed [K,N] matrix = K*N*bits/8 (Table 2: exactly `bits` bits
 * per expert weight).  Returns 0 for an unsupported (bits, K, N). Host only. */
size_t moqe_packed_bytes(int bits, int64_t K, int64_t N);
/* MOQE_OK if (bits, K, N) can be packed, else the status a call would return. */
int moqe_check_matrix(int bits, int64_t K, int64_t N);
/* MOQE_OK if a layer with these dimensions can be run by moqe_expert_ffn. */
int moqe_check_layer(int bits, int64_t E, int64_t d, int64_t f);

/* Scratch sizes (host, pure).  Always > 0 so a caller may allocate blindly.
 * The route scratch needs no initialisation.
 * The FFN / layer scratch carries state from call to call: in FUSED launch mode the
 * router, FFN1 and FFN2 run as phases of one launch and hand their intermediate results
 * over through it (a launch counter, tagged router results, two alternating buffers for
 * the hidden activations in which zero means "not written yet").  Fill the WHOLE buffer
 * with zero once before its first use and always pass the same (pointer, size) pair;
 * after that any mix of calls and batch sizes may use it, one call at a time (calls that
 * may run concurrently need scratch buffers of their own).  The 32-bit word at byte 640
 * is an error flag: it becomes 1 and stays 1 if a wait inside a launch ever timed out
 * (buffer not zeroed, or the device shared so that the grid was not resident).  The calls
 * themselves cannot report that - they return before the kernels run - so every wait is
 * bounded, the grid always drains, the outputs of that and of every later FUSED call on
 * the buffer are invalid, and moqe_workspace_status tells: zero the buffer again after it
 * returned MOQE_ERR_TIMEOUT.  Only launch mode FUSED has such waits. */
size_t moqe_route_workspace_bytes(int64_t T, int64_t E);
size_t moqe_ffn_workspace_bytes(int64_t T, int64_t E, int64_t d, int64_t f);
size_t moqe_layer_workspace_bytes(int64_t T, int64_t E, int64_t d, int64_t f); /* for moqe_moe_layer */
/* Waits for the work queued on `stream`, then reads the workspace's error flag (a 4-byte
 * copy to the host): MOQE_OK, or MOQE_ERR_TIMEOUT if a wait of a FUSED launch that used this
 * FFN / layer workspace has timed out since the buffer was last zeroed.  The one call of
 * the library that synchronises; meant for after a batch of steps, not for the hot loop.
 * workspace NULL: MOQE_ERR_NULL; smaller than 1024 bytes: MOQE_ERR_WORKSPACE. */
moqe_status moqe_workspace_status(const void* workspace, size_t workspace_bytes, void* stream);

/* Measurement aid: a launch that only reads `bytes` bytes (a multiple of 1024) from src with
 * 16-byte streaming loads, in the launch shape of the decode kernels, and writes at most four
 * bytes to sink.  Its duration on buffers that are not cache resident is the ceiling this
 * machine sets for a kernel that must read that many bytes; bench.py reports the expert
 * kernels' rate against it.  MOQE_ERR_SHAPE if bytes is 0, not a multiple of 1024, or 2 GiB
 * and more. */
moqe_status moqe_stream_read(const void* src, size_t bytes, void* sink, void* stream);

/*
 * Offline round-to-nearest quantization and bit packing of a stack of E
 * matrices (App. A "Linear quantization with absolute maximum"; scales in
 * half precision per App. C).
 *   w          [E,K,N] fp32, N contiguous.  A channel is a column (one of the
 *              N outputs of y = x A); the maximum runs over the K rows.
 *   scales_out [E,N]: s = 2 max|A_:,n| / (2^bits - 1) computed in fp64 and
 *              rounded UP to fp16 (so that |a - q s| <= s/2 for every entry);
 *              an all-zero channel gets s = 0 and codes 0.
 *   codes_out  E * moqe_packed_bytes(bits,K,N) bytes, layout above, with
 *              q = clamp(rint(a / s), -2^(bits-1), 2^(bits-1)-1), the division
 *              and the ties-to-even rounding done in fp64 on the stored scale.
 * Non-finite weights or a scale beyond fp16's range are undefined input.
 */
moqe_status moqe_quantize(const float* w, int64_t E, int64_t K, int64_t N, int bits,
                          void* codes_out, moqe_f16* scales_out, void* stream);
/* The same with the other choice of s that App. A names ("per the whole tensor"; the
 * matrix-wise scale App. C compares the channel-wise one against): one
 * s = 2 max|A| / (2^bits - 1) per [K,N] matrix, written to all N entries of its row of
 * scales_out, so that the expert FFN calls take such a layer unchanged.  Arguments, layouts
 * and errors as for moqe_quantize; bits = 16 has no scale to choose and is the same call. */
moqe_status moqe_quantize_tensor_scale(const float* w, int64_t E, int64_t K, int64_t N, int bits,
                                       void* codes_out, moqe_f16* scales_out, void* stream);

/* Codec of a layer's expert weights: the linear absmax codes of moqe_quantize, or the
 * log-scale codes of moqe_quantize_log. */
enum { MOQE_CODEC_LINEAR = 0, MOQE_CODEC_LOG = 1 };

/* The codec App. A describes beside the linear one and the paper sets aside ("Log-scale
 * quantization"): one sign bit and a (bits-1)-bit exponent per weight,
 *   P = sign(A),  T = clip(|A| / s, 2^(1 - 2^(bits-1)), 1),  Q = ceil(log2(2T/3)),  A' = P s 2^Q
 * (the printed clip bounds, a lower bound of 1 above an upper bound below 1, are read as that
 * interval: its ends give exactly the 2^(bits-1) exponents the field can count).  s is the
 * absolute maximum of the output channel, the first of the two choices the paper names, stored
 * in fp16 rounded toward +inf.  Q is decided as the smallest integer with |A| <= 1.5 * 2^Q * s,
 * an exact comparison in fp64.  Stored field: u = sign_bit * 2^(bits-1) + (Q + 2^(bits-1) - 1),
 * in the same packed layout as the linear codes (moqe_unpack returns u - 2^(bits-1)).  A zero
 * weight takes the smallest magnitude with a plus sign (the format has no zero); a channel of
 * zeros has s = 0.  bits must be 2, 3 or 4 (MOQE_ERR_BITS otherwise); other arguments, layouts
 * and errors as for moqe_quantize.  The expert FFN calls take a layer of such codes
 * (moqe_layer.codec = MOQE_CODEC_LOG; the weights unpack to +-2^Q by exponent insert in both
 * FFN kernels, the scale multiplies the finished sum as for linear codes).  A layer's codec
 * field set to MOQE_CODEC_LOG with bits other than 2, 3 or 4, or to any other value, is
 * MOQE_ERR_BITS. */
moqe_status moqe_quantize_log(const float* w, int64_t E, int64_t K, int64_t N, int bits,
                              void* codes_out, moqe_f16* scales_out, void* stream);
/* Dequantization of log-scale codes, A' = P s 2^Q, written as fp32 [E,K,N] (every value is
 * exact): the exponent Q is added to the exponent field of s and the sign bit set, no multiply.
 * w_out must be 16-byte aligned. */
moqe_status moqe_dequantize_log(const void* codes, const moqe_f16* scales, int64_t E, int64_t K, int64_t N,
                                int bits, float* w_out, void* stream);

/* Inverse of the packing, for tests and tools: q_out [E,K,N] int8 codes. */
moqe_status moqe_unpack(const void* codes, int64_t E, int64_t K, int64_t N, int bits,
                        int8_t* q_out, void* stream);

/*
 * Top-1 learned gating and dispatch bookkeeping (App. B "MoE architecture":
 * top-1 gating as in Switch; no capacity limit, jitter or dropout at inference).
 *   x [T,d] fp16, w_gate [d,E] fp16 (E contiguous); logits = x w_gate in fp32.
 *   expert_idx [T]  lowest index attaining the row maximum
 *   gate       [T]  fp32 softmax probability of that expert
 *   seg_offsets[E+1] exclusive prefix sum of the per-expert token counts,
 *                   seg_offsets[E] = T
 *   perm       [T]  sorted position -> token id; tokens of one expert keep
 *                   ascending order (stable), so the result is unique
 * 1 <= E <= 1024, d >= 1 and a multiple of 8, T >= 0.
 */
moqe_status moqe_route(const moqe_f16* x, const moqe_f16* w_gate, int64_t T, int64_t d, int64_t E,
                       int32_t* expert_idx, float* gate, int32_t* seg_offsets, int32_t* perm,
                       void* workspace, size_t workspace_bytes, void* stream);

/* Same, starting from given fp32 logits [T,E] (E contiguous). */
moqe_status moqe_route_logits(const float* logits, int64_t T, int64_t E,
                              int32_t* expert_idx, float* gate, int32_t* seg_offsets, int32_t* perm,
                              void* workspace, size_t workspace_bytes, void* stream);

/* One MoE layer's quantized experts.  The struct itself lives in HOST memory;
 * its pointers are device pointers. codesX: E packed matrices, scalesX and
 * biasX: [E, out] fp16.  Matrix 1 is [d,f] (K = d), matrix 2 is [f,d] (K = f). */
typedef struct {
  int bits;
  int64_t E, d, f;
  const void* codes1;
  const moqe_f16* scales1;
  const moqe_f16* bias1;
  const void* codes2;
  const moqe_f16* scales2;
  const moqe_f16* bias2;
  int codec; /* MOQE_CODEC_LINEAR (0), or MOQE_CODEC_LOG (bits 2, 3 or 4): codes from moqe_quantize_log */
} moqe_layer;

/*
 * Expert FFN with dequantization on the fly (Sec. 2.1: the two-layer
 * Transformer FFN; App. A: A' = Q s) and the gate-weighted combine:
 *   for token t with e = expert_idx[t]:
 *     h = max(0, x_t (Q1_e s1_e) + b1_e)        (fp32 accumulate, h kept in fp16)
 *     y_t = gate[t] * (h (Q2_e s2_e) + b2_e)    (+ residual_t if given), stored fp16
 * expert_idx, gate, seg_offsets, perm are as moqe_route produces them (any
 * consistent routing is accepted; seg_offsets and perm alone drive the
 * dispatch).  residual may be NULL; y may alias residual; y must not alias x
 * unless x == residual.
 */
moqe_status moqe_expert_ffn(const moqe_layer* layer /* host */, const moqe_f16* x, int64_t T,
                            const int32_t* expert_idx, const float* gate,
                            const int32_t* seg_offsets, const int32_t* perm,
                            const moqe_f16* residual, moqe_f16* y,
                            void* workspace, size_t workspace_bytes, void* stream);

/*
 * One whole MoE layer step: moqe_route followed by moqe_expert_ffn (App. B gating,
 * Sec. 2.1 FFN) with the same outputs as the two calls; how many launches it takes is
 * governed by moqe_set_launch_mode.  expert_idx, gate, seg_offsets, perm are outputs.
 * workspace: moqe_layer_workspace_bytes(T, E, d, f), head zeroed as described above.
 */
moqe_status moqe_moe_layer(const moqe_layer* layer /* host */, const moqe_f16* w_gate, const moqe_f16* x,
                           int64_t T, int32_t* expert_idx, float* gate, int32_t* seg_offsets, int32_t* perm,
                           const moqe_f16* residual, moqe_f16* y,
                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * moqe_moe_layer for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the same step with the same outputs,
 * its scratch taken from an array inside the library instead of a workspace argument.  The
 * array holds MOQE_STATIC_SCRATCH_BYTES on every GPU the library runs on, from the first call
 * on that GPU until the process ends; a step whose moqe_layer_workspace_bytes(T, E, d, f)
 * exceeds that is refused with MOQE_ERR_WORKSPACE before anything is launched (d_ff 4096:
 * up to 255 tokens).  The call allocates and frees nothing; its first call on a device looks
 * up the array's address (make that call outside a graph capture).  The array starts zeroed and
 * carries state from call to call exactly as a caller's workspace does; every call on a GPU
 * shares that GPU's array, so calls that may overlap on one GPU (two streams, two threads)
 * race: issue them one after the other, or use moqe_moe_layer with a buffer per stream.
 * Other arguments and errors as for moqe_moe_layer.
 */
#define MOQE_STATIC_SCRATCH_BYTES (4u << 20)
moqe_status moqe_moe_layer_static(const moqe_layer* layer /* host */, const moqe_f16* w_gate, const moqe_f16* x,
                                  int64_t T, int32_t* expert_idx, float* gate, int32_t* seg_offsets,
                                  int32_t* perm, const moqe_f16* residual, moqe_f16* y, void* stream);

/*
 * The two contractions of moqe_expert_ffn as separate calls, for callers that
 * time them or put other work between them.  h is fp16 [T,f] with rows in
 * sorted-token order (row i belongs to token perm[i]); moqe_expert_ffn keeps it
 * in its workspace.
 *   ffn1: h = max(0, x (Q1 s1) + b1)
 *   ffn2: y_t = gate[t] * (h (Q2 s2) + b2) (+ residual_t)
 */
moqe_status moqe_expert_ffn1(const moqe_layer* layer /* host */, const moqe_f16* x, int64_t T,
                             const int32_t* seg_offsets, const int32_t* perm, moqe_f16* h, void* stream);
moqe_status moqe_expert_ffn2(const moqe_layer* layer /* host */, const moqe_f16* h, int64_t T, const float* gate,
                             const int32_t* seg_offsets, const int32_t* perm, const moqe_f16* residual,
                             moqe_f16* y, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MOQE_H */
