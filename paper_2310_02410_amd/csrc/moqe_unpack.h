// Register-level unpacking of the packed 2/3/4-bit codes into fp16 MFMA fragments
// (device only).  One lane's slot of the packed layout is already in the operand order
// of v_mfma_f32_16x16x32_f16: lane (g, j) supplies, per 32-row step, the 8 codes
// k = 32 s + 8 g + 0..7 of output channel j, two per 32-bit register (k even in the low
// half).  A code field is turned into an fp16 number by OR-ing an exponent pattern onto
// the masked bits: with exponent 2^e the field bits sit in the mantissa and the value
// reads base + u (or base + 4 u' for the int3 high plane).  Fields that leave their
// base in the value are corrected after the K-sum: sum_k a_k (base_k + u_k) minus
// sum_k a_k (base_k + zero point), the second sum coming from bias_frag().
#pragma once

#include "moqe_dev.h"

typedef short short2_t __attribute__((ext_vector_type(2)));

__device__ inline half8_t frag_from_words(uint32_t r0, uint32_t r1, uint32_t r2, uint32_t r3) {
  uint4_t v = {r0, r1, r2, r3};
  return __builtin_bit_cast(half8_t, v);
}

__device__ inline uint32_t pk_sub(uint32_t v, float c) {
  half2_t h = __builtin_bit_cast(half2_t, v);
  half2_t k = {(half_t)c, (half_t)c};
  h = h - k;
  return __builtin_bit_cast(uint32_t, h);
}

__device__ inline half8_t const_frag(float c0, float c1, float c2, float c3) {
  half8_t v = {(half_t)c0, (half_t)c0, (half_t)c1, (half_t)c1, (half_t)c2, (half_t)c2, (half_t)c3, (half_t)c3};
  return v;
}

// Masks (scalar registers) and fp16 exponent patterns (vector registers; base << 16 | base
// with a zero mantissa) of the unpack sequences, created once per kernel.
template <int BITS>
struct UnpackConsts {
  uint32_t m_000f, m_00f0;                  // int4 nibble masks
  uint32_t m_00ff;                          // int8 byte mask
  uint32_t m_0030, m_00c0, m_0300;          // 2-bit field masks at bits 4, 6, 8
  uint32_t m_0040, m_0080, m_0100, m_0200;  // single-bit masks at bits 6..9 (int3 high plane)
  uint32_t x1024, x64, x32, x16, x8, x4;    // exponent patterns
  uint32_t l_e3, l_one;                     // log-scale codes: kept bits, exponent offset
  __device__ inline void init() {
    if (BITS == 16) return;  // fp16 weights need no unpacking
    if (BITS == MOQE_LOG2 || BITS == MOQE_LOG3) {
      l_e3 = opaque_sgpr(0x84008400u);  // (2-bit codes) sign and the exponent bit of an fp16 word
      l_one = opaque_vgpr(BITS == MOQE_LOG2 ? 0x38003800u : 0x30003000u);
      return;
    }
    if (BITS == MOQE_LOG4) {
      l_e3 = opaque_sgpr(0x9C009C00u);  // sign and the three exponent bits of an fp16 word
      l_one = opaque_vgpr(0x20002000u);
      return;
    }
    if (BITS == 8) {
      m_00ff = opaque_sgpr(0x00FF00FFu);
      x1024 = opaque_vgpr(0x64006400u);
    } else if (BITS == 4) {
      m_000f = opaque_sgpr(0x000F000Fu);
      m_00f0 = opaque_sgpr(0x00F000F0u);
      x1024 = opaque_vgpr(0x64006400u);
      x64 = opaque_vgpr(0x54005400u);
    } else {
      m_0030 = opaque_sgpr(0x00300030u);
      m_00c0 = opaque_sgpr(0x00C000C0u);
      m_0300 = opaque_sgpr(0x03000300u);
      x64 = opaque_vgpr(0x54005400u);
      x16 = opaque_vgpr(0x4C004C00u);
      x4 = opaque_vgpr(0x44004400u);
    }
    if (BITS == 3) {
      m_0040 = opaque_sgpr(0x00400040u);
      m_0080 = opaque_sgpr(0x00800080u);
      m_0100 = opaque_sgpr(0x01000100u);
      m_0200 = opaque_sgpr(0x02000200u);
      x32 = opaque_vgpr(0x50005000u);
      x8 = opaque_vgpr(0x48004800u);
    }
  }
};

// ---- int4: one word per step; word bit position of code i (i = k % 8): 16 (i & 1) + 4 (i >> 1).
// Nibbles at bits 0-3 get base 1024 and are made exact with a packed subtract (a bias that
// large would cost accuracy if carried through the K-sum); nibbles at bits 4-7 keep base 64
// and their 64 + 8 is removed after the K-sum like the int2 fields.
template <class C>
__device__ inline half8_t unpack4(uint32_t d, const C& c) {
  uint32_t d8 = d >> 8;
  uint32_t r0 = pk_sub((d & c.m_000f) | c.x1024, 1032.0f);
  uint32_t r1 = (d & c.m_00f0) | c.x64;
  uint32_t r2 = pk_sub((d8 & c.m_000f) | c.x1024, 1032.0f);
  uint32_t r3 = (d8 & c.m_00f0) | c.x64;
  return frag_from_words(r0, r1, r2, r3);
}

// ---- 4-bit log-scale codes (App. A: A' = P s 2^Q): same nibble positions as int4; a nibble
// holds the exponent e = Q + 7 in its low three bits and the sign in its top bit.  The fp16
// number +-2^Q has exponent field e + 8 and no mantissa.  The nibble is shifted to the top of
// its 16-bit half; an arithmetic shift right by two (per half) then leaves the sign in bit 15
// and the exponent in bits 10..12 (bits 13 and 14 hold copies of the sign, masked away), and
// 0x2000 adds the 8.  No multiply, and nothing to correct after the K-sum (the value is exact;
// the format has no zero point).  A 32-bit shift may be used to move the nibbles up: what it
// carries from the low half into the high one lands below bit 26 and is masked away.
template <class C>
__device__ inline uint32_t log4_top_nibble(uint32_t v, const C& c) {
  short2_t h = __builtin_bit_cast(short2_t, v);
  h = h >> 2;
  return (__builtin_bit_cast(uint32_t, h) & c.l_e3) | c.l_one;
}
template <class C>
__device__ inline half8_t unpack4_log(uint32_t d, const C& c) {
  return frag_from_words(log4_top_nibble(d << 12, c), log4_top_nibble(d << 8, c), log4_top_nibble(d << 4, c),
                         log4_top_nibble(d, c));
}

// ---- 2-bit and 3-bit log-scale codes.  The exponent field sits where the linear codes keep
// their 2-bit field (register i of a step's fragment: bit 2 i of each half in an even step, bit
// 8 + 2 i in an odd one): one exponent bit for 2-bit codes, whose sign is the field's upper bit,
// two for 3-bit codes, whose sign is the bit of the 1-bit plane (bit 4 ss + i of each half for
// step ss of four).  Exponent bits go to bit 10 (and 11), the sign to bit 15, and l_one holds
// the exponent offset: 2^Q = 2^(e - 1) has exponent field 14 + e, 2^(e - 3) has 12 + e.
template <int POS, int NBITS>
__device__ inline uint32_t log_field_to_exponent(uint32_t d) {
  constexpr uint32_t m = ((1u << NBITS) - 1u) << POS;
  constexpr uint32_t mask = m | (m << 16);
  if constexpr (POS <= 10) return (d & mask) << (10 - POS);
  else return (d & mask) >> (POS - 10);
}
template <int POS>
__device__ inline uint32_t log_bit_to_sign(uint32_t d) {
  constexpr uint32_t mask = (1u << POS) | (1u << (POS + 16));
  return (d & mask) << (15 - POS);
}
// (2-bit codes: the field [sign, exponent bit] is shifted to the top of its half; an arithmetic
// shift right by four then leaves the sign in bit 15 and the exponent bit in bit 10, with
// copies of the sign in between that are masked away - as for the 4-bit codes)
template <int POS, class C>
__device__ inline uint32_t log2_field(uint32_t d, const C& c) {
  short2_t h = __builtin_bit_cast(short2_t, POS == 14 ? d : d << (14 - POS));
  h = h >> 4;
  return (__builtin_bit_cast(uint32_t, h) & c.l_e3) | c.l_one;
}
template <int PARITY, class C>
__device__ inline half8_t unpack2_log(uint32_t d, const C& c) {
  constexpr int P = 8 * PARITY;
  return frag_from_words(log2_field<P + 0>(d, c), log2_field<P + 2>(d, c), log2_field<P + 4>(d, c),
                         log2_field<P + 6>(d, c));
}
template <int SS, class C>
__device__ inline half8_t unpack3_log(uint32_t dl, uint32_t dh, const C& c) {
  constexpr int P = 8 * (SS & 1), H = 4 * SS;
  return frag_from_words(log_field_to_exponent<P + 0, 2>(dl) | log_bit_to_sign<H + 0>(dh) | c.l_one,
                         log_field_to_exponent<P + 2, 2>(dl) | log_bit_to_sign<H + 1>(dh) | c.l_one,
                         log_field_to_exponent<P + 4, 2>(dl) | log_bit_to_sign<H + 2>(dh) | c.l_one,
                         log_field_to_exponent<P + 6, 2>(dl) | log_bit_to_sign<H + 3>(dh) | c.l_one);
}

// ---- int8: two words per step; word bit position of code i: 16 (i & 1) + 8 ((i >> 1) & 1), word
// i >> 2.  Every byte gets base 1024: value = 1024 + u, u = q + 128; the 1152 is removed after
// the K-sum (it is 9 to 1000 times the code, like the bases of the 2-bit fields).
template <class C>
__device__ inline half8_t unpack8(uint32_t d0, uint32_t d1, const C& c) {
  uint32_t r0 = (d0 & c.m_00ff) | c.x1024;
  uint32_t r1 = ((d0 >> 8) & c.m_00ff) | c.x1024;
  uint32_t r2 = (d1 & c.m_00ff) | c.x1024;
  uint32_t r3 = ((d1 >> 8) & c.m_00ff) | c.x1024;
  return frag_from_words(r0, r1, r2, r3);
}

// ---- int2: one word per two steps.  Fields are left with their exponent bias
// (value = base + u); the bias and the zero point are removed after the K-sum
// through bias_frag(): sum_k a_k (base_k + u_k) - sum_k a_k (base_k + 2).
// even step: fields at bits 0,2,4,6 of each half; odd step: bits 8,10,12,14.
template <int PARITY, class C>
__device__ inline half8_t unpack2(uint32_t d, const C& c) {
  if (PARITY == 0) {
    uint32_t dl = d << 4;
    uint32_t r0 = (dl & c.m_0030) | c.x64;  // bits 0-1 -> 4-5
    uint32_t r1 = (dl & c.m_00c0) | c.x16;  // bits 2-3 -> 6-7
    uint32_t r2 = (d & c.m_0030) | c.x64;   // bits 4-5
    uint32_t r3 = (d & c.m_00c0) | c.x16;   // bits 6-7
    return frag_from_words(r0, r1, r2, r3);
  } else {
    uint32_t dr = d >> 6;
    uint32_t r0 = (d & c.m_0300) | c.x4;    // bits 8-9
    uint32_t r1 = (dr & c.m_0030) | c.x64;  // bits 10-11 -> 4-5
    uint32_t r2 = (dr & c.m_00c0) | c.x16;  // bits 12-13 -> 6-7
    uint32_t r3 = (dr & c.m_0300) | c.x4;   // bits 14-15 -> 8-9
    return frag_from_words(r0, r1, r2, r3);
  }
}

// ---- int3 high plane: one word per four steps, one bit per code, worth 4.
// step ss (0..3) owns bits 4 ss .. 4 ss + 3 of each half; they are moved to
// mantissa bits 6..9 where, with bases 64, 32, 16, 8, a set bit adds exactly 4.
template <int SS, class C>
__device__ inline half8_t unpack1x4(uint32_t d, const C& c) {
  uint32_t v = SS == 0 ? (d << 6) : SS == 1 ? (d << 2) : SS == 2 ? (d >> 2) : (d >> 6);
  uint32_t r0 = (v & c.m_0040) | c.x64;
  uint32_t r1 = (v & c.m_0080) | c.x32;
  uint32_t r2 = (v & c.m_0100) | c.x16;
  uint32_t r3 = (v & c.m_0200) | c.x8;
  return frag_from_words(r0, r1, r2, r3);
}

// ---- exact variants: every field is brought down to the signed code q = u - 2^(b-1) with a
// packed subtract, at one more VALU operation per register.  Used where the unpack is
// amortized over several token tiles and K is long: leaving the offsets in the K-sum costs
// accuracy when the activations are all positive (h after ReLU), because the offset term then
// grows like K while the signal grows like sqrt(K).
__device__ inline uint32_t pk_add(uint32_t a, uint32_t b) {
  half2_t x = __builtin_bit_cast(half2_t, a), y = __builtin_bit_cast(half2_t, b);
  x = x + y;
  return __builtin_bit_cast(uint32_t, x);
}

template <class C>
__device__ inline half8_t unpack4_exact(uint32_t d, const C& c) {
  uint32_t d8 = d >> 8;
  uint32_t r0 = pk_sub((d & c.m_000f) | c.x1024, 1032.0f);
  uint32_t r1 = pk_sub((d & c.m_00f0) | c.x64, 72.0f);
  uint32_t r2 = pk_sub((d8 & c.m_000f) | c.x1024, 1032.0f);
  uint32_t r3 = pk_sub((d8 & c.m_00f0) | c.x64, 72.0f);
  return frag_from_words(r0, r1, r2, r3);
}

template <class C>
__device__ inline half8_t unpack8_exact(uint32_t d0, uint32_t d1, const C& c) {
  uint32_t r0 = pk_sub((d0 & c.m_00ff) | c.x1024, 1152.0f);
  uint32_t r1 = pk_sub(((d0 >> 8) & c.m_00ff) | c.x1024, 1152.0f);
  uint32_t r2 = pk_sub((d1 & c.m_00ff) | c.x1024, 1152.0f);
  uint32_t r3 = pk_sub(((d1 >> 8) & c.m_00ff) | c.x1024, 1152.0f);
  return frag_from_words(r0, r1, r2, r3);
}

template <int PARITY, class C>
__device__ inline half8_t unpack2_exact(uint32_t d, const C& c) {
  if (PARITY == 0) {
    uint32_t dl = d << 4;
    uint32_t r0 = pk_sub((dl & c.m_0030) | c.x64, 66.0f);
    uint32_t r1 = pk_sub((dl & c.m_00c0) | c.x16, 18.0f);
    uint32_t r2 = pk_sub((d & c.m_0030) | c.x64, 66.0f);
    uint32_t r3 = pk_sub((d & c.m_00c0) | c.x16, 18.0f);
    return frag_from_words(r0, r1, r2, r3);
  } else {
    uint32_t dr = d >> 6;
    uint32_t r0 = pk_sub((d & c.m_0300) | c.x4, 6.0f);
    uint32_t r1 = pk_sub((dr & c.m_0030) | c.x64, 66.0f);
    uint32_t r2 = pk_sub((dr & c.m_00c0) | c.x16, 18.0f);
    uint32_t r3 = pk_sub((dr & c.m_0300) | c.x4, 6.0f);
    return frag_from_words(r0, r1, r2, r3);
  }
}

// int3, step SS (0..3) of a group of four: low plane word dl (two steps per word, the step's
// parity is SS & 1), high plane word dh (four steps per word).  The two planes are added while
// they still carry their exponent offsets (the sums stay below 256, where fp16 still holds
// every integer), then one subtract removes both offsets and the zero point 4.
template <int SS, class C>
__device__ inline half8_t unpack3_exact(uint32_t dl, uint32_t dh, const C& c) {
  const half8_t lo = unpack2<SS & 1>(dl, c);
  const half8_t hi = unpack1x4<SS>(dh, c);
  const uint4_t l = __builtin_bit_cast(uint4_t, lo), h = __builtin_bit_cast(uint4_t, hi);
  if ((SS & 1) == 0)
    return frag_from_words(pk_sub(pk_add(l.x, h.x), 132.0f), pk_sub(pk_add(l.y, h.y), 52.0f),
                           pk_sub(pk_add(l.z, h.z), 84.0f), pk_sub(pk_add(l.w, h.w), 28.0f));
  return frag_from_words(pk_sub(pk_add(l.x, h.x), 72.0f), pk_sub(pk_add(l.y, h.y), 100.0f),
                         pk_sub(pk_add(l.z, h.z), 36.0f), pk_sub(pk_add(l.w, h.w), 16.0f));
}

// int3 with the two planes added and their offsets left in the value (bias_frag<3>): one
// fragment, hence one MFMA, per step.
template <int SS, class C>
__device__ inline half8_t unpack3_sum(uint32_t dl, uint32_t dh, const C& c) {
  const uint4_t l = __builtin_bit_cast(uint4_t, unpack2<SS & 1>(dl, c));
  const uint4_t h = __builtin_bit_cast(uint4_t, unpack1x4<SS>(dh, c));
  return frag_from_words(pk_add(l.x, h.x), pk_add(l.y, h.y), pk_add(l.z, h.z), pk_add(l.w, h.w));
}

// Constant B fragment holding, per code position, the amount the unpacked value
// exceeds the signed code: exponent bias(es) + zero point.
template <int BITS>
__device__ inline half8_t bias_frag(int parity) {
  if (BITS == 8) return const_frag(1152, 1152, 1152, 1152);
  if (BITS == 4) return const_frag(0, 72, 0, 72);
  if (BITS == 2) return parity == 0 ? const_frag(66, 18, 66, 18) : const_frag(6, 66, 18, 6);
  // int3: low-plane bias + high-plane bias + zero point 4
  return parity == 0 ? const_frag(64 + 64 + 4, 16 + 32 + 4, 64 + 16 + 4, 16 + 8 + 4)
                     : const_frag(4 + 64 + 4, 64 + 32 + 4, 16 + 16 + 4, 4 + 8 + 4);
}

template <int BITS, int KSTEPS>
struct Shape {
  static constexpr int FB = moqe_field_bits(BITS);  // stored bits per code
  static constexpr int SCMAX = FB == 8 ? 2 : FB == 4 ? 4 : 8;
  static constexpr int SC = KSTEPS < SCMAX ? KSTEPS : SCMAX;  // steps per chunk
  static constexpr int NCH = KSTEPS / SC;                     // chunks per wave slice
  static constexpr int LO_BITS = FB == 3 ? 2 : FB;
  static constexpr int LW = SC * LO_BITS / 4;                 // main-plane words per lane per chunk
  static constexpr int HW = FB == 3 ? SC / 4 : 0;             // 1-bit-plane words per lane per chunk
  static constexpr int CHUNK_WORDS = 16 * SC * FB;            // 64 * SC * FB / 4
  static_assert(KSTEPS % SC == 0, "slice must hold whole chunks");
  static_assert(LW >= 1, "lane owns at least a word");
  static_assert(FB != 3 || HW >= 1, "3-bit codes need 4 steps per chunk");
};

template <int N>
__device__ inline void load_words(const uint32_t* p, uint32_t* dst) {
  if (N == 4) {
    uint4_t v = __builtin_nontemporal_load((const uint4_t*)p);
    dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
  } else if (N == 2) {
    uint2_t v = __builtin_nontemporal_load((const uint2_t*)p);
    dst[0] = v.x; dst[1] = v.y;
  } else {
    dst[0] = __builtin_nontemporal_load(p);
  }
}


// The same through a buffer descriptor: a load beyond the descriptor's size returns zero
// and touches no memory, so a wave can issue the loads of a unit it may not have without a
// branch.  Branch-free load sequences matter here: loads return in order under one counter,
// and only for straight-line code does the compiler know how many younger loads may still be
// in flight when it waits for an older one.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ inline rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}
template <int N, int NT = 2>  // NT = 2: streamed once, no reuse worth caching; 0: ordinary cached load
__device__ inline void load_words(rsrc_t r, uint32_t byte_off, uint32_t* dst) {
  if (N == 4) {
    uint4_t v = __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, NT);
    dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
  } else if (N == 2) {
    uint2_t v = __builtin_amdgcn_raw_buffer_load_b64(r, byte_off, 0, NT);
    dst[0] = v.x; dst[1] = v.y;
  } else {
    dst[0] = __builtin_amdgcn_raw_buffer_load_b32(r, byte_off, 0, NT);
  }
}
