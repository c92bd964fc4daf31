// Device-side building blocks of the ECO step for gfx950 (wave64): number formats, the
// Philox4x32-10 generator, the grid encoders (stochastic and nearest-even rounding) and the
// in-wave abs-max reduction.  Everything here is exact integer or single-operation IEEE fp32
// arithmetic, so results are reproducible bit for bit on any conforming implementation.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "eco_internal.hpp"

namespace eco {


__device__ __forceinline__ uint32_t f2u(float x) { return __float_as_uint(x); }
__device__ __forceinline__ float u2f(uint32_t x) { return __uint_as_float(x); }

// Votes over the active lanes of the wave, taken on the comparison's own lane mask.
__device__ __forceinline__ bool wave_all(bool p) { return __builtin_amdgcn_ballot_w64(p) == __builtin_amdgcn_read_exec(); }
__device__ __forceinline__ bool wave_any(bool p) { return __builtin_amdgcn_ballot_w64(p) != 0; }

// ---------------------------------------------------------------------------------- bfloat16
// A bfloat16 is the upper half of an fp32.
__device__ __forceinline__ float bf16_lo(uint32_t packed) { return u2f(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return u2f(packed & 0xFFFF0000u); }

// fp32 -> bfloat16 bits, round to nearest even (finite inputs).
__device__ __forceinline__ uint32_t f32_to_bf16_rne(float x) {
  uint32_t u = f2u(x);
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// Two fp32 -> one dword of two bfloat16 (lo in the low half), round to nearest even.  The vector
// conversion compiles to gfx950's packed conversion instruction, whose result equals
// f32_to_bf16_rne() for every finite fp32 input (compared exhaustively on the device).
typedef __bf16 eco_bf16x2_t __attribute__((ext_vector_type(2)));
typedef float eco_f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t f32x2_to_bf16x2_rne(float lo, float hi) {
  const eco_f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, eco_bf16x2_t));
}

// ---------------------------------------------------------------------------------- E4M3 (OCP)
// Decode byte SEL of a dword holding four codes.  gfx950's fp8 conversion instructions implement
// the OCP E4M3 encoding (bias 7, subnormals, S.1111.111 = NaN), and a decode is exact, so the
// hardware instruction is used; the GPU tests decode all 256 codes against the format definition.
template <int SEL>
__device__ __forceinline__ float e4m3_decode(uint32_t packed) {
  return __builtin_amdgcn_cvt_f32_fp8((int)packed, SEL);
}

// Correctly rounded fp32 square root for 2^-96 <= x <= 2^96: the hardware's reciprocal-square-root estimate r (1 ulp),
// g = x r and h = r / 2 as first approximations of sqrt(x) and 1 / (2 sqrt(x)), one coupled Newton step on the pair,
// and a last correction of g by its exact residual x - g^2 (a fused multiply-add) times h.  It is the textbook
// Newton-Markstein square root without the input scaling and special-value handling that only matter outside that
// range; sqrtf() covers the rest.  (Compared on the device with sqrtf() for every fp32 of the range; the library's
// self-test entry repeats the sweep.)
__device__ __forceinline__ float sqrt_rn_midrange(float x) {
  const float r = __builtin_amdgcn_rsqf(x);
  float g = x * r;
  float h = 0.5f * r;
  const float e = fmaf(-h, g, 0.5f);
  g = fmaf(g, e, g);
  h = fmaf(h, e, h);
  const float d = fmaf(-g, g, x);
  return fmaf(d, h, g);
}
constexpr uint32_t SQRT_MID_LO = 0x0F800000u;   // 2^-96
constexpr uint32_t SQRT_MID_HI = 0x6F800000u;   // 2^96

// Correctly rounded fp32 quotient n / d for 2^-40 <= |n| <= 2^40 and 2^-48 <= |d| <= 2^49.  It is the sequence
// the compiler emits for `/` (reciprocal estimate, one Newton step on the reciprocal, the quotient, and two
// residual corrections, every step a fused multiply-add) without its operand pre-scaling, post-scaling and
// special-case fix-up: in the stated ranges neither operand is scaled (no denormal, the exponents less than
// 96 apart, reciprocal and quotient normal) and the fix-up passes the value through, so the result is the
// one `/` gives, bit for bit; `/` covers everything outside.  (Compared on the device for every d of the
// range against `/`; the library's self-test entry repeats the sweep.)
__device__ __forceinline__ float div_rn_midrange(float n, float d) {
  const float y0 = __builtin_amdgcn_rcpf(d);
  const float e0 = fmaf(-d, y0, 1.0f);
  const float y1 = fmaf(e0, y0, y0);
  const float q0 = n * y1;
  const float r0 = fmaf(-d, q0, n);
  const float q1 = fmaf(r0, y1, q0);
  const float r1 = fmaf(-d, q1, n);
  return fmaf(r1, y1, q1);
}
constexpr float DIV_MID_N_LO = 0x1p-40f, DIV_MID_N_HI = 0x1p40f;      // numerator range of div_rn_midrange

// Position of |y| on the E4M3 code axis, in units of 2^-20 codes: codes are linear in the fp32
// bit pattern above 2^-6 (three mantissa bits kept, twenty dropped) and linear in the value
// below it (spacing 2^-9), where the fp32 addition of 2^-6 performs the round-to-nearest-even
// onto multiples of 2^-29.
//
// Stochastic rounding (Sec. 3.1: up with a probability proportional to the distance from the lower
// neighbour, an unbiased estimator): with F the 20-bit fraction of the axis position and r the
// element's 16 random bits, the code goes up iff F + 16 r + 8 >= 2^20, i.e. with probability
// floor((F + 8) / 16) / 2^16 -- the fraction rounded to the nearest multiple of 2^-16, so that the
// 16-bit resolution has no preferred direction (Assumption 3.2 wants a zero-mean error).  The +8 is
// folded into the constants below.  F = 0 never goes up: 8 + 16 * 65535 < 2^20.
constexpr uint32_t E4M3_MIN_NORMAL_BITS = 0x3C800000u;     // fp32 bit pattern of 2^-6
constexpr uint32_t SR_CENTRE = 8u;                         // half of the 2^4 fraction units one random unit is worth

// f + MUL * h modulo 2^32, h = the low (HALF = 0) or high (HALF = 1) 16 bits of a Philox word: the random field of an
// element, 16 bits that stand for the top 16 of the 20 fraction bits of a grid step.  One v_mad_u32_u16 (u16 x u16 + u32;
// op_sel picks the half of the word).
template <int HALF, uint32_t MUL>
__device__ __forceinline__ uint32_t add_random_field(uint32_t f, uint32_t word) {
  uint32_t t;
  if constexpr (MUL <= 64u) {       // an inline constant
    if (HALF) asm("v_mad_u32_u16 %0, %1, %2, %3 op_sel:[1,0,0,0]" : "=v"(t) : "v"(word), "n"(MUL), "v"(f));
    else asm("v_mad_u32_u16 %0, %1, %2, %3" : "=v"(t) : "v"(word), "n"(MUL), "v"(f));
  } else {                // from a scalar register
    if (HALF) asm("v_mad_u32_u16 %0, %1, %2, %3 op_sel:[1,0,0,0]" : "=v"(t) : "v"(word), "s"(MUL), "v"(f));
    else asm("v_mad_u32_u16 %0, %1, %2, %3" : "=v"(t) : "v"(word), "s"(MUL), "v"(f));
  }
  return t;
}

// The E4M3 code of y (magnitude ay >= 0, sign bit taken from `sign_from`) in the TOP BYTE of the returned word; the
// lower bytes hold leftovers of the rounding arithmetic.  pack_top_bytes4() gathers four such words into a dword of
// codes.  NORMAL_ONLY: the caller guarantees ay >= 2^-6 (the common case, decided once per wave).  The element's
// random field is half HALF of `word`.
template <int ROUND, bool NORMAL_ONLY, int HALF>
__device__ __forceinline__ uint32_t e4m3_encode_top(float ay, uint32_t word, uint32_t sign_from) {
  const uint32_t b = f2u(ay);
  uint32_t t;
  if (ROUND == ROUND_SR) {
    // position on the code axis in units of 2^-24 codes, (b - (0x3C000000 - 8)) << 4 (code 8 <-> 0x3C800000; below
    // 2^28, so the arithmetic modulo 2^32 is exact): one shift-and-add; the random field then enters times 2^8 and
    // the code is the top byte: up iff frac20 + 16 r + 8 >= 2^20
    uint32_t axis = (b << 4) + (0u - ((0x3C000000u - SR_CENTRE) << 4));
    if (!NORMAL_ONLY && b < E4M3_MIN_NORMAL_BITS) axis = (f2u(ay + 0x1p-6f) - (0x3C800000u - SR_CENTRE)) << 4;
    t = add_random_field<HALF, 256u>(axis, word);
  } else {
    uint32_t mag;
    if (NORMAL_ONLY || b >= E4M3_MIN_NORMAL_BITS) {
      const uint32_t k = b - 0x3C000000u;
      mag = (k + 0x7FFFFu + ((k >> 20) & 1u)) >> 20;        // nearest, ties to the even code
    } else {
      mag = f2u(ay + 0x1p14f) - 0x46800000u;                // ulp(2^14) = 2^-9: exact nearest-even
    }
    t = mag << 24;
  }
  t = t < 0x7EFFFFFFu ? t : 0x7EFFFFFFu;                    // saturate at 448 (0x7E)
  return t | (sign_from & 0x80000000u);
}

// Byte j of the result = the top byte of t_j.
__device__ __forceinline__ uint32_t pack_top_bytes4(uint32_t t0, uint32_t t1, uint32_t t2, uint32_t t3) {
  const uint32_t lo = __builtin_amdgcn_perm(t1, t0, 0x0c0c0703u);   // bytes: t0.b3, t1.b3, 0, 0
  const uint32_t hi = __builtin_amdgcn_perm(t3, t2, 0x07030c0cu);   // bytes: 0, 0, t2.b3, t3.b3
  return lo | hi;
}

// ---------------------------------------------------------------------------------- INT4
// Eight two's-complement nibbles in a dword, element j in bits 4j..4j+3.
//
// Decode: gfx950's v_cvt_off_f32_i4 maps the low four bits of its operand, read as a signed nibble n, to
// n / 16 exactly, and takes its operand from any byte of a register.  Odd elements sit in the high nibbles,
// so one shift of the dword by 4 puts them in reach too.  The caller multiplies by 16 * scale instead of
// scale: (n/16) * (16 s) is the same real product as n * s, hence the same rounded fp32 (16 s is exact;
// scales of 2^124 and more, for which it would overflow, are outside what the library supports).
template <int J>
__device__ __forceinline__ float int4_decode_sixteenth(uint32_t packed, uint32_t packed_shr4) {
  const uint32_t src = (J & 1) ? packed_shr4 : packed;
  return __builtin_amdgcn_cvt_off_f32_i4((int)((src >> (8 * (J >> 1))) & 0xFFu));
}

// round(y) in [-7, 7] as a float carrying the sign of y (a zero result keeps y's sign: -0.0f decodes and
// subtracts exactly like +0.0f everywhere it is used).  Needs |y| < 8 + 2^-3, which abs-max scaling guarantees
// (|y| <= 7 (1 + 2^-8) even when a bf16 scale was rounded down).
template <int ROUND, int HALF>
__device__ __forceinline__ float int4_round(float y, uint32_t word) {
  const float ay = __builtin_fabsf(y);
  uint32_t mag;
  if (ROUND == ROUND_SR) {
    // ulp(8.0) = 2^-20: the addition rounds |y| to the nearest-even multiple of 2^-20 and puts it, as a 4.20
    // fixed-point number, into the low 24 bits of the result.  The addend also carries the centring term of the
    // rounding rule, 8 units of 2^-20 -- an exact multiple of the ulp, so it commutes with the rounding -- which
    // leaves "up iff frac20 + 16*r16 + 8 >= 2^20" as one shift-and-add and a bit-field extract.  (|y| + 8 + 2^-17
    // can reach the next binade only for |y| > 7.9999, where bit 23 is set and the result saturates at 7 anyway.)
    const uint32_t t = add_random_field<HALF, 16u>(f2u(ay + (8.0f + 0x1p-17f)), word);
    mag = (t >> 20) & 15u;
  } else {
    mag = f2u(ay + 0x1p23f) - 0x4B000000u;                  // ulp(2^23) = 1: exact nearest-even
  }
  mag = mag < 7u ? mag : 7u;
  return u2f((f2u(y) & 0x80000000u) | f2u((float)mag));
}

// Insert the nibble of q (an integer in [-7, 7] held as a float) for element J into the byte accumulators:
// `even` collects elements 0, 2, 4, 6 in its bytes, `odd` elements 1, 3, 5, 7, each as q + 8 in [1, 15]
// (v_cvt_pk_u8_f32 converts and inserts in one instruction); int4_pack() turns the pair into the dword.
template <int J>
__device__ __forceinline__ void int4_insert(float q, uint32_t &even, uint32_t &odd) {
  if (J & 1) odd = __builtin_amdgcn_cvt_pk_u8_f32(q + 8.0f, J >> 1, odd);
  else even = __builtin_amdgcn_cvt_pk_u8_f32(q + 8.0f, J >> 1, even);
}
__device__ __forceinline__ uint32_t int4_pack(uint32_t even, uint32_t odd) {
  return (even | (odd << 4)) ^ 0x88888888u;                // offset-8 nibbles -> two's complement
}

// ---------------------------------------------------------------------------------- Philox4x32-10
// Salmon, Moraes, Dror, Shaw, "Parallel random numbers: as easy as 1, 2, 3" (SC'11).
struct Philox4 { uint32_t w0, w1, w2, w3; };

__device__ __forceinline__ Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                 uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return Philox4{c0, c1, c2, c3};
}

// ---------------------------------------------------------------------------------- abs-max
// All-reduce max over groups of `lanes` consecutive lanes (4, 8, 16, 32 or 64; wave-uniform) of
// the bit patterns of non-negative floats (for which unsigned integer order is float order): DPP
// row operations inside a 16-lane row, LDS-crossbar swizzles across rows.  max is exact and order
// independent, so every lane of a group ends with the same bits.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_umax(uint32_t x) {
  const uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xF, 0xF, true);
  return x > o ? x : o;
}

__device__ __forceinline__ uint32_t group_umax(uint32_t x, int lanes) {
  x = dpp_umax<0xB1>(x);                    // quad_perm [1,0,3,2]
  x = dpp_umax<0x4E>(x);                    // quad_perm [2,3,0,1]
  if (lanes >= 8) x = dpp_umax<0x141>(x);   // row_half_mirror
  if (lanes >= 16) x = dpp_umax<0x140>(x);  // row_mirror
  if (lanes >= 32) { const uint32_t o = (uint32_t)__shfl_xor((int)x, 16, 64); x = x > o ? x : o; }
  if (lanes >= 64) { const uint32_t o = (uint32_t)__shfl_xor((int)x, 32, 64); x = x > o ? x : o; }
  return x;
}

}  // namespace eco
