// Device-side number formats and random numbers for the 4/6 NVFP4 kernels (gfx950).
//
// Every routine here is a scalar or per-lane building block; nothing touches
// memory.  Arithmetic on values is IEEE binary32 with one rounding per
// operation (the translation unit is compiled with -ffp-contract=off).
//
// The three narrow-format roundings (fp32 -> E2M1, fp32 -> E4M3, fp32 -> BF16) are the
// gfx950 conversion instructions v_cvt_scalef32_pk_fp4_f32, v_cvt_pk_fp8_f32 and
// v_cvt_pk_bf16_f32: the GPU tests compare each with the CPU oracle over its whole
// input range (round to nearest, ties to even, saturating).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#define NV_DEV __device__ __forceinline__

namespace nvfp4_46 {

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

NV_DEV uint32_t f2u(float f) { return __float_as_uint(f); }
NV_DEV float u2f(uint32_t u) { return __uint_as_float(u); }

// ------------------------------------------------------------------ BF16

// A 32-bit word holds two BF16 values; element 0 is the low half.
NV_DEV float bf16_lo(uint32_t w) { return u2f(w << 16); }
NV_DEV float bf16_hi(uint32_t w) { return u2f(w & 0xffff0000u); }

// Two fp32 -> one word of two BF16 (a in the low half), round to nearest even, overflow
// to infinity (v_cvt_pk_bf16_f32).
NV_DEV uint32_t pack_bf16x2(float a, float b) {
  f32x2 v = {a, b};
  bf16x2 h = __builtin_convertvector(v, bf16x2);
  return *reinterpret_cast<uint32_t *>(&h);
}

// ------------------------------------------------------------------ E2M1

// A 4-bit code is sign<<3 | index into {0,.5,1,1.5,2,3,4,6} (Section 1).

// Stochastic rounding of y with uniform u in [0,1): lo <= |y| < hi neighbours on the
// grid, up iff u < (|y|-lo)/(hi-lo).  The grid step around a = min(|y|, 6) is a power of
// two (0.5 below 2, then 1, then 2), so q = a/step is an exact scaling, lo/step = floor(q)
// and the probability (|y|-lo)/(hi-lo) = q - floor(q), all without rounding.  Returns the
// signed rounded value (exactly representable), from which code and dequantized value
// both follow.
NV_DEV float e2m1_sr_value(float y, float u) {
  const float a = fminf(fabsf(y), 6.0f);
  uint32_t e = f2u(a) & 0x7f800000u;                    // 2^floor(log2 a)
  e = e > 0x3f800000u ? e : 0x3f800000u;                // everything below 2 steps by 0.5
  const uint32_t step_bits = e - 0x00800000u;           // step = 2^(exponent-1)
  const float q = a * u2f(0x7f000000u - step_bits);     // a / step, in [0, 4)
  const float fl = __builtin_floorf(q);
  const float up = (u < q - fl) ? 1.0f : 0.0f;
  const float r = (fl + up) * u2f(step_bits);
  return u2f(f2u(r) | (f2u(y) & 0x80000000u));
}

// v_cvt_scalef32_sr_pk_fp4_f32: byte SEL of `old` <- the stochastically rounded E2M1 codes of
// the two values of src (first in the low nibble), the other bytes kept.  Written as inline
// assembly because the compiler's builtin for it drops `old` (the other bytes come out as
// whatever the destination register held); the s_nop gives the partial register write its one
// wait state before any reader, which the compiler only inserts for instructions it emits
// itself.  (The host-side test build of this header substitutes a description of the
// instruction.)
// SEL = kSrFirstByteOfNewWord writes byte 0 and leaves the other three bytes undefined (no
// previous word has to be brought into the destination register).
constexpr int kSrFirstByteOfNewWord = 4;
template <int SEL>
NV_DEV uint32_t cvt_sr_pk_fp4(uint32_t old, f32x2 src, uint32_t rnd) {
#ifdef NVFP4_46_CVT_SR_PK_FP4_ON_HOST
  return NVFP4_46_CVT_SR_PK_FP4_ON_HOST(old, src, rnd, SEL & 3);
#else
  if constexpr (SEL == 0)
    asm("v_cvt_scalef32_sr_pk_fp4_f32 %0, %1, %2, 1.0\n\ts_nop 0" : "+v"(old) : "v"(src), "v"(rnd));
  else if constexpr (SEL == kSrFirstByteOfNewWord)
    asm("v_cvt_scalef32_sr_pk_fp4_f32 %0, %1, %2, 1.0\n\ts_nop 0" : "=v"(old) : "v"(src), "v"(rnd));
  else if constexpr (SEL == 1)
    asm("v_cvt_scalef32_sr_pk_fp4_f32 %0, %1, %2, 1.0 op_sel:[0,0,1,0]\n\ts_nop 0" : "+v"(old) : "v"(src), "v"(rnd));
  else if constexpr (SEL == 2)
    asm("v_cvt_scalef32_sr_pk_fp4_f32 %0, %1, %2, 1.0 op_sel:[0,0,0,1]\n\ts_nop 0" : "+v"(old) : "v"(src), "v"(rnd));
  else
    asm("v_cvt_scalef32_sr_pk_fp4_f32 %0, %1, %2, 1.0 op_sel:[0,0,1,1]\n\ts_nop 0" : "+v"(old) : "v"(src), "v"(rnd));
  return old;
#endif
}

// A word whose content does not matter (every byte of it is about to be overwritten by
// instructions that replace one byte each): whatever register the compiler picks, with no
// instruction spent on initialising it.
NV_DEV uint32_t any_register() {
  uint32_t w = 0u;
#ifndef NVFP4_46_CVT_SR_PK_FP4_ON_HOST
  asm("" : "=v"(w));
#endif
  return w;
}

// Makes the compiler hold a two-float vector in an aligned pair of vector registers at this
// point (.x in the even one, .y in the odd one).
NV_DEV void in_register_pair(f32x2 &p) {
#ifndef NVFP4_46_CVT_SR_PK_FP4_ON_HOST
  asm("" : "+v"(p));
#endif
}

// A constant the compiler must keep in a vector register, and in an odd-numbered one: it would
// otherwise put a literal used this often into a scalar register, and an fp32 instruction with
// a scalar-register source issues at half the rate (measured: v_fma_f32 2.4 against 4.2 cycles
// per wave and SIMD); a three-source instruction also falls to half rate when all three sources
// sit in registers of the same parity, which a known parity of one of them can rule out.
NV_DEV float in_odd_vector_register(float c) {
#ifndef NVFP4_46_CVT_SR_PK_FP4_ON_HOST
  f32x2 p;
  asm("v_mov_b32 %0, %1" : "=v"(p.y) : "s"(c));
  p.x = p.y;
  asm("" : "+v"(p));
  return p.y;
#else
  return c;
#endif
}

// The rounding of e2m1_sr_value() by that instruction, for the element whose random word is
// w (passed as not_w = ~w and wf = (float)w, which a caller rounding the same element under
// several scales computes once).  Only the first source position is used: with ~w as the
// random operand the instruction adds the operand's top 22 bits to the 22 bits below the kept
// mantissa bit and truncates (the second position reads other bits of the operand and cannot
// be given an independent uniform; its nibble is left to be masked off by the caller).  With
// k = w >> 8, so that u = k * 2^-24:
//   |y| >= 1: one step up iff (k >> 2) < (low 22 mantissa bits): exactly u < p, because p has
//             22 bits there;
//   |y| < 1 : the grid step is 0.5 and p = frac(2|y|); the instruction cuts |y| to a multiple
//             of 2^-23 first, i.e. compares k >> 2 with P = floor(|y| * 2^23) mod 2^22.  That
//             is u < p unless k >> 2 == P, which implies |A - k| < 4 for A = |y| * 2^25 (below
//             0.5) or A = |y| * 2^25 - 2^24 (from 0.5 up).
// Magnitudes above 6 give 6, the sign bit is the input's also when the magnitude becomes 0.
// (The GPU tests compare the instruction, used this way, with the CPU oracle and with this
// description on every fp32 value, for several words.)
// The risk is tested 256 times larger, on the whole word, which saves the shift: with
// t = fl(|y| * 2^33 - wf), |wf - w| <= 128 and w = 256 k + (0..255), |A - k| < 4 implies
// |t| < 1024 + 383 + rounding, and |A - 2^24 - k| < 4 implies |t - 2^32| < 1407 + 256 (t is
// rounded to a multiple of 512 up there).  `margin` is lowered to the smaller of |t| and
// |t - 2^32| where that is smaller still: a caller that finds margin <= kSrMarginAtRisk after a
// group of elements must redo the group with e2m1_sr_value().  Returns `old` with the low
// nibble of byte SEL replaced by the code; the high nibble of that byte is left undefined.
template <int SEL>
NV_DEV uint32_t e2m1_sr_code_fast(uint32_t old, float y, uint32_t not_w, float wf, float &margin) {
  // {y, t} is the register pair the conversion reads: y in its even half, so with the constant
  // in an odd register the three sources of the fma never share a parity.  The second source
  // position of the conversion only has to be some register: t is at hand, and as a value
  // computed here it can be placed next to y without a copy.
  const float t = __builtin_fmaf(fabsf(y), in_odd_vector_register(0x1p33f), -wf);
  margin = fminf(fminf(margin, fabsf(t)), fabsf(t - 0x1p32f));   // one v_min3_f32
  const f32x2 src = {y, t};
  return cvt_sr_pk_fp4<SEL>(old, src, not_w);
}
constexpr float kSrMarginAtRisk = 2048.0f;

// Code of a value that is already on the grid (sign included).
NV_DEV uint32_t e2m1_code_of_grid_value(float r) {
  uint32_t u = f2u(r);
  uint32_t m = u & 0x7fffffffu;
  uint32_t k = (m >= 0x3f800000u) ? (m >> 22) - 252u : (m ? 1u : 0u);
  return k | ((u >> 28) & 8u);
}

// ------------------------------------------------------------------ E4M3

// Value of an E4M3 byte 0x00..0x7E (bias 7, subnormals m * 2^-9).
NV_DEV float e4m3_decode(uint32_t b) {
  uint32_t e = (b >> 3) & 15u, m = b & 7u;
  return e ? u2f(((e + 120u) << 23) | (m << 20)) : (float)m * 0x1p-9f;
}

// Non-negative fp32 -> E4M3 byte, round to nearest even, saturating at 448 (the clamp
// comes first: the conversion instruction alone turns values past 448 into NaN).
NV_DEV uint32_t e4m3_encode(float x) {
  x = fminf(x, 448.0f);
  return (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(x, x, 0, false) & 0xffu;
}

// Two of them with one conversion instruction: byte 0 = e4m3(a), byte 1 = e4m3(b).
NV_DEV uint32_t e4m3_encode2(float a, float b) {
  return (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(fminf(a, 448.0f), fminf(b, 448.0f), 0, false) & 0xffffu;
}

// --------------------------------------------------------------- Philox

// a ^ b ^ c in one instruction (v_bitop3_b32 with the truth table of a 3-input XOR)
NV_DEV uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
  return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

// Philox4x32-10 (Salmon et al., SC'11).
struct Philox4 {
  uint32_t w[4];
};

NV_DEV Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                             uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;   // one 32x32->64 multiply each
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    c0 = xor3((uint32_t)(p1 >> 32), c1, k0);
    c1 = (uint32_t)p1;
    c2 = xor3((uint32_t)(p0 >> 32), c3, k1);
    c3 = (uint32_t)p0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return Philox4{{c0, c1, c2, c3}};
}

// The four random words of the element group q = g >> 2 (g = flat element index).  An
// element's uniform is the top 24 bits of its word, u = (w >> 8) * 2^-24.
NV_DEV void sr_words4(uint64_t seed, uint64_t q, uint32_t w[4]) {
  Philox4 p = philox4x32_10((uint32_t)q, (uint32_t)(q >> 32), 0u, 0u, (uint32_t)seed,
                            (uint32_t)(seed >> 32));
#pragma unroll
  for (int j = 0; j < 4; ++j) w[j] = p.w[j];
}
NV_DEV float sr_uniform_of_word(uint32_t w) { return (float)(w >> 8) * 0x1p-24f; }

// Sign word of the block at position B along the blocked axis (bit j = negate element j).
NV_DEV uint32_t rht_sign_word(uint64_t seed, uint64_t B) {
  return philox4x32_10((uint32_t)B, (uint32_t)(B >> 32), 0u, 1u, (uint32_t)seed,
                       (uint32_t)(seed >> 32)).w[0];
}

// ------------------------------------------------------------ Hadamard

// v <- (1/4) H16 v: butterflies with strides 1, 2, 4, 8.
NV_DEV void hadamard16_quarter(float (&v)[16]) {
#pragma unroll
  for (int h = 1; h < 16; h <<= 1) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      if ((i & h) == 0) {
        float p = v[i], q = v[i + h];
        v[i] = p + q;
        v[i + h] = p - q;
      }
    }
  }
#pragma unroll
  for (int j = 0; j < 16; ++j) v[j] *= 0.25f;
}
// v <- (1/4) H16 (s .* v): sign flips (bit j of sign_word negates element j), then the butterflies.
NV_DEV void rht16(float (&v)[16], uint32_t sign_word) {
#pragma unroll
  for (int j = 0; j < 16; ++j) v[j] = u2f(f2u(v[j]) ^ (((sign_word >> j) & 1u) << 31));
  hadamard16_quarter(v);
}

// The same with the sign flips given as sixteen XOR masks (0 or 0x80000000), for callers
// that meet the same sign word block after block.
NV_DEV void rht_sign_masks(uint32_t sign_word, uint32_t (&mask)[16]) {
#pragma unroll
  for (int j = 0; j < 16; ++j) mask[j] = ((sign_word >> j) & 1u) << 31;
}
NV_DEV void rht16_masked(float (&v)[16], const uint32_t (&mask)[16]) {
#pragma unroll
  for (int j = 0; j < 16; ++j) v[j] = u2f(f2u(v[j]) ^ mask[j]);
  hadamard16_quarter(v);
}

}  // namespace nvfp4_46
