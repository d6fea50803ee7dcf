// Device-side number formats and random numbers for the 4/6 NVFP4 kernels (gfx950).
//
// Every routine here is a scalar or per-lane building block; nothing touches
// memory.  Arithmetic on values is IEEE binary32 with one rounding per
// operation (the translation unit is compiled with -ffp-contract=off).
//
// Two implementations exist for the three narrow-format conversions:
//   *_sw  -- integer / magic-number code whose rounding can be read off the
//            source (round to nearest, ties to even, saturating);
//   *_hw  -- the gfx950 conversion instructions (v_cvt_scalef32_pk_fp4_f32,
//            v_cvt_pk_fp8_f32, v_cvt_pk_bf16_f32).
// NVFP4_46_HW_FP4 / _FP8 / _BF16 (0 or 1) pick which one the kernels use.  A
// hardware conversion is switched on only after the GPU tests have compared
// it with the CPU oracle over its whole input range.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#ifndef NVFP4_46_HW_FP4
#define NVFP4_46_HW_FP4 0
#endif
#ifndef NVFP4_46_HW_FP8
#define NVFP4_46_HW_FP8 0
#endif
#ifndef NVFP4_46_HW_BF16
#define NVFP4_46_HW_BF16 0
#endif

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

// fp32 -> BF16 bits, round to nearest even (finite inputs; overflow -> inf).
NV_DEV uint32_t bf16_rne_sw(float f) {
  uint32_t u = f2u(f);
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// Two fp32 -> one word of two BF16 (a in the low half).
NV_DEV uint32_t pack_bf16x2(float a, float b) {
#if NVFP4_46_HW_BF16
  f32x2 v = {a, b};
  bf16x2 h = __builtin_convertvector(v, bf16x2);
  return *reinterpret_cast<uint32_t *>(&h);
#else
  return bf16_rne_sw(a) | (bf16_rne_sw(b) << 16);
#endif
}

// ------------------------------------------------------------------ E2M1

// Value of a 4-bit code: sign<<3 | index into {0,.5,1,1.5,2,3,4,6} (Section 1).
NV_DEV float e2m1_decode_sw(uint32_t code) {
  uint32_t k = code & 7u;
  // index k >= 2 is a normal number 2^(k/2 - 1) * (1 + (k&1)/2); 0 and 1 are 0 and 0.5
  uint32_t bits = (k >= 2u) ? (((k >> 1) + 126u) << 23) | ((k & 1u) << 22)
                            : (k ? 0x3f000000u : 0u);
  return u2f(bits | ((code & 8u) << 28));
}

// Round |y| (clamped to 6) to the nearest E2M1 magnitude, ties to the even
// index (Eq. 3 with half-even rounding).  Returns the 3-bit index and writes
// the rounded magnitude.
NV_DEV uint32_t e2m1_rtn_mag_sw(float a, float &r) {
  // below 2 the grid step is 0.5: adding 2^22 (whose ulp is 0.5) rounds to a
  // multiple of 0.5 half-even, and the low mantissa bits are then the index
  if (a < 2.0f) {
    float t = a + 4194304.0f;
    r = t - 4194304.0f;
    return f2u(t) & 7u;
  }
  // from 2 up the grid is "one mantissa bit": round the fp32 mantissa to its
  // top bit half-even; a carry moves into the exponent as it should
  uint32_t u = f2u(a);
  u = (u + 0x1fffffu + ((u >> 22) & 1u)) >> 22;   // (exponent << 1) | mantissa bit
  r = u2f(u << 22);
  return u - 252u;                                 // exponent 128 -> index 4
}

// Code of y under round-to-nearest-even, saturating at +-6.
NV_DEV uint32_t e2m1_rtn_sw(float y) {
  float r;
  uint32_t k = e2m1_rtn_mag_sw(fminf(fabsf(y), 6.0f), r);
  return k | ((f2u(y) >> 28) & 8u);
}

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

// Code of a value that is already on the grid (sign included).
NV_DEV uint32_t e2m1_code_of_grid_value(float r) {
  uint32_t u = f2u(r);
  uint32_t m = u & 0x7fffffffu;
  uint32_t k = (m >= 0x3f800000u) ? (m >> 22) - 252u : (m ? 1u : 0u);
  return k | ((u >> 28) & 8u);
}

// ------------------------------------------------------------------ E4M3

// Value of an E4M3 byte 0x00..0x7E (bias 7, subnormals m * 2^-9).
NV_DEV float e4m3_decode_sw(uint32_t b) {
  uint32_t e = (b >> 3) & 15u, m = b & 7u;
  return e ? u2f(((e + 120u) << 23) | (m << 20)) : (float)m * 0x1p-9f;
}

// Non-negative fp32 -> E4M3 byte, round to nearest even, saturating at 448.
NV_DEV uint32_t e4m3_encode_sw(float x) {
  x = fminf(x, 448.0f);
  if (x < 0x1p-6f) {
    // subnormal range: multiples of 2^-9; the scaling is exact and rint is
    // half-even; a result of 8 is the byte of 2^-6, the first normal value
    return (uint32_t)__builtin_rintf(x * 512.0f);
  }
  uint32_t u = f2u(x);
  u = (u + 0x7ffffu + ((u >> 20) & 1u)) >> 20;       // (exponent << 3) | 3 mantissa bits
  return u - (120u << 3);
}

NV_DEV uint32_t e4m3_encode(float x) {
#if NVFP4_46_HW_FP8
  x = fminf(x, 448.0f);
  return (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(x, x, 0, false) & 0xffu;
#else
  return e4m3_encode_sw(x);
#endif
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

// The four uniforms of the element group q = g >> 2 (g = flat element index).
NV_DEV void sr_uniforms4(uint64_t seed, uint64_t q, float u[4]) {
  Philox4 p = philox4x32_10((uint32_t)q, (uint32_t)(q >> 32), 0u, 0u, (uint32_t)seed,
                            (uint32_t)(seed >> 32));
#pragma unroll
  for (int j = 0; j < 4; ++j) u[j] = (float)(p.w[j] >> 8) * 0x1p-24f;
}

// Sign word of the block at position B along the blocked axis (bit j = negate element j).
NV_DEV uint32_t rht_sign_word(uint64_t seed, uint64_t B) {
  return philox4x32_10((uint32_t)B, (uint32_t)(B >> 32), 0u, 1u, (uint32_t)seed,
                       (uint32_t)(seed >> 32)).w[0];
}

// ------------------------------------------------------------ Hadamard

// v <- (1/4) H16 (s .* v): sign flips, then butterflies with strides 1, 2, 4, 8.
NV_DEV void rht16(float (&v)[16], uint32_t sign_word) {
#pragma unroll
  for (int j = 0; j < 16; ++j) v[j] = u2f(f2u(v[j]) ^ (((sign_word >> j) & 1u) << 31));
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

}  // namespace nvfp4_46
