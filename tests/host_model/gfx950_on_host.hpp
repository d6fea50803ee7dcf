// Test infrastructure: lets the kernels' per-block headers (csrc/codec.hpp, csrc/block.hpp)
// compile for the host, so that the CPU tests can run the very code the GPU runs -- block
// scales, both candidates, the estimate-then-verify 4-vs-6 decision, stochastic rounding --
// against the oracle on inputs no GPU run is needed for.
//
// It supplies what the device compiler provides and the host compiler does not: the
// launch-geometry variables, the workgroup barrier, bit casts, and the gfx950 conversion
// instructions.  Each round-to-nearest conversion is written here from the format definitions
// (nearest value of the format by threshold search, ties to the even code), independently of
// the oracle and of the kernels; that the instructions themselves round this way is what the
// GPU codec tests establish over their whole input range.
#pragma once

#include <hip/hip_runtime.h>   // vector types and the (empty on the host) function attributes

#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>

namespace host_model {

inline uint32_t bits_of(float f) {
  uint32_t u;
  std::memcpy(&u, &f, 4);
  return u;
}
inline float float_of(uint32_t u) {
  float f;
  std::memcpy(&f, &u, 4);
  return f;
}

// E2M1 magnitudes by code index
static const float kGrid[8] = {0.0f, 0.5f, 1.0f, 1.5f, 2.0f, 3.0f, 4.0f, 6.0f};

// nearest grid magnitude, ties to the even index, saturating
inline uint32_t e2m1_nearest(float x) {
  const float a = std::fabs(x);
  uint32_t k = 7;
  for (uint32_t i = 0; i < 7; ++i) {
    const float mid = 0.5f * (kGrid[i] + kGrid[i + 1]);   // exact
    if (a < mid || (a == mid && (i & 1u) == 0)) {
      k = i;
      break;
    }
  }
  return k | ((bits_of(x) >> 28) & 8u);
}

// v_cvt_scalef32_pk_fp4_f32: byte `sel` of `old` <- code(a / scale) | code(b / scale) << 4
inline uint32_t cvt_scalef32_pk_fp4_f32(uint32_t old, float a, float b, float scale, int sel) {
  const uint32_t byte = e2m1_nearest(a / scale) | (e2m1_nearest(b / scale) << 4);
  return (old & ~(0xffu << (8 * sel))) | (byte << (8 * sel));
}

typedef float hm_f32x2 __attribute__((ext_vector_type(2)));

// v_cvt_scalef32_pk_f32_fp4: the two codes of byte `sel`, as values times scale
inline hm_f32x2 cvt_scalef32_pk_f32_fp4(uint32_t src, float scale, int sel) {
  const uint32_t byte = (src >> (8 * sel)) & 0xffu;
  auto val = [&](uint32_t c) { return ((c & 8u) ? -kGrid[c & 7u] : kGrid[c & 7u]) * scale; };
  hm_f32x2 r = {val(byte & 15u), val(byte >> 4)};
  return r;
}

// v_cvt_scalef32_sr_pk_fp4_f32 as the kernels use it: only the code of the first source
// position counts (the nibble of the second is filled with a pattern here, so that nothing can
// depend on it).  Not a format definition but a description of what the instruction was
// measured to do, which the GPU codec tests check against the device over every fp32 value:
// the top 22 bits of the random operand are added to the 22 bits below the kept mantissa bit
// and the sum is truncated; below 1 the value is first cut to a multiple of 2^-23.
inline uint32_t cvt_scalef32_sr_pk_fp4_f32(uint32_t old, hm_f32x2 src, uint32_t rnd, int sel) {
  const float x = src.x, a = std::fabs(x);
  const uint32_t b = bits_of(a);
  uint32_t k;
  if (a >= 6.0f) {
    k = 7;
  } else if (a >= 1.0f) {
    k = (b >> 22) - 252u + (((rnd >> 10) + (b & 0x3fffffu)) >> 22);
  } else {
    const uint32_t p = (uint32_t)std::floor(std::ldexp((double)a, 23));   // < 2^23
    k = (p >> 22) + (((rnd >> 10) + (p & 0x3fffffu)) >> 22);
  }
  const uint32_t byte = k | ((bits_of(x) >> 28) & 8u) | 0xa0u;
  return (old & ~(0xffu << (8 * sel))) | (byte << (8 * sel));
}

// nearest E4M3 value of 0 <= x <= 448 (bias 7, subnormals m * 2^-9), ties to even
inline uint32_t e4m3_nearest(float x) {
  if (x < 0x1p-6f) return (uint32_t)std::nearbyint(std::ldexp((double)x, 9));   // 8 = first normal
  int e;
  const double m = std::frexp((double)x, &e);                 // x = m 2^e, m in [0.5, 1)
  int q = (int)std::nearbyint(std::ldexp(m, 4));              // 8 .. 16 eighths of 2^(e-1)
  e -= 1;
  if (q == 16) {
    q = 8;
    e += 1;
  }
  return (uint32_t)(((e + 7) << 3) | (q - 8));
}

// v_cvt_pk_fp8_f32 (OCP E4M3 on gfx950), used by the kernels on values already clamped to 448
inline int cvt_pk_fp8_f32(float a, float b, int old, bool hi) {
  const uint32_t two = e4m3_nearest(a) | (e4m3_nearest(b) << 8);
  return hi ? (int)(((uint32_t)old & 0xffffu) | (two << 16)) : (int)(((uint32_t)old & 0xffff0000u) | two);
}

inline uint32_t bitop3(uint32_t a, uint32_t b, uint32_t c, uint32_t table) {
  uint32_t r = 0;
  for (int i = 0; i < 32; ++i) {
    const uint32_t idx = (((a >> i) & 1u) << 2) | (((b >> i) & 1u) << 1) | ((c >> i) & 1u);
    r |= ((table >> idx) & 1u) << i;
  }
  return r;
}

struct Dim {
  unsigned x, y, z;
};

}  // namespace host_model

// one "lane" runs the whole workgroup's loops
static const host_model::Dim threadIdx = {0, 0, 0}, blockDim = {1, 1, 1};
inline void __syncthreads() {}
inline uint32_t __float_as_uint(float f) { return host_model::bits_of(f); }
inline float __uint_as_float(uint32_t u) { return host_model::float_of(u); }

#define __builtin_amdgcn_cvt_scalef32_pk_fp4_f32 host_model::cvt_scalef32_pk_fp4_f32
#define __builtin_amdgcn_cvt_scalef32_pk_f32_fp4 host_model::cvt_scalef32_pk_f32_fp4
#define NVFP4_46_CVT_SR_PK_FP4_ON_HOST host_model::cvt_scalef32_sr_pk_fp4_f32
#define __builtin_amdgcn_cvt_pk_fp8_f32 host_model::cvt_pk_fp8_f32
#define __builtin_amdgcn_bitop3_b32 host_model::bitop3
