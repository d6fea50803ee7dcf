// One-lane-per-block 4/6 quantization of 16 fp32 values held in registers
// (arXiv 2512.02010, Table 3 lines 1-14, with the tensor scale of Eq. (1)-(3)).
#pragma once

#include "codec.hpp"

namespace nvfp4_46 {

enum : int { kRTN = 0, kSR = 1 };
enum : int { kSel46 = 0, kSelForce6 = 1, kSelForce4 = 2 };

// (dec, enc) for every E4M3 scale byte under one tensor scale:
//   dec = value(S) * alpha   -- what one unit of code is worth (Table 3 line 5)
//   enc = 1 / dec            -- multiplying by it is the division of Eq. (3);
//                               0 when dec is 0, so an all-zero block encodes to zeros
// Both depend on (S, alpha) only, so a workgroup computes the 127 pairs once
// into LDS instead of one IEEE division per block and candidate.
struct ScaleTable {
  float2 e[128];
};

NV_DEV void build_scale_table(ScaleTable &tab, float alpha) {
  for (uint32_t s = threadIdx.x; s < 128u; s += blockDim.x) {
    float dec = (s < 127u) ? e4m3_decode_sw(s) * alpha : 0.0f;
    float enc = (dec == 0.0f) ? 0.0f : 1.0f / dec;
    tab.e[s] = make_float2(dec, enc);
  }
  __syncthreads();
}

// The packed FP4 conversions take the destination / source byte as an immediate.
template <int SEL>
NV_DEV uint32_t hw_pk_fp4(uint32_t old, float a, float b) {
  return __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(old, a, b, 1.0f, SEL);
}
NV_DEV uint32_t hw_pk_fp4_sel(uint32_t old, float a, float b, int sel) {
  switch (sel) {
    case 0: return hw_pk_fp4<0>(old, a, b);
    case 1: return hw_pk_fp4<1>(old, a, b);
    case 2: return hw_pk_fp4<2>(old, a, b);
    default: return hw_pk_fp4<3>(old, a, b);
  }
}
template <int SEL>
NV_DEV f32x2 hw_pk_f32_fp4(uint32_t src) {
  return __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(src, 1.0f, SEL);
}
NV_DEV f32x2 hw_pk_f32_fp4_sel(uint32_t src, int sel) {
  switch (sel) {
    case 0: return hw_pk_f32_fp4<0>(src);
    case 1: return hw_pk_f32_fp4<1>(src);
    case 2: return hw_pk_f32_fp4<2>(src);
    default: return hw_pk_f32_fp4<3>(src);
  }
}

// Sum of 16 squared errors in the fixed order: each half 8 -> 4 -> 2 -> 1,
// then the two halves.
NV_DEV float error_tree(const float (&e)[16]) {
  float c[2];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    float a0 = e[8 * h + 0] + e[8 * h + 4];
    float a1 = e[8 * h + 1] + e[8 * h + 5];
    float a2 = e[8 * h + 2] + e[8 * h + 6];
    float a3 = e[8 * h + 3] + e[8 * h + 7];
    float b0 = a0 + a2;
    float b1 = a1 + a3;
    c[h] = b0 + b1;
  }
  return c[0] + c[1];
}

// Quantize the block with scale (dec, enc): codes (element i in nibble i of
// lo for i < 8, of hi for i >= 8) and the block's squared error.
template <int ROUNDING>
NV_DEV float candidate(const float (&v)[16], const float (&u)[16], float dec, float enc,
                       uint32_t &lo, uint32_t &hi) {
  float e[16];
  uint32_t c[2] = {0u, 0u};
#pragma unroll
  for (int i = 0; i < 16; i += 2) {
    float y0 = v[i] * enc, y1 = v[i + 1] * enc;
    float g0, g1;
    if (ROUNDING == kSR) {
      g0 = e2m1_sr_value(y0, u[i]);
      g1 = e2m1_sr_value(y1, u[i + 1]);
      c[i >> 3] |= (e2m1_code_of_grid_value(g0) | (e2m1_code_of_grid_value(g1) << 4))
                   << (4 * (i & 7));
    } else {
#if NVFP4_46_HW_FP4
      // v_cvt_scalef32_pk_fp4_f32 writes byte (i&7)/2 of the word: first source in
      // the low nibble; v_cvt_scalef32_pk_f32_fp4 reads the same byte back.
      c[i >> 3] = hw_pk_fp4_sel(c[i >> 3], y0, y1, (i & 7) >> 1);
      f32x2 g = hw_pk_f32_fp4_sel(c[i >> 3], (i & 7) >> 1);
      g0 = g.x;
      g1 = g.y;
#else
      float r0, r1;
      uint32_t k0 = e2m1_rtn_mag_sw(fminf(fabsf(y0), 6.0f), r0) | ((f2u(y0) >> 28) & 8u);
      uint32_t k1 = e2m1_rtn_mag_sw(fminf(fabsf(y1), 6.0f), r1) | ((f2u(y1) >> 28) & 8u);
      g0 = u2f(f2u(r0) | (f2u(y0) & 0x80000000u));
      g1 = u2f(f2u(r1) | (f2u(y1) & 0x80000000u));
      c[i >> 3] |= (k0 | (k1 << 4)) << (4 * (i & 7));
#endif
    }
    float D0 = g0 * dec, D1 = g1 * dec;
    float d0 = D0 - v[i], d1 = D1 - v[i + 1];
    e[i] = d0 * d0;
    e[i + 1] = d1 * d1;
  }
  lo = c[0];
  hi = c[1];
  return error_tree(e);
}

struct BlockResult {
  uint32_t lo, hi;   // 16 codes
  uint32_t scale;    // E4M3 byte
  uint32_t four;     // 1 if the block was scaled to 4
  float dec;         // value(scale) * alpha, for dequantizing the chosen codes
};

// The whole per-block procedure.  c6 = alpha*6 and c4 = alpha*4 are the
// denominators of Eq. (2).
template <int ROUNDING, int SELECT>
NV_DEV BlockResult quantize_block(const float (&v)[16], const float (&u)[16], float c6, float c4,
                                  const ScaleTable &tab) {
  float b = 0.0f;
#pragma unroll
  for (int i = 0; i < 16; i += 2) b = fmaxf(fmaxf(b, fabsf(v[i])), fabsf(v[i + 1]));

  BlockResult r6{}, r4{};
  float E6 = 0.0f, E4 = 0.0f;
  if (SELECT != kSelForce4) {
    r6.scale = e4m3_encode(b / c6);
    float2 t = tab.e[r6.scale];
    r6.dec = t.x;
    r6.four = 0u;
    E6 = candidate<ROUNDING>(v, u, t.x, t.y, r6.lo, r6.hi);
  }
  if (SELECT != kSelForce6) {
    r4.scale = e4m3_encode(b / c4);
    float2 t = tab.e[r4.scale];
    r4.dec = t.x;
    r4.four = 1u;
    E4 = candidate<ROUNDING>(v, u, t.x, t.y, r4.lo, r4.hi);
  }
  if (SELECT == kSelForce6) return r6;
  if (SELECT == kSelForce4) return r4;
  return (E4 < E6) ? r4 : r6;   // strict: ties keep 6 (Table 3 line 13)
}

// Dequantized fp32 values of 8 codes packed in one word: value(code) * dec.
NV_DEV void dequant8(uint32_t codes, float dec, float (&D)[8]) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
#if NVFP4_46_HW_FP4
    f32x2 g = hw_pk_f32_fp4_sel(codes, j);
    D[2 * j] = g.x * dec;
    D[2 * j + 1] = g.y * dec;
#else
    D[2 * j] = e2m1_decode_sw((codes >> (8 * j)) & 15u) * dec;
    D[2 * j + 1] = e2m1_decode_sw((codes >> (8 * j + 4)) & 15u) * dec;
#endif
  }
}

}  // namespace nvfp4_46
