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

// Per-tensor constants of Eq. (2): the denominators alpha*6 and alpha*4 and their
// reciprocals (each one IEEE operation).
struct ScaleConsts {
  float c6, c4, rc6, rc4;
};

// Fills the table (entry 127, which is no scale byte, carries the two reciprocals
// of ScaleConsts) and returns the constants.  Ends with a barrier.
NV_DEV ScaleConsts build_scale_table(ScaleTable &tab, float alpha) {
  ScaleConsts k;
  k.c6 = alpha * 6.0f;
  k.c4 = alpha * 4.0f;
  for (uint32_t s = threadIdx.x; s < 128u; s += blockDim.x) {
    if (s < 127u) {
      float dec = e4m3_decode_sw(s) * alpha;
      float enc = (dec == 0.0f) ? 0.0f : 1.0f / dec;
      tab.e[s] = make_float2(dec, enc);
    } else {
      tab.e[s] = make_float2(1.0f / k.c6, 1.0f / k.c4);
    }
  }
  __syncthreads();
  const float2 r = tab.e[127];
  k.rc6 = r.x;
  k.rc4 = r.y;
  return k;
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
  for (int h = 0; h < 2; ++h) {
    float g[8];
#if NVFP4_46_HW_FP4
    if (ROUNDING == kRTN) {
      // v_cvt_scalef32_pk_fp4_f32 fills byte j of the word (first source in the low
      // nibble); the word is complete before v_cvt_scalef32_pk_f32_fp4 reads the bytes
      // back, so no partial copies of it have to be kept.
      uint32_t w = 0u;
#pragma unroll
      for (int j = 0; j < 4; ++j)
        w = hw_pk_fp4_sel(w, v[8 * h + 2 * j] * enc, v[8 * h + 2 * j + 1] * enc, j);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        f32x2 p = hw_pk_f32_fp4_sel(w, j);
        g[2 * j] = p.x;
        g[2 * j + 1] = p.y;
      }
      c[h] = w;
    } else
#endif
    {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float y = v[8 * h + j] * enc;
        uint32_t k;
        if (ROUNDING == kSR) {
          g[j] = e2m1_sr_value(y, u[8 * h + j]);
          k = e2m1_code_of_grid_value(g[j]);
        } else {
          float r;
          k = e2m1_rtn_mag_sw(fminf(fabsf(y), 6.0f), r) | ((f2u(y) >> 28) & 8u);
          g[j] = u2f(f2u(r) | (f2u(y) & 0x80000000u));
        }
        c[h] |= k << (4 * j);
      }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float D = g[j] * dec;
      const float d = D - v[8 * h + j];
      e[8 * h + j] = d * d;
    }
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

// True when the E4M3 byte of q = fl(b * fl(1/c)) might differ from the byte of the
// correctly rounded quotient fl(b / c).  q is within 3.01 * 2^-24 (relative) of that
// quotient, and the byte is a monotone step function of its argument, so the two can
// differ only if a rounding boundary lies within about 3 ulp of q:
//   - in the normal E4M3 range the boundaries are the fp32 values whose low 20
//     mantissa bits are 0x80000; anything within 16 ulp of one is reported;
//   - in the subnormal E4M3 range (below 2^-6) the boundaries have no fixed bit
//     position, so every q in [2^-12, 2^-6) is reported; below 2^-11 both round to 0.
// Values from 448 up all saturate to the same byte, so false alarms there are harmless.
NV_DEV bool scale_byte_at_risk(float q) {
  const uint32_t bits = f2u(q);
  const bool near_midpoint = ((bits & 0xfffffu) - 0x7fff0u) <= 32u;
  const bool subnormal_range = (bits - 0x39800000u) < (0x3c800000u - 0x39800000u);
  return near_midpoint | subnormal_range;
}

// The whole per-block procedure (Table 3 lines 1-14).
template <int ROUNDING, int SELECT>
NV_DEV BlockResult quantize_block(const float (&v)[16], const float (&u)[16],
                                  const ScaleConsts &k, const ScaleTable &tab) {
  float b = 0.0f;
#pragma unroll
  for (int i = 0; i < 16; i += 2) b = fmaxf(fmaxf(b, fabsf(v[i])), fabsf(v[i + 1]));

  // Eq. (2): S_M = e4m3(b / (alpha*M)).  The quotient is first approximated by one
  // multiplication; the exact division runs only for the rare block whose byte could
  // depend on the difference (so the result is always that of the division).
  uint32_t S6 = 0u, S4 = 0u;
  const float q6 = b * k.rc6, q4 = b * k.rc4;
  bool risk = false;
  if (SELECT != kSelForce4) {
    S6 = e4m3_encode(q6);
    risk |= scale_byte_at_risk(q6);
  }
  if (SELECT != kSelForce6) {
    S4 = e4m3_encode(q4);
    risk |= scale_byte_at_risk(q4);
  }
  if (risk) {
    if (SELECT != kSelForce4) S6 = e4m3_encode(b / k.c6);
    if (SELECT != kSelForce6) S4 = e4m3_encode(b / k.c4);
  }

  BlockResult r6{}, r4{};
  float E6 = 0.0f, E4 = 0.0f;
  if (SELECT != kSelForce4) {
    float2 t = tab.e[S6];
    r6.scale = S6;
    r6.dec = t.x;
    r6.four = 0u;
    E6 = candidate<ROUNDING>(v, u, t.x, t.y, r6.lo, r6.hi);
  }
  if (SELECT != kSelForce6) {
    float2 t = tab.e[S4];
    r4.scale = S4;
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
