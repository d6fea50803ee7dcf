// One-lane-per-block 4/6 quantization of 16 fp32 values held in registers
// (arXiv 2512.02010, Table 3 lines 1-14, with the tensor scale of Eq. (1)-(3)).
#pragma once

#include "codec.hpp"

namespace nvfp4_46 {

enum : int { kRTN = 0, kSR = 1, kSRAfterRtnSelect = 2 };
enum : int { kSel46 = 0, kSelForce6 = 1, kSelForce4 = 2, kSel46Mae = 3, kSel46AbsMax = 4 };
// what candidate() returns besides the codes
enum : int { kErrNone = 0, kErrMseEstimate = 1, kErrMae = 2, kErrAbsMax = 3 };

// (dec, enc, dec^2) for every E4M3 scale byte under one tensor scale:
//   dec = value(S) * alpha   -- what one unit of code is worth (Table 3 line 5)
//   enc = 1 / dec            -- multiplying by it is the division of Eq. (3);
//                               0 when dec is 0, so an all-zero block encodes to zeros
//   dec^2                    -- for the tolerance of the 4-vs-6 decision
// All depend on (S, alpha) only, so a workgroup computes the 127 entries once
// into LDS instead of one IEEE division per block and candidate.
struct ScaleTable {
  float4 e[128];   // .x dec, .y enc, .z dec * dec
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
      float dec = e4m3_decode(s) * alpha;
      float enc = (dec == 0.0f) ? 0.0f : 1.0f / dec;
      tab.e[s] = make_float4(dec, enc, dec * dec, 0.0f);
    } else {
      tab.e[s] = make_float4(1.0f / k.c6, 1.0f / k.c4, 0.0f, 0.0f);
    }
  }
  __syncthreads();
  const float4 r = tab.e[127];
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
// byte `sel` of a word that is filled in the order 0, 1, 2, 3
NV_DEV uint32_t e2m1_sr_code_fast_sel(uint32_t old, float y, uint32_t not_w, float wf, float &margin,
                                      int sel) {
  switch (sel) {
    case 0: return e2m1_sr_code_fast<kSrFirstByteOfNewWord>(old, y, not_w, wf, margin);
    case 1: return e2m1_sr_code_fast<1>(old, y, not_w, wf, margin);
    case 2: return e2m1_sr_code_fast<2>(old, y, not_w, wf, margin);
    default: return e2m1_sr_code_fast<3>(old, y, not_w, wf, margin);
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

// Grid values (sign included) of 8 codes packed in one word.
NV_DEV void grid8(uint32_t codes, float (&g)[8]) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    f32x2 p = hw_pk_f32_fp4_sel(codes, j);
    g[2 * j] = p.x;
    g[2 * j + 1] = p.y;
  }
}

// Quantize the block with scale (dec, enc): codes (element i in nibble i of lo for
// i < 8, of hi for i >= 8).  Also returns a cheap estimate E' of the block's squared
// error: d' = fma(g, dec, -v) and a running fma(d', d', E'), i.e. two instructions per
// element where the defining sequence (product, difference, square, tree sum, each
// rounded) takes four.  E' is only ever used through decide_from_estimates() below.
// Stochastic rounding (not_w, wf: the complement of each element's random word, and the word
// rounded to a float) comes in two forms: FAST_SR = true rounds with the conversion
// instruction and lowers `sr_margin` (see e2m1_sr_code_fast: the codes are only valid if
// sr_margin stays above kSrMarginAtRisk); FAST_SR = false applies the rule in software and is
// always valid.
template <int ROUNDING, int ERR, bool FAST_SR>
NV_DEV float candidate_as(const float (&v)[16], const uint32_t (&not_w)[16], const float (&wf)[16],
                          float dec, float enc, uint32_t &lo, uint32_t &hi, float &sr_margin) {
  uint32_t c[2] = {0u, 0u};
  float acc[2] = {0.0f, 0.0f};
  f32x2 sq = {0.0f, 0.0f};
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    float g[8];
    if (ROUNDING == kRTN) {
      // v_cvt_scalef32_pk_fp4_f32 fills byte j of the word (first source in the low
      // nibble); the word is complete before v_cvt_scalef32_pk_f32_fp4 reads the bytes
      // back, so no partial copies of it have to be kept.
      uint32_t w = any_register();   // all four bytes are written below
#pragma unroll
      for (int j = 0; j < 4; ++j)
        w = hw_pk_fp4_sel(w, v[8 * h + 2 * j] * enc, v[8 * h + 2 * j + 1] * enc, j);
      if (ERR != kErrNone) grid8(w, g);
      c[h] = w;
    } else if (FAST_SR) {
      // one conversion per element (only the first source position rounds as defined):
      // even elements into the bytes of one word, odd ones into another
      uint32_t we = 0u, wo = 0u;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int e = 8 * h + 2 * j, o = e + 1;
        we = e2m1_sr_code_fast_sel(we, v[e] * enc, not_w[e], wf[e], sr_margin, j);
        wo = e2m1_sr_code_fast_sel(wo, v[o] * enc, not_w[o], wf[o], sr_margin, j);
      }
      const uint32_t w = (we & 0x0f0f0f0fu) | ((wo << 4) & 0xf0f0f0f0u);
      if (ERR != kErrNone) grid8(w, g);
      c[h] = w;
    } else {
      // the rounded values are on the grid, so the conversion that packs them is exact
#pragma unroll
      for (int j = 0; j < 8; ++j)
        g[j] = e2m1_sr_value(v[8 * h + j] * enc, sr_uniform_of_word(~not_w[8 * h + j]));
      uint32_t w = 0u;
#pragma unroll
      for (int j = 0; j < 4; ++j) w = hw_pk_fp4_sel(w, g[2 * j], g[2 * j + 1], j);
      c[h] = w;
    }
    if (ERR == kErrMseEstimate) {
      // A three-source instruction issues at half rate when all three sources sit in registers
      // of the same parity (measured), which d * d + acc is whenever d and acc do.  The two
      // differences of a pair of elements are therefore kept in an aligned register pair (even,
      // odd) and each is added into the accumulator of the other parity.
#pragma unroll
      for (int j = 0; j < 8; j += 2) {
        f32x2 d = {__builtin_fmaf(g[j], dec, -v[8 * h + j]), __builtin_fmaf(g[j + 1], dec, -v[8 * h + j + 1])};
        in_register_pair(d);
        sq.y = __builtin_fmaf(d.x, d.x, sq.y);
        sq.x = __builtin_fmaf(d.y, d.y, sq.x);
        in_register_pair(sq);
      }
    }
    if (ERR == kErrMae || ERR == kErrAbsMax) {
      // the other two rules of Section 3.1 are cheap enough to evaluate as defined:
      // D = fl(g*dec), d = fl(D - v), then the fixed-order sum of |d| or the largest |d|
      float e[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float D = g[j] * dec;
        e[j] = fabsf(D - v[8 * h + j]);
      }
      if (ERR == kErrMae) {
        acc[h] = ((e[0] + e[4]) + (e[2] + e[6])) + ((e[1] + e[5]) + (e[3] + e[7]));
      } else {
        acc[h] = fmaxf(fmaxf(fmaxf(e[0], e[1]), fmaxf(e[2], e[3])),
                       fmaxf(fmaxf(e[4], e[5]), fmaxf(e[6], e[7])));
      }
    }
  }
  lo = c[0];
  hi = c[1];
  if (ERR == kErrMseEstimate) return sq.x + sq.y;
  return ERR == kErrAbsMax ? fmaxf(acc[0], acc[1]) : acc[0] + acc[1];
}

// The candidate as the kernels use it: stochastic rounding by the conversion instruction,
// redone in software for the rare block in which an element came too close to the one case
// where the instruction's answer may differ.
template <int ROUNDING, int ERR>
NV_DEV float candidate(const float (&v)[16], const uint32_t (&rw)[16], float dec, float enc,
                       uint32_t &lo, uint32_t &hi) {
  // (the same for every scale the block is tried under: computed once after inlining, and
  // the words themselves need not stay in registers)
  uint32_t not_w[16];
  float wf[16];
  if (ROUNDING != kRTN) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      not_w[i] = ~rw[i];
      wf[i] = (float)rw[i];
    }
  }
  float margin = __builtin_inff();
  float E = candidate_as<ROUNDING, ERR, true>(v, not_w, wf, dec, enc, lo, hi, margin);
  if (ROUNDING != kRTN && !(margin > kSrMarginAtRisk))
    E = candidate_as<ROUNDING, ERR, false>(v, not_w, wf, dec, enc, lo, hi, margin);
  return E;
}

// The block's squared error exactly as it is defined (Table 3 lines 5-6 / 11-12 in fp32):
// D = fl(g*dec), d = fl(D - v), e = fl(d*d), fixed summation tree.
NV_DEV float exact_error(const float (&v)[16], uint32_t lo, uint32_t hi, float dec) {
  float e[16];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    float g[8];
    grid8(h ? hi : lo, g);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float D = g[j] * dec;
      const float d = D - v[8 * h + j];
      e[8 * h + j] = d * d;
    }
  }
  return error_tree(e);
}

// Table 3 line 13: is the defined error of the M=4 candidate strictly smaller than that
// of the M=6 candidate?  Decided from the estimates whenever they differ by more than
// they can be off, otherwise from the defined errors themselves, so the answer is always
// the defined one.
//
// Bound used (u = 2^-24, S = sum of the exact real squares t_i^2, t_i = g_i*dec - v_i,
// |g_i| <= 6, m = max(dec^2, S)), first for operations that do not underflow:
//   defined value E:  D_i carries a relative error u, d_i another, so d_i = t_i + eps_i
//     with |eps_i| <= u(6 dec + |t_i|)(1+u); squaring and summing 16 terms through a
//     4-level tree (and sum|t_i| <= 4 sqrt(S), dec sqrt(S) <= m) gives
//     |E - S| <= 48.1 u m + 7.1 u S;
//   estimate E':  one rounding in d', at most 9 more per term in the accumulation:
//     |E' - S| <= 18.1 u S.
// Hence |E - E'| <= 48.1 u m + 25.2 u S <= 48.1 u dec^2 + 73.3 u S < 64 u (dec^2 + 2 E').
// Underflow adds absolute errors that no relative bound covers: the contract keeps
// dec >= 2^-109, so products g*dec and the differences are never inexact for being small,
// but each of the 16 squares of the defined value and each of the 16 accumulation steps of
// the estimate may round in the subnormal range, by at most 2^-150 each: 2^-145 per
// candidate.  The tolerance therefore carries the absolute term 2^-126 (which also covers
// dec*dec or the tolerance's own products flushing towards zero):
//   tol := 64 u ((dec6^2 + dec4^2) + 2 (E6' + E4')) + 2^-126
// (the squares come out of the scale table; four instructions).
// If |E4' - E6'| > tol the order of E4 and E6 is the order of the estimates; tensors so
// small that all squared errors lie below 2^-126 always take the defined path.
// Overflowed (infinite / NaN) estimates fail the test and take the exact path.
NV_DEV float decision_tolerance(float m6, float E6p, float m4, float E4p) {
  return __builtin_fmaf(0x1p-18f, __builtin_fmaf(2.0f, E6p + E4p, m6 + m4), 0x1p-126f);
}

// The same for a 16x16 tile whose error is the sum of its sixteen row errors (each row an
// estimate as above, E6t and E4t their sums in the fixed order): each row estimate is within
// 2^-18 (max(dec^2, E'r) + E'r) + 2^-145 of the row's defined error, so the tile sums differ
// from the defined tile errors by less than 2^-18 (16 dec^2 + 2 E't) + 2^-141 plus the
// rounding of two 16-term trees (< 2^-20 E't).
NV_DEV float tile_decision_tolerance(float dec6, float E6t, float dec4, float E4t) {
  return __builtin_fmaf(0x1p-18f, (16.0f * dec6 * dec6 + 3.0f * E6t) + (16.0f * dec4 * dec4 + 3.0f * E4t),
                        0x1p-126f);
}

// Exact ties are common and must not pay for the exact path: a block whose maximum is an
// outlier quantizes every other element to zero under both scalings, and then the two
// candidates dequantize to the very same values.  same_dequantized() recognises the two
// ways this happens from the codes alone.
NV_DEV bool same_dequantized(uint32_t lo6, uint32_t hi6, uint32_t lo4, uint32_t hi4, float dec6,
                             float dec4) {
  // (a) the same scale byte: identical candidates
  const bool identical = (lo6 == lo4) & (hi6 == hi4) & (dec6 == dec4);
  // (b) every M=6 code in {0, 1.5, 3, 6} and the M=4 code the matching one of {0, 1, 2, 4}
  // (as 3-bit indices 0,3,5,7 -> 0,2,4,6: the M=4 nibble is the M=6 nibble with its low
  // bit cleared, and a nibble's low bit is set exactly when one of its two upper magnitude
  // bits is), and fl(1.5 * dec6) == dec4: then fl(1.5*2^k * dec6) = 2^k * fl(1.5 * dec6)
  // = fl(2^k * dec4) for every element, i.e. the rounded dequantized values coincide.
  const uint32_t ones = 0x11111111u;
  const bool scaled = 1.5f * dec6 == dec4;
  const bool lo_ok = (lo4 == (lo6 & ~ones)) & ((((lo6 >> 1) | (lo6 >> 2)) & ones) == (lo6 & ones));
  const bool hi_ok = (hi4 == (hi6 & ~ones)) & ((((hi6 >> 1) | (hi6 >> 2)) & ones) == (hi6 & ones));
  return identical | (scaled & lo_ok & hi_ok);
}

// Outcome of comparing the two estimates.
enum : int { kKeepSix = 0, kKeepFour = 1, kUndecided = 2 };

// kKeepFour / kKeepSix when the estimates (or the codes, for exact ties) settle Table 3
// line 13, kUndecided when only the defined errors can.
NV_DEV int decide_from_estimates(float E6p, float E4p, float dec6, float dec4, float dec6_squared,
                                 float dec4_squared, uint32_t lo6, uint32_t hi6, uint32_t lo4,
                                 uint32_t hi4) {
  const float tol = decision_tolerance(dec6_squared, E6p, dec4_squared, E4p);
  const float diff = E4p - E6p;
  if (fabsf(diff) > tol) return diff < 0.0f ? kKeepFour : kKeepSix;
  // identical dequantized values: equal errors, and ties keep 6
  return same_dequantized(lo6, hi6, lo4, hi4, dec6, dec4) ? kKeepSix : kUndecided;
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

// The same for the two quotients of one block, q4 = 1.5 q6 up to rounding: the subnormal
// range is tested once, on the union [2^-12 / 1.5, 2^-6) for q6 (a superset of both ranges:
// more false alarms on a sliver of values, never a missed one).
NV_DEV bool scale_bytes_at_risk(float q6, float q4) {
  const uint32_t b6 = f2u(q6), b4 = f2u(q4);
  const bool near_midpoint = (((b6 & 0xfffffu) - 0x7fff0u) <= 32u) | (((b4 & 0xfffffu) - 0x7fff0u) <= 32u);
  // q4 in [2^-12, 2^-6) implies q6 >= 2^-12 / 1.51 > 2^-13 and q6 < 2^-6; q6 in its own range too
  const bool subnormal_range = (b6 - 0x39000000u) < (0x3c800000u - 0x39000000u);
  return near_midpoint | subnormal_range;
}

// Eq. (2) for both candidates: S_M = e4m3(b / (alpha*M)).  The quotients are first
// approximated by one multiplication each and converted together; the exact divisions run
// only for the rare block whose bytes could depend on the difference (so the result is always
// that of the divisions).
NV_DEV void block_scales(float b, const ScaleConsts &k, uint32_t &S6, uint32_t &S4) {
  const float q6 = b * k.rc6, q4 = b * k.rc4;
  const uint32_t both = e4m3_encode2(q6, q4);
  S6 = both & 0xffu;
  S4 = both >> 8;
  if (scale_bytes_at_risk(q6, q4)) {
    S6 = e4m3_encode(b / k.c6);
    S4 = e4m3_encode(b / k.c4);
  }
}

// The per-block procedure (Table 3 lines 1-14) in one pass.  DEFINED_ERRORS = false: the
// squared-error rule compares the cheap estimates and reports through `undecided` when they
// cannot tell (the result is then provisional).  DEFINED_ERRORS = true: the errors are
// evaluated exactly as defined.  The other rules are always evaluated as defined.
template <int ROUNDING, int SELECT, bool DEFINED_ERRORS>
NV_DEV BlockResult quantize_block_pass(const float (&v)[16], const uint32_t (&rw)[16],
                                       const ScaleConsts &k, const ScaleTable &tab,
                                       bool &undecided) {
  float b = 0.0f;
#pragma unroll
  for (int i = 0; i < 16; i += 2) b = fmaxf(fmaxf(b, fabsf(v[i])), fabsf(v[i + 1]));

  uint32_t S6 = 0u, S4 = 0u;
  if (SELECT == kSelForce4 || SELECT == kSelForce6) {
    // one candidate only: the same multiply-then-guard for its scale alone
    const float c = SELECT == kSelForce4 ? k.c4 : k.c6, q = b * (SELECT == kSelForce4 ? k.rc4 : k.rc6);
    uint32_t S = e4m3_encode(q);
    if (scale_byte_at_risk(q)) S = e4m3_encode(b / c);
    (SELECT == kSelForce4 ? S4 : S6) = S;
  } else {
    block_scales(b, k, S6, S4);
  }

  constexpr int kErr = SELECT == kSel46 ? (DEFINED_ERRORS ? kErrNone : kErrMseEstimate)
                       : SELECT == kSel46Mae ? kErrMae
                       : SELECT == kSel46AbsMax ? kErrAbsMax : kErrNone;
  // Appendix A.3's second alternative compares round-to-nearest candidates and rounds
  // only the winner stochastically.
  constexpr int kCandRounding = ROUNDING == kSRAfterRtnSelect ? kRTN : ROUNDING;
  BlockResult r6{}, r4{};
  float E6p = 0.0f, E4p = 0.0f, enc6 = 0.0f, enc4 = 0.0f, m6 = 0.0f, m4 = 0.0f;
  if (SELECT != kSelForce4) {
    const float4 t = tab.e[S6];
    m6 = t.z;
    r6.scale = S6;
    r6.dec = t.x;
    r6.four = 0u;
    enc6 = t.y;
    if (!(ROUNDING == kSRAfterRtnSelect && SELECT == kSelForce6))
      E6p = candidate<kCandRounding, kErr>(v, rw, t.x, t.y, r6.lo, r6.hi);
  }
  if (SELECT != kSelForce6) {
    const float4 t = tab.e[S4];
    m4 = t.z;
    r4.scale = S4;
    r4.dec = t.x;
    r4.four = 1u;
    enc4 = t.y;
    if (!(ROUNDING == kSRAfterRtnSelect && SELECT == kSelForce4))
      E4p = candidate<kCandRounding, kErr>(v, rw, t.x, t.y, r4.lo, r4.hi);
  }
  bool four;
  if (SELECT == kSelForce6) {
    four = false;
  } else if (SELECT == kSelForce4) {
    four = true;
  } else if (SELECT == kSel46Mae || SELECT == kSel46AbsMax) {
    four = E4p < E6p;   // as defined
  } else if (DEFINED_ERRORS) {
    four = exact_error(v, r4.lo, r4.hi, r4.dec) < exact_error(v, r6.lo, r6.hi, r6.dec);
  } else {
    const int d = decide_from_estimates(E6p, E4p, r6.dec, r4.dec, m6, m4, r6.lo, r6.hi, r4.lo, r4.hi);
    four = d == kKeepFour;
    undecided = d == kUndecided;
  }
  BlockResult r = four ? r4 : r6;
  if (ROUNDING == kSRAfterRtnSelect)
    (void)candidate<kSR, kErrNone>(v, rw, r.dec, four ? enc4 : enc6, r.lo, r.hi);
  return r;
}

// The whole per-block procedure.  `again(w, ww)` must produce the block's values (and its
// stochastic-rounding words) once more: the rare block that the estimates cannot decide
// is redone from those with the defined errors, so that nothing of the first pass has to
// stay in registers for it -- keeping the sixteen values and both candidates alive across
// the common path cost the rowwise kernel three of its eight waves per SIMD.
template <int ROUNDING, int SELECT, typename Again>
NV_DEV BlockResult quantize_block(const float (&v)[16], const uint32_t (&rw)[16],
                                  const ScaleConsts &k, const ScaleTable &tab, Again &&again) {
  bool undecided = false;
  BlockResult r = quantize_block_pass<ROUNDING, SELECT, false>(v, rw, k, tab, undecided);
  if (SELECT == kSel46 && undecided) {
    float w[16];
    uint32_t ww[16];
    again(w, ww);
    r = quantize_block_pass<ROUNDING, SELECT, true>(w, ww, k, tab, undecided);
  }
  return r;
}

// Dequantized fp32 values of 8 codes packed in one word: value(code) * dec.
NV_DEV void dequant8(uint32_t codes, float dec, float (&D)[8]) {
  float g[8];
  grid8(codes, g);
#pragma unroll
  for (int j = 0; j < 8; ++j) D[j] = g[j] * dec;
}

}  // namespace nvfp4_46
