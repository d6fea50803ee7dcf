// Test infrastructure: the kernels' per-block code (csrc/block.hpp) compiled for the host and
// exported with a C interface.  See gfx950_on_host.hpp.
#include "gfx950_on_host.hpp"

#include "block.hpp"

using namespace nvfp4_46;

namespace {

int g_second_passes = 0;   // blocks that the estimates could not decide

// a uniform k * 2^-24 as the random word whose top 24 bits are k (the low byte, which nothing
// may depend on, is filled with a pattern)
uint32_t word_of(float u) { return ((uint32_t)(u * 0x1p24f) << 8) | 0xa5u; }

template <int ROUNDING>
BlockResult run_block(const float (&v)[16], const uint32_t (&u)[16], const ScaleConsts &k,
                      const ScaleTable &tab, int select) {
  // the kernels fetch the block again from memory; here it is simply copied
  auto again = [&](float (&w)[16], uint32_t (&uu)[16]) {
    ++g_second_passes;
    for (int i = 0; i < 16; ++i) {
      w[i] = v[i];
      uu[i] = u[i];
    }
  };
  switch (select) {
    case kSel46: return quantize_block<ROUNDING, kSel46>(v, u, k, tab, again);
    case kSelForce6: return quantize_block<ROUNDING, kSelForce6>(v, u, k, tab, again);
    case kSelForce4: return quantize_block<ROUNDING, kSelForce4>(v, u, k, tab, again);
    case kSel46Mae: return quantize_block<ROUNDING, kSel46Mae>(v, u, k, tab, again);
    default: return quantize_block<ROUNDING, kSel46AbsMax>(v, u, k, tab, again);
  }
}

// the sixteen row values of a tile combined as the kernel's XOR shuffles 4, 2, 1, 8 do
void over_tile(float (&e)[16], bool use_max) {
  const int order[4] = {4, 2, 1, 8};
  for (int s = 0; s < 4; ++s) {
    float n[16];
    for (int l = 0; l < 16; ++l) n[l] = use_max ? fmaxf(e[l], e[l ^ order[s]]) : e[l] + e[l ^ order[s]];
    for (int l = 0; l < 16; ++l) e[l] = n[l];
  }
}

}  // namespace

extern "C" {

int hm_second_passes() { return g_second_passes; }

// quantize_block<rounding, select> on `n` blocks of 16 values (u: the uniforms of stochastic
// rounding, ignored for round-to-nearest).  codes: 2 words per block.
void hm_quantize_blocks(const float *v, const float *u, int64_t n, float alpha, int rounding,
                        int select, uint32_t *codes, uint8_t *scale, uint8_t *four) {
  ScaleTable tab;
  const ScaleConsts k = build_scale_table(tab, alpha);
  for (int64_t b = 0; b < n; ++b) {
    float vv[16];
    uint32_t uu[16];
    for (int i = 0; i < 16; ++i) {
      vv[i] = v[16 * b + i];
      uu[i] = u ? word_of(u[16 * b + i]) : 0u;
    }
    const BlockResult r = rounding == kRTN  ? run_block<kRTN>(vv, uu, k, tab, select)
                          : rounding == kSR ? run_block<kSR>(vv, uu, k, tab, select)
                                            : run_block<kSRAfterRtnSelect>(vv, uu, k, tab, select);
    codes[2 * b] = r.lo;
    codes[2 * b + 1] = r.hi;
    scale[b] = (uint8_t)r.scale;
    four[b] = (uint8_t)r.four;
  }
}

// The squared-error decision of one 16x16 tile as k_block2d takes it (round to nearest or
// stochastic rounding of both candidates): v = 16 rows x 16 values.  Returns the choice;
// *took_defined_path = 1 when the estimates were too close and the defined errors decided.
int hm_tile_decision(const float *v, const float *u, float alpha, int rounding, uint8_t *scale6,
                     uint8_t *scale4, int *took_defined_path) {
  ScaleTable tab;
  const ScaleConsts sc = build_scale_table(tab, alpha);
  float b = 0.0f;
  for (int i = 0; i < 256; ++i) b = fmaxf(b, fabsf(v[i]));
  uint32_t S6, S4;
  block_scales(b, sc, S6, S4);
  *scale6 = (uint8_t)S6;
  *scale4 = (uint8_t)S4;
  const float4 t6 = tab.e[S6], t4 = tab.e[S4];
  float E6[16], E4[16], e6[16], e4[16];
  for (int r = 0; r < 16; ++r) {
    float vv[16];
    uint32_t uu[16];
    for (int i = 0; i < 16; ++i) {
      vv[i] = v[16 * r + i];
      uu[i] = u ? word_of(u[16 * r + i]) : 0u;
    }
    uint32_t lo6, hi6, lo4, hi4;
    if (rounding == kSR) {
      E6[r] = candidate<kSR, kErrMseEstimate>(vv, uu, t6.x, t6.y, lo6, hi6);
      E4[r] = candidate<kSR, kErrMseEstimate>(vv, uu, t4.x, t4.y, lo4, hi4);
    } else {
      E6[r] = candidate<kRTN, kErrMseEstimate>(vv, uu, t6.x, t6.y, lo6, hi6);
      E4[r] = candidate<kRTN, kErrMseEstimate>(vv, uu, t4.x, t4.y, lo4, hi4);
    }
    e6[r] = exact_error(vv, lo6, hi6, t6.x);
    e4[r] = exact_error(vv, lo4, hi4, t4.x);
  }
  over_tile(E6, false);
  over_tile(E4, false);
  const float tol = tile_decision_tolerance(t6.x, E6[0], t4.x, E4[0]);
  const float diff = E4[0] - E6[0];
  bool four = diff < 0.0f;
  *took_defined_path = 0;
  if (!(fabsf(diff) > tol)) {
    *took_defined_path = 1;
    over_tile(e6, false);
    over_tile(e4, false);
    four = e4[0] < e6[0];
  }
  return four ? 1 : 0;
}

// stochastic rounding of n (y, u) pairs by the two device routines: the rule in software, and
// the conversion instruction (code in bits 0-3, bit 7 = the kernels would not trust it)
void hm_e2m1_sr(const float *y, const float *u, int64_t n, uint8_t *out, uint8_t *out_fast) {
  for (int64_t i = 0; i < n; ++i) {
    const uint32_t w = word_of(u[i]);
    out[i] = (uint8_t)e2m1_code_of_grid_value(e2m1_sr_value(y[i], sr_uniform_of_word(w)));
    float margin = __builtin_inff();
    const uint32_t code = e2m1_sr_code_fast<0>(0u, y[i], ~w, (float)w, margin) & 0x0fu;
    out_fast[i] = (uint8_t)(code | (margin > kSrMarginAtRisk ? 0u : 0x80u));
  }
}

// the scale byte of Eq. (2) as the kernels compute it (multiply, guard, division): with
// pair != 0 both bytes at once as the 4/6 rules do (result = S6 | S4 << 8), else the one for M
int hm_block_scale(float b, float alpha, int M, int pair) {
  ScaleTable tab;
  const ScaleConsts k = build_scale_table(tab, alpha);
  if (pair) {
    uint32_t S6, S4;
    block_scales(b, k, S6, S4);
    return (int)(S6 | (S4 << 8));
  }
  const float q = b * (M == 6 ? k.rc6 : k.rc4);
  uint32_t S = e4m3_encode(q);
  if (scale_byte_at_risk(q)) S = e4m3_encode(b / (M == 6 ? k.c6 : k.c4));
  return (int)S;
}

void hm_philox(const uint32_t *ctr, uint32_t k0, uint32_t k1, uint32_t *out) {
  const Philox4 p = philox4x32_10(ctr[0], ctr[1], ctr[2], ctr[3], k0, k1);
  for (int j = 0; j < 4; ++j) out[j] = p.w[j];
}

void hm_rht16(float *v, uint32_t sign_word) {
  float a[16];
  for (int i = 0; i < 16; ++i) a[i] = v[i];
  rht16(a, sign_word);
  for (int i = 0; i < 16; ++i) v[i] = a[i];
}

}  // extern "C"
