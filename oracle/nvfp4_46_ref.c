/*
 * CPU oracle for Four Over Six (4/6) NVFP4 quantization.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, scalar statement of
 * what the method computes, written from the paper's definitions so that a
 * reader can check it by eye.  It shares no code with the HIP library and is
 * used only by the tests, the smoke check and the benchmark's CPU-baseline leg.
 * The product path never calls it.
 *
 * Source of each step (arXiv 2512.02010):
 *   - formats: FP4 E2M1 grid +-{0,.5,1,1.5,2,3,4,6} (Section 1); FP8 E4M3 with
 *     largest value 448, one scale per 16 values, one FP32 tensor scale
 *     (Section 2.1);
 *   - tensor scale: Eq. (1), with 448 replaced by 256 for 4/6 (Section 3.1,
 *     last paragraph);
 *   - block scale: Eq. (2); E2M1 rounding: Eq. (3);
 *   - the 4/6 procedure (quantize with M=6 and M=4, dequantize, squared error,
 *     keep M=4 only if its error is strictly smaller): Table 3 lines 1-14 and
 *     Section 3.1;
 *   - the two alternative selection rules of Section 3.1 / Table 4 (mean absolute
 *     error, the rule Section 4.1 and Appendix A.1 recommend for pre-training, and
 *     largest absolute error);
 *   - stochastic rounding of gradients with selection on the rounded values
 *     ("biased selection"): Section 2.2, Section 4.1, Appendix A.3; and the
 *     appendix's second alternative, selection on round-to-nearest candidates
 *     followed by stochastic rounding with the selected scale;
 *   - 16-point random Hadamard transform: named in Section 2.2 / 4.1 / Fig. 3;
 *   - 2D (16x16) block quantization of weight matrices: named in Section 4.1.
 *
 * Where the paper fixes no detail (tie rules, operation order, overflow,
 * nibble order, the random-number construction, the Hadamard ordering) the
 * choice made here is marked READING.
 *
 * All arithmetic on values is IEEE binary32, one rounding per operation, no
 * fused multiply-add (compile with -ffp-contract=off, never -ffast-math).
 * Inputs must be finite.  The fp32 tensor scale must lie in [2^-100, 2^118]
 * (this keeps every reciprocal finite and non-zero); tensor_scale() itself
 * guarantees that for any tensor whose absolute maximum is at least 2^-89.
 *
 * parity pinned: every function here is pinned by tests/ (worked blocks of
 * Table 3, exact-rational rounding, brute force over all E4M3 scales,
 * published Philox known-answer vectors, dense-matrix Hadamard, invariants).
 * parity unpinned: the tensor-level MSE figures reported for the synthetic
 * workloads (the paper prints no such number); only their ordering is pinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define BLOCK 16

enum { REF_RTN = 0, REF_SR = 1, REF_SR_AFTER_RTN_SELECT = 2 };
enum { REF_SEL_46_MSE = 0, REF_SEL_FORCE6 = 1, REF_SEL_FORCE4 = 2, REF_SEL_46_MAE = 3,
       REF_SEL_46_ABSMAX = 4 };
enum { REF_ROWWISE = 1, REF_COLWISE = 2 };

/* ------------------------------------------------------------------ formats */

/* BF16 -> fp32 is exact: the 16 bits are the top half of the fp32 pattern. */
float ref_bf16_to_f32(uint16_t h) {
  uint32_t u = (uint32_t)h << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

/* fp32 -> BF16, round to nearest, ties to even; overflow goes to infinity.
 * READING (paper silent on the output cast of a dequantized value). */
uint16_t ref_f32_to_bf16(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u); /* NaN */
  uint32_t keep = u >> 16, rest = u & 0xffffu;
  if (rest > 0x8000u || (rest == 0x8000u && (keep & 1u))) keep += 1;
  return (uint16_t)keep;
}

/* E2M1 magnitudes by 3-bit index (Section 1). A code is sign<<3 | index. */
static const float E2M1_GRID[8] = {0.0f, 0.5f, 1.0f, 1.5f, 2.0f, 3.0f, 4.0f, 6.0f};

float ref_e2m1_decode(uint8_t code) {
  float m = E2M1_GRID[code & 7];
  return (code & 8) ? -m : m;
}

static uint8_t grid_index(float mag) {
  for (int k = 0; k < 8; ++k)
    if (E2M1_GRID[k] == mag) return (uint8_t)k;
  return 7; /* unreachable for values produced below */
}

/* Eq. (3): round a scaled value onto the E2M1 grid.  The three cases are
 * tested top-down; the integer rounding inside each is round-half-to-even
 * (READING: the paper's rounding brackets carry no tie rule; half-even makes
 * Eq. (3) identical to IEEE round-to-nearest-even onto E2M1).  Magnitudes
 * above 6 saturate to 6 (Table 3 line 4 rounds 6.15 to 6).  The sign bit is
 * the input's sign bit even when the magnitude rounds to zero (READING). */
uint8_t ref_e2m1_rtn(float y) {
  float a = fabsf(y);
  if (a > 6.0f) a = 6.0f;
  float r;
  if (a < 2.0f)
    r = 0.5f * rintf(2.0f * a);
  else if (a < 4.0f)
    r = rintf(a);
  else
    r = 2.0f * rintf(a / 2.0f);
  return (uint8_t)((signbit(y) ? 8 : 0) | grid_index(r));
}

/* Stochastic rounding onto the E2M1 grid (READING; the paper only names it).
 * lo <= |y| <= hi are adjacent grid points; a value already on the grid is
 * kept, otherwise it goes up with probability p = (|y|-lo)/(hi-lo), decided
 * as u < p for the supplied uniform u in [0,1). */
uint8_t ref_e2m1_sr(float y, float u) {
  float a = fabsf(y);
  if (a > 6.0f) a = 6.0f;
  int k = 0;
  while (k < 7 && E2M1_GRID[k + 1] <= a) ++k; /* grid[k] <= a < grid[k+1], or k == 7 */
  float lo = E2M1_GRID[k];
  if (a != lo) {
    float hi = E2M1_GRID[k + 1];
    float p = (a - lo) / (hi - lo); /* exact: numerator exact, denominator a power of two */
    if (u < p) ++k;
  }
  return (uint8_t)((signbit(y) ? 8 : 0) | k);
}

/* E4M3 ("FN" flavour: bias 7, no infinity, largest finite 448 = 0x7E,
 * subnormals m * 2^-9).  Section 2.1 gives the format and its maximum. */
float ref_e4m3_decode(uint8_t b) {
  int e = (b >> 3) & 15, m = b & 7;
  float v;
  if (e == 15 && m == 7)
    v = NAN;
  else if (e == 0)
    v = ldexpf((float)m, -9);
  else
    v = ldexpf((float)(8 + m), e - 10);
  return (b & 0x80) ? -v : v;
}

/* fp32 -> E4M3 for a non-negative scale: round to nearest even, and saturate
 * to 448 instead of overflowing (READING; Section 3.1 only says that 672
 * "would overflow").  Table 3 lines 2 and 8 give 6.67 -> 6.5 and 45 -> 44. */
uint8_t ref_e4m3_encode(float x) {
  if (!(x > 0.0f)) return 0;
  if (x >= 448.0f) return 0x7E;
  int e;
  (void)frexpf(x, &e);         /* x = f * 2^e with f in [0.5, 1) */
  int E = e - 1;               /* floor(log2 x) */
  if (E < -6) E = -6;          /* subnormal range shares the 2^-6 binade's quantum */
  float quantum = ldexpf(1.0f, E - 3);
  int n = (int)rintf(x / quantum); /* exact scaling, then half-even; n in [0, 16] */
  if (n == 0) return 0;
  if (n == 16) {               /* rounded up into the next binade */
    n = 8;
    E += 1;
  }
  if (n < 8) return (uint8_t)n;     /* subnormal (only possible when E == -6) */
  return (uint8_t)(((E + 7) << 3) | (n - 8));
}

/* --------------------------------------------------------- random numbers */

/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): 10 rounds of
 *   (c0,c1,c2,c3) <- (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1, lo(M0*c0))
 * with M0 = 0xD2511F53, M1 = 0xCD9E8D57, and the key bumped by
 * (0x9E3779B9, 0xBB67AE85) between rounds. */
void ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    uint32_t n1 = (uint32_t)p1;
    uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Uniform in [0,1) for the element with flat index g = row*cols + col of the
 * logical input (READING): word (g & 3) of Philox(key = seed, counter =
 * (g>>2, 0, 0)), top 24 bits scaled by 2^-24. */
float ref_sr_uniform(uint64_t seed, uint64_t g) {
  uint64_t q = g >> 2;
  uint32_t ctr[4] = {(uint32_t)q, (uint32_t)(q >> 32), 0u, 0u};
  uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  uint32_t w[4];
  ref_philox4x32_10(ctr, key, w);
  return (float)(w[g & 3] >> 8) * 0x1p-24f;
}

/* Sign word of the block at position B along the blocked axis (READING):
 * word 0 of Philox(key = seed, counter = (B, 0, 0, 1)); bit j set means
 * element j of the block is negated.  Every row (rowwise) or every column
 * (columnwise) uses the same word for the same B. */
uint32_t ref_rht_sign_word(uint64_t seed, uint64_t B) {
  uint32_t ctr[4] = {(uint32_t)B, (uint32_t)(B >> 32), 0u, 1u};
  uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  uint32_t w[4];
  ref_philox4x32_10(ctr, key, w);
  return w[0];
}

/* -------------------------------------------------------------- transform */

/* 16-point random Hadamard transform of one block, in place (READING: the
 * paper names the transform only).  v <- (1/4) * H16 * (s .* v) with H16 in
 * Sylvester order, H[i][j] = (-1)^popcount(i & j), evaluated as four
 * butterfly stages with strides 1, 2, 4, 8; every add/sub is one fp32
 * operation and the final scaling by 1/4 is exact. */
void ref_rht16(float v[BLOCK], uint32_t sign_word) {
  for (int j = 0; j < BLOCK; ++j)
    if ((sign_word >> j) & 1u) v[j] = -v[j];
  for (int h = 1; h < BLOCK; h <<= 1)
    for (int i = 0; i < BLOCK; ++i)
      if ((i & h) == 0) {
        float p = v[i], q = v[i + h];
        v[i] = p + q;
        v[i + h] = p - q;
      }
  for (int j = 0; j < BLOCK; ++j) v[j] *= 0.25f;
}

/* ------------------------------------------------------------ one block */

/* Sum of 16 squared errors in a fixed order (READING: the error is compared
 * in fp32 and the order of the additions must be stated for the comparison
 * to be reproducible).  Each half of the block is folded 8 -> 4 -> 2 -> 1,
 * then the two halves are added.  The 1/n of Table 3 lines 6 and 12 is the
 * same for both candidates and is left out. */
static float error_sum(const float e[BLOCK]) {
  float c[2];
  for (int half = 0; half < 2; ++half) {
    const float *p = e + 8 * half;
    float a[4], b[2];
    for (int j = 0; j < 4; ++j) a[j] = p[j] + p[j + 4];
    for (int j = 0; j < 2; ++j) b[j] = a[j] + a[j + 2];
    c[half] = b[0] + b[1];
  }
  return c[0] + c[1];
}

/* Quantize one block with a given E4M3 scale byte S under tensor scale alpha
 * (Table 3 lines 3-6 / 9-12, with the tensor scale of Eq. (1)-(3) put back):
 *   dec = value(S) * alpha                  -- what one unit of code is worth
 *   enc = 1 / dec (0 if dec is 0)           -- READING: Eq. (3) divides each
 *                                              element by alpha*Delta; one
 *                                              reciprocal and 16 products here
 *   y_i = v_i * enc;  q_i = e2m1(y_i)       -- RTN or SR
 *   D_i = grid(q_i) * dec  (signed)
 *   E   = sum_i (D_i - v_i)^2               -- fixed order, no FMA
 * Writes the 16 codes and the 16 dequantized values, returns E. */
float ref_block_with_scale(const float v[BLOCK], float alpha, uint8_t S, int rounding,
                           const float u[BLOCK], uint8_t q[BLOCK], float D[BLOCK]) {
  float dec = ref_e4m3_decode(S) * alpha;
  float enc = (dec == 0.0f) ? 0.0f : 1.0f / dec;
  float e[BLOCK];
  for (int i = 0; i < BLOCK; ++i) {
    float y = v[i] * enc;
    q[i] = (rounding == REF_SR) ? ref_e2m1_sr(y, u[i]) : ref_e2m1_rtn(y);
    D[i] = ref_e2m1_decode(q[i]) * dec;
    float d = D[i] - v[i];
    e[i] = d * d;
  }
  return error_sum(e);
}

/* The other two selection metrics of Section 3.1 (Table 4), from a candidate's
 * dequantized values: the sum of |D_i - v_i| (the mean without its common 1/n,
 * added in the same fixed order as the squared errors), or the largest
 * |D_i - v_i|.  READING: the paper prints the latter as max_i(Xbar_i - X_i),
 * without absolute value and on the codes; it is taken as max_i |D_i - X_i|. */
float ref_block_abs_metric(const float v[BLOCK], const float D[BLOCK], int select) {
  float e[BLOCK];
  for (int i = 0; i < BLOCK; ++i) e[i] = fabsf(D[i] - v[i]);
  if (select == REF_SEL_46_MAE) return error_sum(e);
  float m = 0.0f;
  for (int i = 0; i < BLOCK; ++i)
    if (e[i] > m) m = e[i];
  return m;
}

/* Eq. (2) for a block whose largest magnitude is b, mapped to M (6 or 4):
 * one fp32 product and one fp32 division, then the cast to E4M3. */
uint8_t ref_block_scale(float b, float alpha, float M) {
  float sf = b / (alpha * M);
  return ref_e4m3_encode(sf);
}

/* The 4/6 procedure on one block of 16 fp32 values (Table 3).  `select`
 * can force either candidate (standard NVFP4 is "always 6").  Outputs: the
 * chosen codes, scale byte and dequantized values, whether 4 was chosen, and
 * both candidates' errors under the rule in force (E[0] for M=6, E[1] for M=4;
 * squared error unless `select` names another metric; a forced mode fills only
 * its own). */
void ref_quantize_block(const float v[BLOCK], float alpha, int rounding, int select,
                        const float u[BLOCK], uint8_t q_out[BLOCK], float D_out[BLOCK],
                        uint8_t *S_out, uint8_t *four_out, float E[2]) {
  float b = 0.0f;
  for (int i = 0; i < BLOCK; ++i) {
    float a = fabsf(v[i]);
    if (a > b) b = a;
  }
  uint8_t q6[BLOCK], q4[BLOCK];
  float D6[BLOCK], D4[BLOCK];
  uint8_t S6 = 0, S4 = 0;
  E[0] = E[1] = 0.0f;
  /* Appendix A.3, second alternative: the candidates that are compared are rounded to
   * nearest, and only the winner is then rounded stochastically (below). */
  int cand_rounding = (rounding == REF_SR_AFTER_RTN_SELECT) ? REF_RTN : rounding;
  if (select != REF_SEL_FORCE4) {
    S6 = ref_block_scale(b, alpha, 6.0f);
    E[0] = ref_block_with_scale(v, alpha, S6, cand_rounding, u, q6, D6);
  }
  if (select != REF_SEL_FORCE6) {
    S4 = ref_block_scale(b, alpha, 4.0f);
    E[1] = ref_block_with_scale(v, alpha, S4, cand_rounding, u, q4, D4);
  }
  if (select == REF_SEL_46_MAE || select == REF_SEL_46_ABSMAX) {
    E[0] = ref_block_abs_metric(v, D6, select);
    E[1] = ref_block_abs_metric(v, D4, select);
  }
  int four;
  if (select == REF_SEL_FORCE6)
    four = 0;
  else if (select == REF_SEL_FORCE4)
    four = 1;
  else
    four = (E[1] < E[0]); /* Table 3 line 13: strict, so ties keep 6 */
  memcpy(q_out, four ? q4 : q6, BLOCK);
  memcpy(D_out, four ? D4 : D6, BLOCK * sizeof(float));
  *S_out = four ? S4 : S6;
  *four_out = (uint8_t)four;
  if (rounding == REF_SR_AFTER_RTN_SELECT)
    (void)ref_block_with_scale(v, alpha, *S_out, REF_SR, u, q_out, D_out);
}

/* ---------------------------------------------------------- whole tensors */

/* The input tensor: BF16 bit patterns (activations, gradients, and weights held in
 * BF16) or fp32 values (the master weights of Fig. 3, which enter the quantizer without a
 * BF16 rounding in between).  Either way the method's arithmetic starts from the fp32
 * value of each element. */
typedef struct {
  const void *p;
  int f32;
  int64_t row0; /* the tensor handed in is rows row0.. of a taller one (0: it is the whole) */
} xin;
static float x_at(xin x, uint64_t g) {
  return x.f32 ? ((const float *)x.p)[g] : ref_bf16_to_f32(((const uint16_t *)x.p)[g]);
}
static xin x_bf16(const uint16_t *p) {
  xin x = {p, 0, 0};
  return x;
}
static xin x_f32(const float *p) {
  xin x = {p, 1, 0};
  return x;
}

/* Fetch the block with index (line, blk) along the blocked axis as fp32:
 * rowwise -> row `line`, columns 16*blk..; columnwise -> column `line`,
 * rows 16*blk.. (i.e. the rowwise block of the transposed tensor, which is
 * how Fig. 3 feeds the DGRAD/WGRAD operands).  Applies the Hadamard
 * transform when asked.  Also returns each element's flat index. */
static void fetch_block(xin x, int64_t rows, int64_t cols, int layout, int64_t line,
                        int64_t blk, int rht, uint64_t rht_seed, float v[BLOCK],
                        uint64_t g[BLOCK]) {
  (void)rows;
  for (int i = 0; i < BLOCK; ++i) {
    int64_t r = (layout == REF_ROWWISE) ? line : blk * BLOCK + i;
    int64_t c = (layout == REF_ROWWISE) ? blk * BLOCK + i : line;
    g[i] = (uint64_t)r * (uint64_t)cols + (uint64_t)c;
    v[i] = x_at(x, g[i]);
  }
  /* the sign vector belongs to the block's position along the blocked axis of the whole
   * tensor */
  if (rht)
    ref_rht16(v, ref_rht_sign_word(rht_seed, (uint64_t)(blk + (layout == REF_ROWWISE
                                                                   ? 0
                                                                   : x.row0 / BLOCK))));
}

static int64_t n_lines(int64_t rows, int64_t cols, int layout) {
  return layout == REF_ROWWISE ? rows : cols;
}
static int64_t n_blocks(int64_t rows, int64_t cols, int layout) {
  return (layout == REF_ROWWISE ? cols : rows) / BLOCK;
}

/* Eq. (1): alpha = max|X| / (6 * fp8_max), fp8_max = 256 for 4/6 (Section
 * 3.1) or 448 for standard NVFP4.  The maximum runs over the values that get
 * quantized, i.e. after the Hadamard transform when it is on (READING).  One
 * fp32 division by the exactly representable constant.  An all-zero tensor
 * gets alpha = 1 (READING; Eq. (2) would divide by zero). */
static int tensor_scale_impl(xin x, int64_t rows, int64_t cols, int layout, int rht,
                             uint64_t rht_seed, float fp8_max, float *alpha) {
  int64_t L = n_lines(rows, cols, layout), NB = n_blocks(rows, cols, layout);
  float amax = 0.0f;
#pragma omp parallel for reduction(max : amax) schedule(static)
  for (int64_t line = 0; line < L; ++line)
    for (int64_t blk = 0; blk < NB; ++blk) {
      float v[BLOCK];
      uint64_t g[BLOCK];
      fetch_block(x, rows, cols, layout, line, blk, rht, rht_seed, v, g);
      for (int i = 0; i < BLOCK; ++i) {
        float a = fabsf(v[i]);
        if (a > amax) amax = a;
      }
    }
  *alpha = (amax == 0.0f) ? 1.0f : amax / (6.0f * fp8_max);
  return 0;
}
int nvfp4_46_ref_tensor_scale(const uint16_t *x, int64_t rows, int64_t cols, int layout, int rht,
                              uint64_t rht_seed, float fp8_max, float *alpha) {
  return tensor_scale_impl(x_bf16(x), rows, cols, layout, rht, rht_seed, fp8_max, alpha);
}
int nvfp4_46_ref_tensor_scale_f32(const float *x, int64_t rows, int64_t cols, int layout, int rht,
                                  uint64_t rht_seed, float fp8_max, float *alpha) {
  return tensor_scale_impl(x_f32(x), rows, cols, layout, rht, rht_seed, fp8_max, alpha);
}

/* Quantize a [rows][cols] BF16 tensor in one orientation.
 * Outputs, indexed by (line, position along the blocked axis):
 *   codes  [lines][len/2]  two codes per byte, even position in the low
 *                          nibble (READING)
 *   scales [lines][len/16] one E4M3 byte per block, plain row-major
 *   choice [lines][len/16] 1 if the block was scaled to 4, else 0 (optional)
 *   deq    [rows][cols]    BF16 of the chosen candidate's dequantized values,
 *                          always in the input's own row-major order (optional)
 * Only rows are distributed over threads; each block is independent. */
static int quantize_impl(xin x, int64_t rows, int64_t cols, int layout, int rounding,
                         int select, int rht, uint64_t sr_seed, uint64_t rht_seed, float alpha,
                         uint8_t *codes, uint8_t *scales, uint8_t *choice, uint16_t *deq) {
  int64_t L = n_lines(rows, cols, layout), NB = n_blocks(rows, cols, layout);
#pragma omp parallel for schedule(static)
  for (int64_t line = 0; line < L; ++line)
    for (int64_t blk = 0; blk < NB; ++blk) {
      float v[BLOCK], u[BLOCK], D[BLOCK], E[2];
      uint64_t g[BLOCK];
      uint8_t q[BLOCK], S, four;
      fetch_block(x, rows, cols, layout, line, blk, rht, rht_seed, v, g);
      /* the uniform belongs to the element's flat index in the whole tensor */
      for (int i = 0; i < BLOCK; ++i)
        u[i] = (rounding != REF_RTN)
                   ? ref_sr_uniform(sr_seed, g[i] + (uint64_t)x.row0 * (uint64_t)cols)
                   : 0.0f;
      ref_quantize_block(v, alpha, rounding, select, u, q, D, &S, &four, E);
      if (codes)
        for (int i = 0; i < BLOCK; i += 2)
          codes[(line * NB + blk) * (BLOCK / 2) + i / 2] = (uint8_t)(q[i] | (q[i + 1] << 4));
      if (scales) scales[line * NB + blk] = S;
      if (choice) choice[line * NB + blk] = four;
      if (deq)
        for (int i = 0; i < BLOCK; ++i) deq[g[i]] = ref_f32_to_bf16(D[i]);
    }
  return 0;
}
int nvfp4_46_ref_quantize(const uint16_t *x, int64_t rows, int64_t cols, int layout, int rounding,
                          int select, int rht, uint64_t sr_seed, uint64_t rht_seed, float alpha,
                          uint8_t *codes, uint8_t *scales, uint8_t *choice, uint16_t *deq) {
  return quantize_impl(x_bf16(x), rows, cols, layout, rounding, select, rht, sr_seed, rht_seed,
                       alpha, codes, scales, choice, deq);
}
/* Rows row0 .. row0 + rows - 1 of a taller [.][cols] BF16 tensor, handed in on their own:
 * the result is that slice of the whole tensor's quantization (random numbers and sign
 * vectors are keyed by positions in the whole tensor).  row0 must be a multiple of 16.
 * Lets a test check a tensor of billions of elements a few rows at a time. */
int nvfp4_46_ref_quantize_rows(const uint16_t *x, int64_t rows, int64_t cols, int64_t row0,
                               int layout, int rounding, int select, int rht, uint64_t sr_seed,
                               uint64_t rht_seed, float alpha, uint8_t *codes, uint8_t *scales,
                               uint8_t *choice, uint16_t *deq) {
  xin xi = x_bf16(x);
  xi.row0 = row0;
  return quantize_impl(xi, rows, cols, layout, rounding, select, rht, sr_seed, rht_seed, alpha,
                       codes, scales, choice, deq);
}
/* The same for an fp32 tensor (FP32 master weights, Fig. 3). */
int nvfp4_46_ref_quantize_f32(const float *x, int64_t rows, int64_t cols, int layout,
                              int rounding, int select, int rht, uint64_t sr_seed,
                              uint64_t rht_seed, float alpha, uint8_t *codes, uint8_t *scales,
                              uint8_t *choice, uint16_t *deq) {
  return quantize_impl(x_f32(x), rows, cols, layout, rounding, select, rht, sr_seed, rht_seed,
                       alpha, codes, scales, choice, deq);
}

/* 2D block quantization of weight matrices (named in Section 4.1 as part of the
 * training recipe; READING throughout): one E4M3 scale per 16x16 tile instead of one per
 * 16 values of a row, so that a matrix and its transpose are quantized consistently.  The
 * tile is treated as sixteen row blocks that share their scale:
 *   b      = largest magnitude of the 256 values;  S_M = e4m3(b / (alpha*M))   (Eq. 2)
 *   each row of the tile is quantized with S_M exactly as a 1x16 block is (Eq. 3)
 *   E_M    = the sixteen row errors added in the same fixed order in which a row adds
 *            its sixteen element errors (for the largest-absolute-error rule: their
 *            maximum)
 *   keep M = 4 iff E_4 < E_6.
 * Outputs: codes [rows][cols/2] packed along rows as in the rowwise layout, scales and
 * choice [rows/16][cols/16], deq [rows][cols] (each optional).  With
 * REF_SR_AFTER_RTN_SELECT the tile is chosen from round-to-nearest candidates and then
 * rounded stochastically; uniforms are those of the elements' flat indices. */
static int quantize_2d_impl(xin x, int64_t rows, int64_t cols, int rounding,
                            int select, uint64_t sr_seed, float alpha, uint8_t *codes,
                            uint8_t *scales, uint8_t *choice, uint16_t *deq) {
  int64_t TR = rows / BLOCK, TCB = cols / BLOCK;
#pragma omp parallel for schedule(static)
  for (int64_t tr = 0; tr < TR; ++tr)
    for (int64_t tc = 0; tc < TCB; ++tc) {
      float v[BLOCK][BLOCK], u[BLOCK][BLOCK];
      float b = 0.0f;
      for (int r = 0; r < BLOCK; ++r)
        for (int c = 0; c < BLOCK; ++c) {
          uint64_t g = (uint64_t)(tr * BLOCK + r) * (uint64_t)cols + (uint64_t)(tc * BLOCK + c);
          v[r][c] = x_at(x, g);
          u[r][c] = (rounding != REF_RTN) ? ref_sr_uniform(sr_seed, g) : 0.0f;
          float a = fabsf(v[r][c]);
          if (a > b) b = a;
        }
      int cand_rounding = (rounding == REF_SR_AFTER_RTN_SELECT) ? REF_RTN : rounding;
      uint8_t S[2] = {0, 0}, q[2][BLOCK][BLOCK];
      float D[2][BLOCK][BLOCK], E[2] = {0.0f, 0.0f};
      for (int m = 0; m < 2; ++m) {
        if ((m == 0 && select == REF_SEL_FORCE4) || (m == 1 && select == REF_SEL_FORCE6)) continue;
        S[m] = ref_block_scale(b, alpha, m == 0 ? 6.0f : 4.0f);
        float rowerr[BLOCK];
        for (int r = 0; r < BLOCK; ++r) {
          rowerr[r] = ref_block_with_scale(v[r], alpha, S[m], cand_rounding, u[r], q[m][r], D[m][r]);
          if (select == REF_SEL_46_MAE || select == REF_SEL_46_ABSMAX)
            rowerr[r] = ref_block_abs_metric(v[r], D[m][r], select);
        }
        if (select == REF_SEL_46_ABSMAX) {
          E[m] = 0.0f;
          for (int r = 0; r < BLOCK; ++r)
            if (rowerr[r] > E[m]) E[m] = rowerr[r];
        } else {
          E[m] = error_sum(rowerr);
        }
      }
      int four = (select == REF_SEL_FORCE6) ? 0 : (select == REF_SEL_FORCE4) ? 1 : (E[1] < E[0]);
      if (rounding == REF_SR_AFTER_RTN_SELECT)
        for (int r = 0; r < BLOCK; ++r)
          (void)ref_block_with_scale(v[r], alpha, S[four], REF_SR, u[r], q[four][r], D[four][r]);
      if (scales) scales[tr * TCB + tc] = S[four];
      if (choice) choice[tr * TCB + tc] = (uint8_t)four;
      for (int r = 0; r < BLOCK; ++r) {
        int64_t row = tr * BLOCK + r;
        if (codes)
          for (int c = 0; c < BLOCK; c += 2)
            codes[row * (cols / 2) + tc * (BLOCK / 2) + c / 2] =
                (uint8_t)(q[four][r][c] | (q[four][r][c + 1] << 4));
        if (deq)
          for (int c = 0; c < BLOCK; ++c)
            deq[row * cols + tc * BLOCK + c] = ref_f32_to_bf16(D[four][r][c]);
      }
    }
  return 0;
}

int nvfp4_46_ref_quantize_2d(const uint16_t *x, int64_t rows, int64_t cols, int rounding,
                             int select, uint64_t sr_seed, float alpha, uint8_t *codes,
                             uint8_t *scales, uint8_t *choice, uint16_t *deq) {
  return quantize_2d_impl(x_bf16(x), rows, cols, rounding, select, sr_seed, alpha, codes, scales,
                          choice, deq);
}
int nvfp4_46_ref_quantize_2d_f32(const float *x, int64_t rows, int64_t cols, int rounding,
                                 int select, uint64_t sr_seed, float alpha, uint8_t *codes,
                                 uint8_t *scales, uint8_t *choice, uint16_t *deq) {
  return quantize_2d_impl(x_f32(x), rows, cols, rounding, select, sr_seed, alpha, codes, scales,
                          choice, deq);
}

/* The same 2D-block quantization laid out for the transposed matrix (READING: "a matrix and
 * its transpose are quantized consistently" is taken literally -- the tiles are decided once,
 * in the matrix's own orientation, and W^T gets the very same codes and scales, only packed
 * along its own rows): codes_col [cols][rows/2] with the element at the even ROW in the low
 * nibble, scales_col and choice_col [cols/16][rows/16].  Pure re-indexing. */
int nvfp4_46_ref_repack_2d_columnwise(const uint8_t *codes, const uint8_t *scales,
                                      const uint8_t *choice, int64_t rows, int64_t cols,
                                      uint8_t *codes_col, uint8_t *scales_col,
                                      uint8_t *choice_col) {
  int64_t TR = rows / BLOCK, TCB = cols / BLOCK;
  for (int64_t c = 0; c < cols; ++c)
    for (int64_t r = 0; r < rows; r += 2) {
      uint8_t b0 = codes[r * (cols / 2) + c / 2], b1 = codes[(r + 1) * (cols / 2) + c / 2];
      uint8_t q0 = (c & 1) ? (b0 >> 4) : (b0 & 15), q1 = (c & 1) ? (b1 >> 4) : (b1 & 15);
      codes_col[c * (rows / 2) + r / 2] = (uint8_t)(q0 | (q1 << 4));
    }
  for (int64_t tr = 0; tr < TR; ++tr)
    for (int64_t tc = 0; tc < TCB; ++tc) {
      scales_col[tc * TR + tr] = scales[tr * TCB + tc];
      if (choice && choice_col) choice_col[tc * TR + tr] = choice[tr * TCB + tc];
    }
  return 0;
}

/* Dequantize columnwise-packed 2D-block data into the matrix's own row-major order. */
int nvfp4_46_ref_dequantize_2d_columnwise(const uint8_t *codes_col, const uint8_t *scales_col,
                                          float alpha, int64_t rows, int64_t cols,
                                          uint16_t *out) {
  int64_t TR = rows / BLOCK;
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t c = 0; c < cols; ++c) {
      float dec = ref_e4m3_decode(scales_col[(c / BLOCK) * TR + r / BLOCK]) * alpha;
      uint8_t byte = codes_col[c * (rows / 2) + r / 2];
      uint8_t code = (r & 1) ? (byte >> 4) : (byte & 15);
      out[r * cols + c] = ref_f32_to_bf16(ref_e2m1_decode(code) * dec);
    }
  return 0;
}

/* Dequantize 2D-block data: scales [rows/16][cols/16], codes as above. */
int nvfp4_46_ref_dequantize_2d(const uint8_t *codes, const uint8_t *scales, float alpha,
                               int64_t rows, int64_t cols, uint16_t *out) {
  int64_t TCB = cols / BLOCK;
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t c = 0; c < cols; ++c) {
      float dec = ref_e4m3_decode(scales[(r / BLOCK) * TCB + c / BLOCK]) * alpha;
      uint8_t byte = codes[r * (cols / 2) + c / 2];
      uint8_t code = (c & 1) ? (byte >> 4) : (byte & 15);
      out[r * cols + c] = ref_f32_to_bf16(ref_e2m1_decode(code) * dec);
    }
  return 0;
}

/* Table 3 lines 5 / 11 applied to stored data: out = bf16(grid(code) *
 * (value(S) * alpha)).  `layout` says how codes/scales are laid out; the
 * output is always [rows][cols] row-major. */
int nvfp4_46_ref_dequantize(const uint8_t *codes, const uint8_t *scales, float alpha, int64_t rows,
                            int64_t cols, int layout, uint16_t *out) {
  int64_t L = n_lines(rows, cols, layout), NB = n_blocks(rows, cols, layout);
#pragma omp parallel for schedule(static)
  for (int64_t line = 0; line < L; ++line)
    for (int64_t blk = 0; blk < NB; ++blk) {
      float dec = ref_e4m3_decode(scales[line * NB + blk]) * alpha;
      for (int i = 0; i < BLOCK; ++i) {
        uint8_t byte = codes[(line * NB + blk) * (BLOCK / 2) + i / 2];
        uint8_t code = (i & 1) ? (byte >> 4) : (byte & 15);
        int64_t r = (layout == REF_ROWWISE) ? line : blk * BLOCK + i;
        int64_t c = (layout == REF_ROWWISE) ? blk * BLOCK + i : line;
        out[r * cols + c] = ref_f32_to_bf16(ref_e2m1_decode(code) * dec);
      }
    }
  return 0;
}

/* Quantize-then-dequantize without materialising the codes; by construction
 * the same values as nvfp4_46_ref_dequantize(nvfp4_46_ref_quantize(x)).  With
 * the Hadamard transform on, the result stays in the transformed domain
 * (READING). */
int nvfp4_46_ref_fake_quant(const uint16_t *x, int64_t rows, int64_t cols, int layout,
                            int rounding, int select, int rht, uint64_t sr_seed,
                            uint64_t rht_seed, float alpha, uint16_t *out) {
  return nvfp4_46_ref_quantize(x, rows, cols, layout, rounding, select, rht, sr_seed, rht_seed,
                               alpha, NULL, NULL, NULL, out);
}

/* Per-block errors of both candidates for every block under the metric that
 * `select` names (test helper for the invariant E_chosen <= E_6).
 * E6 / E4: [lines][len/16] fp32. */
int nvfp4_46_ref_block_errors_sel(const uint16_t *x, int64_t rows, int64_t cols, int layout,
                                  int rounding, int select, int rht, uint64_t sr_seed,
                                  uint64_t rht_seed, float alpha, float *E6, float *E4) {
  int64_t L = n_lines(rows, cols, layout), NB = n_blocks(rows, cols, layout);
#pragma omp parallel for schedule(static)
  for (int64_t line = 0; line < L; ++line)
    for (int64_t blk = 0; blk < NB; ++blk) {
      float v[BLOCK], u[BLOCK], D[BLOCK], E[2];
      uint64_t g[BLOCK];
      uint8_t q[BLOCK], S, four;
      fetch_block(x_bf16(x), rows, cols, layout, line, blk, rht, rht_seed, v, g);
      for (int i = 0; i < BLOCK; ++i)
        u[i] = (rounding != REF_RTN) ? ref_sr_uniform(sr_seed, g[i]) : 0.0f;
      ref_quantize_block(v, alpha, rounding, select, u, q, D, &S, &four, E);
      E6[line * NB + blk] = E[0];
      E4[line * NB + blk] = E[1];
    }
  return 0;
}

int nvfp4_46_ref_block_errors(const uint16_t *x, int64_t rows, int64_t cols, int layout,
                              int rounding, int rht, uint64_t sr_seed, uint64_t rht_seed,
                              float alpha, float *E6, float *E4) {
  return nvfp4_46_ref_block_errors_sel(x, rows, cols, layout, rounding, REF_SEL_46_MSE, rht,
                                       sr_seed, rht_seed, alpha, E6, E4);
}

/* Matrix product of two NVFP4 tensors, the consumer of the quantizer's output (Fig. 3: FPROP,
 * DGRAD and WGRAD all multiply two NVFP4 operands quantized along the contraction axis):
 *   C[m][n] = alpha_a * alpha_b * sum_k a[m][k] * b[n][k],
 *   a[m][k] = grid(code_a[m][k]) * value(scale_a[m][k/16]), b likewise
 * with both operands in the rowwise layout over the contraction axis K (codes [M][K/2] and
 * [N][K/2], scales [M][K/16] and [N][K/16]).  The paper does not state the accumulation
 * arithmetic of the matrix unit (READING): this is the plain definition, every product and the
 * running sum in fp64 in the order k = 0, 1, ...; each product is exact in fp64 (at most 12
 * significant bits) and so is alpha_a * alpha_b.  `C` gets the fp64 values; `Cabs` (optional)
 * gets alpha_a * alpha_b * sum_k |a[m][k] * b[n][k]|, the quantity an error bound for a
 * lower-precision accumulation is stated in.
 * tiles_a / tiles_b = 1: that operand was quantized with 16x16 tiles (Section 4.1), so its
 * scales are [rows/16][K/16] and row m uses line m / 16. */
int nvfp4_46_ref_gemm(const uint8_t *codes_a, const uint8_t *scales_a, float alpha_a,
                      const uint8_t *codes_b, const uint8_t *scales_b, float alpha_b, int64_t M,
                      int64_t N, int64_t K, int tiles_a, int tiles_b, double *C, double *Cabs) {
  const int64_t KB = K / BLOCK;
  const double alpha = (double)alpha_a * (double)alpha_b;
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n) {
      double acc = 0.0, acc_abs = 0.0;
      for (int64_t k = 0; k < K; ++k) {
        uint8_t ba = codes_a[m * (K / 2) + k / 2], bb = codes_b[n * (K / 2) + k / 2];
        uint8_t ca = (k & 1) ? (ba >> 4) : (ba & 15), cb = (k & 1) ? (bb >> 4) : (bb & 15);
        int64_t la = tiles_a ? m / BLOCK : m, lb = tiles_b ? n / BLOCK : n;
        double a = (double)ref_e2m1_decode(ca) * (double)ref_e4m3_decode(scales_a[la * KB + k / BLOCK]);
        double b = (double)ref_e2m1_decode(cb) * (double)ref_e4m3_decode(scales_b[lb * KB + k / BLOCK]);
        acc += a * b;
        acc_abs += fabs(a * b);
      }
      C[m * N + n] = alpha * acc;
      if (Cabs) Cabs[m * N + n] = alpha * acc_abs;
    }
  return 0;
}

/* Range helpers for exhaustive comparisons of the scalar codecs: evaluate a
 * codec on n consecutive fp32 bit patterns starting at `first_bits`. */
void ref_e2m1_rtn_bits_range(uint32_t first_bits, int64_t n, uint8_t *out) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    uint32_t u = first_bits + (uint32_t)i;
    float f;
    memcpy(&f, &u, 4);
    out[i] = ref_e2m1_rtn(f);
  }
}

/* ref_e2m1_sr on n consecutive fp32 bit patterns, all with the uniform u. */
void ref_e2m1_sr_bits_range(uint32_t first_bits, int64_t n, float u, uint8_t *out) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    uint32_t b = first_bits + (uint32_t)i;
    float f;
    memcpy(&f, &b, 4);
    out[i] = ref_e2m1_sr(f, u);
  }
}

/* ref_e2m1_sr on n (y, u) pairs. */
void ref_e2m1_sr_n(const float *y, const float *u, int64_t n, uint8_t *out) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) out[i] = ref_e2m1_sr(y[i], u[i]);
}

void ref_e4m3_encode_bits_range(uint32_t first_bits, int64_t n, uint8_t *out) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    uint32_t u = first_bits + (uint32_t)i;
    float f;
    memcpy(&f, &u, 4);
    out[i] = ref_e4m3_encode(f);
  }
}
