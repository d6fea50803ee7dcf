/*
 * nvfp4_46 -- Four Over Six (4/6) NVFP4 quantization for AMD MI355X (gfx950).
 *
 * C ABI of libnvfp4_46.so.  The library quantizes BF16 tensors to block-scaled
 * NVFP4 (FP4 E2M1 codes, one FP8 E4M3 scale per 16 values, one FP32 scale per
 * tensor; arXiv 2512.02010 Section 2.1) with the paper's adaptive block scaling:
 * every block is quantized with its maximum mapped to 6 and again mapped to 4,
 * and the candidate with the smaller squared error is kept (Section 3, Table 3).
 *
 * General conventions (all entry points)
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library
 *     allocates no memory and keeps no state between calls (the one exception is the
 *     fixed scratch array of nvfp4_46_tensor_scale_static, described there).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Work is enqueued on it and the call returns without synchronising; a call
 *     that fails validation enqueues nothing.
 *   - The return value is an nvfp4_status; nothing is printed, thrown or aborted.
 *   - Tensors are dense row-major: x is [rows][cols], BF16 (2 bytes per element) or, with
 *     nvfp4_46_params.x_dtype = NVFP4_X_F32, fp32 (4 bytes per element).
 *   - Inputs must be finite.  The tensor scale must lie in [2^-100, 2^118]
 *     (nvfp4_46_tensor_scale guarantees this whenever max|x| >= 2^-89).
 *   - x and every output buffer must be 16-byte aligned.
 *   - Shapes: rowwise needs cols % 16 == 0; columnwise needs rows % 16 == 0 and
 *     cols % 8 == 0 (rows of x are read in 128-bit pieces); rows, cols <= 2^31 and
 *     rows * cols <= 2^40.
 *
 * Storage formats
 *   - code   4 bits: bit 3 = sign, bits 2..0 = index into {0, .5, 1, 1.5, 2, 3, 4, 6}
 *            (Section 1).  Two codes per byte: the element at the even position
 *            along the blocked axis sits in the low nibble.  The sign bit is the
 *            input's sign bit even when the magnitude rounds to zero.
 *   - scale  one FP8 E4M3 byte (bias 7, no infinity, largest value 448 = 0x7E;
 *            Section 2.1) per 16 consecutive elements along the blocked axis,
 *            stored as plain row-major bytes (no GEMM-specific swizzle).
 *   - rowwise layout  (blocks = 16 consecutive columns of one row):
 *            codes [rows][cols/2], scales [rows][cols/16], choice [rows][cols/16]
 *   - columnwise layout (blocks = 16 consecutive rows of one column, i.e. the
 *            rowwise quantization of the transposed tensor, as needed for the
 *            second operand orientation of Fig. 3):
 *            codes [cols][rows/2], scales [cols][rows/16], choice [cols][rows/16]
 *   - choice one byte per block: 0 = block scaled to 6, 1 = block scaled to 4.
 */
#ifndef NVFP4_46_H
#define NVFP4_46_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  NVFP4_OK = 0,
  NVFP4_ERR_NULL = 1,        /* a required pointer is NULL                                  */
  NVFP4_ERR_SHAPE = 2,       /* non-positive dims, or blocked axis not a multiple of 16      */
  NVFP4_ERR_ALIGN = 3,       /* a buffer is not 16-byte aligned                              */
  NVFP4_ERR_PARAM = 4,       /* unknown enum value, fp8_max outside (0, 448]                 */
  NVFP4_ERR_UNSUPPORTED = 5, /* a valid but unimplemented combination                        */
  NVFP4_ERR_HIP = 6          /* the HIP runtime reported a launch error                      */
} nvfp4_status;

/* layout bits; NVFP4_ROWWISE | NVFP4_COLWISE = both outputs from one read of x.
 * NVFP4_BLOCK2D only occurs in nvfp4_46_dequantize's `layout` argument, for data written
 * with nvfp4_46_params.block2d = 1: NVFP4_BLOCK2D alone = the rowwise packing (codes
 * [rows][cols/2], scales [rows/16][cols/16]), NVFP4_BLOCK2D | NVFP4_COLWISE = the packing for
 * the transposed matrix (codes [cols][rows/2], scales [cols/16][rows/16]). */
enum { NVFP4_ROWWISE = 1, NVFP4_COLWISE = 2, NVFP4_BLOCK2D = 4 };
/* rounding of scaled values onto the E2M1 grid */
enum { NVFP4_RTN = 0, NVFP4_SR = 1, NVFP4_SR_AFTER_RTN_SELECT = 2 };
/* element type of the input tensor x */
enum { NVFP4_X_BF16 = 0, NVFP4_X_F32 = 1 };
/* how the block scale is chosen */
enum { NVFP4_SEL_46_MSE = 0, NVFP4_SEL_FORCE6 = 1, NVFP4_SEL_FORCE4 = 2, NVFP4_SEL_46_MAE = 3,
       NVFP4_SEL_46_ABSMAX = 4 };

typedef struct {
  int64_t rows, cols;  /* logical shape of x                                                  */
  uint32_t layout;     /* NVFP4_ROWWISE, NVFP4_COLWISE or both                                */
  uint32_t rounding;   /* NVFP4_RTN: round to nearest, ties to the even code (Eq. 3).
                          NVFP4_SR: stochastic rounding (Section 2.2, Appendix A.3): a
                          scaled magnitude between grid neighbours lo < a < hi goes up iff
                          u < (a-lo)/(hi-lo), where u = (w >> 8) * 2^-24 and w is word (g&3)
                          of Philox4x32-10(key = sr_seed, counter = (g>>2, 0, 0)), g = the
                          element's flat index row*cols + col.  Both candidates use the same
                          u and the 4-vs-6 decision is taken on the rounded values.
                          NVFP4_SR_AFTER_RTN_SELECT (Appendix A.3, second alternative): the
                          4-vs-6 decision is taken on round-to-nearest candidates, then the
                          block is rounded stochastically (same u) with the selected scale.    */
  uint32_t select;     /* NVFP4_SEL_46_MSE: keep 4 iff its squared error is strictly
                          smaller (Table 3 line 13).  FORCE6 = standard NVFP4.  _46_MAE /
                          _46_ABSMAX: the same with the sum of |D_i - x_i| or the largest
                          |D_i - x_i| as the error (the other rules of Section 3.1, Table 4). */
  uint32_t rht;        /* 1: apply the 16-point random Hadamard transform (Section 2.2) to
                          each block before anything else: y = (1/4) H16 (s .* x), Sylvester
                          ordering, s_j = -1 iff bit j of word 0 of Philox4x32-10(key =
                          rht_seed, counter = (B, 0, 0, 1)), B = block position along the
                          blocked axis.  The outputs then describe the transformed values.     */
  uint64_t sr_seed, rht_seed;
  float fp8_max;       /* the FP8 constant of Eq. (1): 256 for 4/6 (Section 3.1), 448 for
                          standard NVFP4                                                       */
  uint32_t block2d;    /* 1: one scale (and one 4-vs-6 choice) per 16x16 tile instead of per 16
                          values of a row -- the 2D block quantization of weight matrices that
                          Section 4.1 names, under which a matrix and its transpose get the
                          same scales.  The tile's maximum sets the two candidate scales, each
                          row of the tile is quantized with them, and the tile's error is the
                          sum (largest, for _ABSMAX) of its sixteen row errors in the same
                          fixed order as within a row.  Needs rht = 0 and rows % 16 == cols % 16
                          == 0; codes_row is [rows][cols/2] as usual, scales_row and choice_row
                          are [rows/16][cols/16].  With NVFP4_COLWISE in `layout` the same tiles
                          are also (or only) written for the transposed matrix: codes_col
                          [cols][rows/2] holds the very same codes packed along the rows of x
                          (even row in the low nibble), scales_col and choice_col are
                          [cols/16][rows/16] -- the tiles are decided once, in x's orientation. */
  uint32_t x_dtype;    /* NVFP4_X_BF16, or NVFP4_X_F32: x holds fp32 values, which enter the
                          quantizer as they are -- the weights of Fig. 3, which are stored in
                          FP32 and quantized on every use.  Everything after the load is the
                          same arithmetic (it is fp32 throughout either way); outputs of
                          nvfp4_46_fake_quant stay BF16.                                       */
} nvfp4_46_params;

/* Eq. (1) with Section 3.1's constant: alpha = max|v| / (6 * fp8_max) over the values
 * that get quantized (after the Hadamard transform when rht = 1); alpha = 1 for an
 * all-zero tensor.  Uses rows, cols, layout (one orientation, matters only with rht),
 * rht, rht_seed and fp8_max of `p`.
 *   x      in   [rows][cols] BF16 (fp32 with x_dtype = NVFP4_X_F32)
 *   alpha  out  1 float (device); also used as scratch while the kernels run
 * Errors: NULL x/p/alpha -> ERR_NULL; bad dims -> ERR_SHAPE; x misaligned -> ERR_ALIGN;
 * bad fp8_max / layout / x_dtype -> ERR_PARAM; rht with both layouts -> ERR_UNSUPPORTED.        */
int nvfp4_46_tensor_scale(const void *x, const nvfp4_46_params *p, float *alpha,
                          void *stream);

/* nvfp4_46_tensor_scale in one kernel launch instead of three, for callers that can lend it
 * a few KiB of device memory: the reduction keeps its running maxima and completion counts
 * there instead of in the alpha word, and the last workgroup to finish applies Eq. (1).
 * Same result, bit for bit.
 *   workspace        in/out  at least NVFP4_46_TENSOR_SCALE_WS_BYTES bytes (device), 16-byte
 *                            aligned, owned by the caller.  Must be zero when the call's work
 *                            starts (zero it once after allocating it); the call leaves it zero,
 *                            so it can serve any number of calls -- one at a time: calls whose
 *                            work may overlap (different streams) need a workspace each.
 *   workspace_bytes  in      size of the workspace
 * Errors: as nvfp4_46_tensor_scale, plus workspace NULL -> ERR_NULL, too small -> ERR_PARAM,
 * misaligned -> ERR_ALIGN.                                                                      */
#define NVFP4_46_TENSOR_SCALE_WS_BYTES 4352
int nvfp4_46_tensor_scale_ws(const void *x, const nvfp4_46_params *p, float *alpha,
                             void *workspace, size_t workspace_bytes, void *stream);

/* nvfp4_46_tensor_scale_ws for callers that can neither allocate device memory nor lend any:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * scratch words live in a 4352-byte static device array inside the library (one copy per
 * GPU, held until the process ends); the call allocates nothing.  The scratch need does not
 * grow with the tensor, so every shape the other entry points accept is accepted (rows, cols
 * <= 2^31, rows * cols <= 2^40; beyond that ERR_SHAPE as everywhere).  Same result as
 * nvfp4_46_tensor_scale, bit for bit.
 * The array is zero when the library is loaded and every call's last workgroup leaves it zero
 * again.  All calls on one GPU share it: two calls whose work may overlap on that GPU (two
 * streams, two host threads) race and give wrong results -- use nvfp4_46_tensor_scale_ws
 * with a workspace each for those.  The first call on a device looks the array's address up
 * (hipGetSymbolAddress); make that call before starting a stream capture.
 * Errors: as nvfp4_46_tensor_scale; ERR_HIP if the address lookup fails.                       */
int nvfp4_46_tensor_scale_static(const void *x, const nvfp4_46_params *p, float *alpha,
                                 void *stream);

/* The 4/6 quantizer (Eq. (2), Eq. (3), Table 3 lines 1-14) in the requested
 * orientation(s).
 *   x           in   [rows][cols] BF16 (fp32 with x_dtype = NVFP4_X_F32)
 *   alpha       in   1 float (device): the tensor scale, from nvfp4_46_tensor_scale or
 *                    written by the caller
 *   codes_row, scales_row   out  required iff layout has NVFP4_ROWWISE, else must be NULL
 *   codes_col, scales_col   out  required iff layout has NVFP4_COLWISE, else must be NULL
 *   choice_row, choice_col  out  optional (NULL to skip) per-block 4-vs-6 flags
 * Errors: as above, plus a required output NULL -> ERR_NULL; an output given for a
 * layout that was not requested -> ERR_PARAM; rht = 1 with both layouts ->
 * ERR_UNSUPPORTED (the two orientations would be two different transformed tensors). */
int nvfp4_46_quantize(const void *x, const nvfp4_46_params *p, const float *alpha,
                      void *codes_row, void *scales_row, void *codes_col, void *scales_col,
                      void *choice_row, void *choice_col, void *stream);

/* Table 3 lines 5 / 11 on stored data: out = bf16_rne(value(code) * (value(scale) * alpha)).
 *   codes, scales  in   in the layout named by `layout` (NVFP4_ROWWISE, NVFP4_COLWISE,
 *                       NVFP4_BLOCK2D or NVFP4_BLOCK2D | NVFP4_COLWISE)
 *   out            out  [rows][cols] BF16, always row-major in the tensor's own orientation
 * Errors: NULL pointer -> ERR_NULL; bad dims -> ERR_SHAPE; misaligned -> ERR_ALIGN;
 * layout not one of the four values -> ERR_PARAM.                                      */
int nvfp4_46_dequantize(const void *codes, const void *scales, const float *alpha, int64_t rows,
                        int64_t cols, uint32_t layout, void *out_bf16, void *stream);

/* Quantize and dequantize in one kernel: out = what nvfp4_46_dequantize would return
 * for nvfp4_46_quantize's outputs, bit for bit, without writing codes or scales.
 * `layout` must name exactly one orientation.  With rht = 1 the result stays in the
 * transformed domain.  out_bf16 may not alias x.                                       */
int nvfp4_46_fake_quant(const void *x, const nvfp4_46_params *p, const float *alpha,
                        void *out_bf16, void *stream);

/* element type of nvfp4_46_gemm's output */
enum { NVFP4_OUT_BF16 = 0, NVFP4_OUT_F32 = 1 };
/* nvfp4_46_gemm flags: the operand was quantized with block2d = 1, i.e. its scales are one
 * line per 16 rows, [rows/16][K/16] (rows must then be a multiple of 16) */
enum { NVFP4_GEMM_A_TILE_SCALES = 1, NVFP4_GEMM_B_TILE_SCALES = 2 };

/* The consumer of the quantizer's output: the product of two NVFP4 tensors (Fig. 3: FPROP,
 * DGRAD and WGRAD each multiply two operands quantized along the contraction axis),
 *   C[m][n] = alpha_a * alpha_b * sum_k a[m][k] * b[n][k],
 *   a[m][k] = value(code_a[m][k]) * value(scale_a[m][k/16]),  b likewise.
 * The expanded operands are exact (in FP16) and every product is exact; the sum is
 * accumulated in fp32 by the matrix unit in an order that differs from k = 0, 1, ..., so
 * C agrees with the exactly rounded result to within 2 K 2^-24 alpha_a alpha_b
 * sum_k |a b| plus the output rounding, and is bit-reproducible from call to call.
 *   codes_a  in   [M][K/2]   rowwise NVFP4 codes of A   (nvfp4_46_quantize's codes_row)
 *   scales_a in   [M][K/16]  E4M3 scale bytes of A, each <= 0x7E ([M/16][K/16] with
 *                            NVFP4_GEMM_A_TILE_SCALES in `flags`; likewise for B)
 *   codes_b, scales_b  in    the same for B, which is [N][K] -- for y = x W^T pass the
 *                            rowwise quantization of W [N][K]; an operand that is needed
 *                            transposed is the columnwise output of the quantizer
 *   alpha_a, alpha_b   in    1 float each (device): the operands' tensor scales
 *   out      out  [M][N] row-major, BF16 (round to nearest even) or fp32 per `out_dtype`
 * K must be a multiple of 32.  Errors: NULL pointer -> ERR_NULL; non-positive dims,
 * K % 32 != 0 or a tile-scaled operand whose rows are not a multiple of 16 -> ERR_SHAPE;
 * misaligned buffer -> ERR_ALIGN; bad out_dtype or flags -> ERR_PARAM. */
int nvfp4_46_gemm(const void *codes_a, const void *scales_a, const float *alpha_a,
                  const void *codes_b, const void *scales_b, const float *alpha_b, int64_t M,
                  int64_t N, int64_t K, uint32_t out_dtype, uint32_t flags, void *out,
                  void *stream);

/* Human-readable name of a status code (static storage, never NULL). */
const char *nvfp4_46_status_string(int status);

/* ---- scalar codecs, exposed so that tests can compare them exhaustively ------------
 * Each evaluates exactly the device routine the kernels above use, on `n` inputs.     */

/* out[i] = E2M1 code (round to nearest even, saturating) of the fp32 value whose bit
 * pattern is first_bits + i.  out: n bytes (device). */
int nvfp4_46_debug_e2m1_rtn_range(uint32_t first_bits, int64_t n, void *out_u8, void *stream);
/* out[i] = E4M3 byte (round to nearest even, saturating at 448) of the non-negative fp32
 * value with bit pattern first_bits + i. */
int nvfp4_46_debug_e4m3_range(uint32_t first_bits, int64_t n, void *out_u8, void *stream);
/* For each E2M1 code c in 0..15: out_f32[c] = its value; for each E4M3 byte b in 0..255:
 * out_f32[16 + b] = its value.  out: 272 floats (device). */
int nvfp4_46_debug_decode_tables(void *out_f32, void *stream);
/* out[i] = BF16 (round to nearest even) of the fp32 value with bit pattern
 * first_bits + i * stride.  out: n uint16 (device). */
int nvfp4_46_debug_bf16_range(uint32_t first_bits, uint32_t stride, int64_t n, void *out_u16,
                              void *stream);
/* Stochastic rounding of y[i] (fp32, device) with the uniform u = (words[i] >> 8) * 2^-24
 * (uint32, device), by the two device routines the kernels use:
 *   out_u8[i]      = E2M1 code by the rule evaluated in software;
 *   out_fast_u8[i] = E2M1 code by the conversion instruction in bits 0-3, and bit 7 set when
 *                    the kernels would not trust that code and redo the element's block with
 *                    the software rule.
 * Both n bytes (device). */
int nvfp4_46_debug_e2m1_sr(const float *y, const uint32_t *words, int64_t n, void *out_u8,
                           void *out_fast_u8, void *stream);
/* Philox4x32-10: ctr [n][4] (uint32, device), key words by value -> out [n][4] (device). */
int nvfp4_46_debug_philox(const uint32_t *ctr, uint32_t key0, uint32_t key1, int64_t n,
                          uint32_t *out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* NVFP4_46_H */
