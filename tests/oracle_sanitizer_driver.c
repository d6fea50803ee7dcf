/* Test infrastructure: runs every entry point of the CPU oracle on exactly-sized heap buffers
 * so that a build with -fsanitize=address,undefined (tests/test_oracle_sanitizers.py) reports
 * any out-of-bounds access, signed overflow, bad shift or misaligned access in it.  The oracle
 * source is #included, so its static helpers are instrumented too.  Prints a checksum (it
 * only has to be the same from run to run) and returns 0. */
#include "../oracle/nvfp4_46_ref.c"

#include <stdio.h>
#include <stdlib.h>

static uint32_t lcg_state = 0x1234567u;
static uint32_t lcg(void) { return lcg_state = lcg_state * 1664525u + 1013904223u; }

/* a value of wide dynamic range, sometimes zero, sometimes huge */
static float draw(void) {
  uint32_t r = lcg();
  if ((r & 63u) == 0) return 0.0f;
  float m = (float)((int32_t)(lcg() >> 8) - (1 << 23)) / (float)(1 << 23);
  int e = (int)((r >> 8) % 40u) - 30;
  return ldexpf(m, e);
}

static uint64_t sum_bytes(const void *p, size_t n) {
  const uint8_t *b = (const uint8_t *)p;
  uint64_t s = 0;
  for (size_t i = 0; i < n; ++i) s = s * 1099511628211ull + b[i];
  return s;
}

int main(void) {
  uint64_t check = 0;
  const int shapes[][2] = {{16, 16}, {48, 176}, {32, 64}, {1, 32}, {16, 8}, {144, 272}};
  for (unsigned si = 0; si < sizeof shapes / sizeof shapes[0]; ++si) {
    const int64_t rows = shapes[si][0], cols = shapes[si][1], n = rows * cols;
    uint16_t *xb = malloc(n * sizeof *xb);
    float *xf = malloc(n * sizeof *xf);
    for (int64_t i = 0; i < n; ++i) {
      xf[i] = draw();
      xb[i] = ref_f32_to_bf16(xf[i]);
    }
    for (int layout = REF_ROWWISE; layout <= REF_COLWISE; ++layout) {
      if (layout == REF_ROWWISE && cols % 16) continue;
      if (layout == REF_COLWISE && rows % 16) continue;
      const int64_t lines = layout == REF_ROWWISE ? rows : cols, len = layout == REF_ROWWISE ? cols : rows;
#ifdef PLANT_SHORT_BUFFER   /* the test's self-check: the sanitizer must catch the oracle's own store */
      uint8_t *codes = malloc(lines * len / 2), *scales = malloc(lines * len / 16 - 1),
              *choice = malloc(lines * len / 16);
#else
      uint8_t *codes = malloc(lines * len / 2), *scales = malloc(lines * len / 16),
              *choice = malloc(lines * len / 16);
#endif
      uint16_t *deq = malloc(n * sizeof *deq), *deq2 = malloc(n * sizeof *deq2);
      float *E6 = malloc(lines * len / 16 * sizeof *E6), *E4 = malloc(lines * len / 16 * sizeof *E4);
      for (int rht = 0; rht <= 1; ++rht) {
        float alpha, alpha_f;
        nvfp4_46_ref_tensor_scale(xb, rows, cols, layout, rht, 77, 256.0f, &alpha);
        nvfp4_46_ref_tensor_scale_f32(xf, rows, cols, layout, rht, 77, 448.0f, &alpha_f);
        for (int rounding = REF_RTN; rounding <= REF_SR_AFTER_RTN_SELECT; ++rounding)
          for (int select = REF_SEL_46_MSE; select <= REF_SEL_46_ABSMAX; ++select) {
            nvfp4_46_ref_quantize(xb, rows, cols, layout, rounding, select, rht, 5, 77, alpha, codes,
                                  scales, choice, deq);
            check += sum_bytes(codes, lines * len / 2) + sum_bytes(scales, lines * len / 16) +
                     sum_bytes(choice, lines * len / 16) + sum_bytes(deq, n * 2);
            nvfp4_46_ref_quantize_f32(xf, rows, cols, layout, rounding, select, rht, 5, 77, alpha_f,
                                      codes, scales, NULL, NULL);
            check += sum_bytes(codes, lines * len / 2);
            nvfp4_46_ref_fake_quant(xb, rows, cols, layout, rounding, select, rht, 5, 77, alpha, deq2);
            check += sum_bytes(deq2, n * 2);
            nvfp4_46_ref_block_errors_sel(xb, rows, cols, layout, rounding, select, rht, 5, 77, alpha,
                                          E6, E4);
          }
        nvfp4_46_ref_quantize(xb, rows, cols, layout, REF_RTN, REF_SEL_46_MSE, rht, 0, 77, alpha, codes,
                              scales, choice, NULL);
        nvfp4_46_ref_dequantize(codes, scales, alpha, rows, cols, layout, deq);
        check += sum_bytes(deq, n * 2);
        if (rows % 32 == 0)
          nvfp4_46_ref_quantize_rows(xb + 16 * cols, rows - 16, cols, 16, layout, REF_SR, REF_SEL_46_MSE,
                                     rht, 5, 77, alpha, codes, scales, choice, deq);
      }
      free(codes); free(scales); free(choice); free(deq); free(deq2); free(E6); free(E4);
    }
    if (rows % 16 == 0 && cols % 16 == 0) {
      uint8_t *codes = malloc(n / 2), *scales = malloc(n / 256), *choice = malloc(n / 256);
      uint8_t *cc = malloc(n / 2), *sc = malloc(n / 256), *fc = malloc(n / 256);
      uint16_t *deq = malloc(n * sizeof *deq);
      float alpha;
      nvfp4_46_ref_tensor_scale(xb, rows, cols, REF_ROWWISE, 0, 0, 256.0f, &alpha);
      for (int rounding = REF_RTN; rounding <= REF_SR_AFTER_RTN_SELECT; ++rounding)
        for (int select = REF_SEL_46_MSE; select <= REF_SEL_46_ABSMAX; ++select) {
          nvfp4_46_ref_quantize_2d(xb, rows, cols, rounding, select, 5, alpha, codes, scales, choice, deq);
          nvfp4_46_ref_quantize_2d_f32(xf, rows, cols, rounding, select, 5, alpha, codes, scales, choice, deq);
          check += sum_bytes(codes, n / 2) + sum_bytes(scales, n / 256);
        }
      nvfp4_46_ref_repack_2d_columnwise(codes, scales, choice, rows, cols, cc, sc, fc);
      nvfp4_46_ref_dequantize_2d(codes, scales, alpha, rows, cols, deq);
      check += sum_bytes(deq, n * 2);
      nvfp4_46_ref_dequantize_2d_columnwise(cc, sc, alpha, rows, cols, deq);
      check += sum_bytes(deq, n * 2) + sum_bytes(cc, n / 2) + sum_bytes(sc, n / 256) + sum_bytes(fc, n / 256);
      /* the product of the matrix with itself, row scales and tile scales */
      uint8_t *rc = malloc(n / 2), *rs = malloc(n / 16);
      nvfp4_46_ref_quantize(xb, rows, cols, REF_ROWWISE, REF_RTN, REF_SEL_46_MSE, 0, 0, 0, alpha, rc, rs,
                            NULL, NULL);
      double *C = malloc(rows * rows * sizeof *C), *Ca = malloc(rows * rows * sizeof *Ca);
      nvfp4_46_ref_gemm(rc, rs, alpha, rc, rs, alpha, rows, rows, cols, 0, 0, C, Ca);
      nvfp4_46_ref_gemm(codes, scales, alpha, rc, rs, alpha, rows, rows, cols, 1, 0, C, NULL);
      check += sum_bytes(C, rows * rows * sizeof *C);
      free(codes); free(scales); free(choice); free(cc); free(sc); free(fc); free(deq);
      free(rc); free(rs); free(C); free(Ca);
    }
    free(xb); free(xf);
  }
  /* scalar codecs over awkward arguments */
  const float odd[] = {0.0f, -0.0f, 1e-45f, 1e-38f, 0.25f, 5.0f, 6.0f, 7.0f, 447.9f, 448.0f, 1e30f, 3.4e38f};
  for (unsigned i = 0; i < sizeof odd / sizeof odd[0]; ++i) {
    check += ref_e2m1_rtn(odd[i]) + ref_e2m1_rtn(-odd[i]) + ref_e4m3_encode(odd[i]) +
             ref_f32_to_bf16(odd[i]) + ref_e2m1_sr(odd[i], 0.5f) + ref_block_scale(odd[i], 1e-20f, 6.0f);
  }
  uint8_t range[4096];
  ref_e2m1_rtn_bits_range(0x3e7ff800u, 4096, range);
  ref_e4m3_encode_bits_range(0x43dff800u, 4096, range);
  ref_e2m1_rtn_bits_range(0xfffff000u, 4096, range);      /* up to the last bit pattern */
  for (int c = 0; c < 256; ++c) check += (uint64_t)(ref_e4m3_decode((uint8_t)c) != 0.0f) + (uint64_t)ref_e2m1_decode((uint8_t)c);
  printf("oracle sanitizer driver: ok, checksum %016llx\n", (unsigned long long)check);
  return 0;
}
