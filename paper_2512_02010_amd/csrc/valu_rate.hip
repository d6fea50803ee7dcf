// nvfp4_46_debug_valu_rate: how fast one class of vector-ALU instruction issues on this GPU.
//
// The quantizing kernels are bound by vector arithmetic in several configurations, and on
// gfx950 a wave's instruction does not cost the same in every class: the common fp32
// operations and the two-operand logic/shift/add operations issue about twice as fast as
// conversions, comparisons, selects, min/max, integer multiplies and the three-operand
// integer operations, and the FP4 / FP8 packing conversions take twice as long again.  The
// kernel below runs nothing but one instruction, 32 times per loop round on eight
// independent registers, in enough waves to fill the chip; the caller times it.
#include <hip/hip_runtime.h>

#include "nvfp4_46.h"

namespace nvfp4_46 {

constexpr int kRateThreads = 256;
constexpr int kRateGrid = 2048;        // 8 workgroups (32 waves) per compute unit on 256 units
constexpr int kRateKinds = 24;

#define NV_RATE_CASE(K, TEXT) \
  if (KIND == K) asm volatile(TEXT : "+v"(a[i]), "+v"(u[i]), "+v"(w[i]) : "v"(b), "v"(u[(i + 1) & 7]), "v"(u[(i + 2) & 7]), "s"(mask), "v"(c) : "vcc")

// Operands: %0 fp32 register, %1 32-bit integer register, %2 64-bit register pair (all
// read-write, one set per independent chain), %3 an fp32 value, %4 and %5 integer
// registers of neighbouring chains, %6 a 64-bit scalar lane mask, %7 a second fp32 value.
// (Three-source instructions are slower when two sources are one register or share a
// register bank, so the sources are kept distinct.)
template <int KIND>
__global__ __launch_bounds__(kRateThreads) void k_valu_rate(float *out, int iters, float b, float c) {
  float a[8];
  uint32_t u[8];
  uint64_t w[8];
  const uint64_t mask = 0x5555555555555555ull;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = threadIdx.x * 0.001f + i;
    u[i] = threadIdx.x * 77u + i;
    w[i] = u[i];
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        NV_RATE_CASE(0, "v_fma_f32 %0, %0, %3, %7");
        NV_RATE_CASE(1, "v_mul_f32 %0, %0, %3");
        NV_RATE_CASE(2, "v_add_f32 %0, %0, %3");
        NV_RATE_CASE(3, "v_max_f32 %0, %0, %3");
        NV_RATE_CASE(4, "v_max3_f32 %0, %0, %3, %7");
        NV_RATE_CASE(5, "v_xor_b32 %1, %1, %4");
        NV_RATE_CASE(6, "v_lshrrev_b32 %1, 8, %1");
        NV_RATE_CASE(7, "v_lshlrev_b32 %1, 3, %1");
        NV_RATE_CASE(8, "v_add_u32 %1, %1, %4");
        NV_RATE_CASE(9, "v_max_u32 %1, %1, %4");
        NV_RATE_CASE(10, "v_mad_u64_u32 %2, vcc, %1, %4, %2");
        NV_RATE_CASE(11, "v_mul_lo_u32 %1, %1, %4");
        NV_RATE_CASE(12, "v_cvt_f32_u32 %0, %1");
        NV_RATE_CASE(13, "v_floor_f32 %0, %0");
        NV_RATE_CASE(14, "v_rcp_f32 %0, %0");
        NV_RATE_CASE(15, "v_cndmask_b32_e64 %1, %1, %4, %6");
        NV_RATE_CASE(16, "v_cmp_lt_f32 vcc, %0, %3");
        NV_RATE_CASE(17, "v_bitop3_b32 %1, %1, %4, %5 bitop3:0x96");
        NV_RATE_CASE(18, "v_and_or_b32 %1, %1, %4, %5");
        NV_RATE_CASE(19, "v_perm_b32 %1, %1, %4, %5");
        NV_RATE_CASE(20, "v_cvt_scalef32_pk_fp4_f32 %1, %0, %3, %7");
        NV_RATE_CASE(21, "v_cvt_scalef32_pk_f32_fp4 %2, %1, %3");
        NV_RATE_CASE(22, "v_cvt_pk_fp8_f32 %1, %0, %3");
        NV_RATE_CASE(23, "v_cvt_pk_bf16_f32 %1, %0, %3");
      }
    }
  }
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < 8; ++i) s += a[i] + (float)u[i] + (float)(uint32_t)w[i];
  if (s == 12345.678f) out[0] = s;     // keeps every chain alive; practically never true
}

template <int KIND>
static void launch_rate(uint32_t kind, float *out, int iters, hipStream_t s) {
  if (kind == (uint32_t)KIND)
    hipLaunchKernelGGL(k_valu_rate<KIND>, dim3(kRateGrid), dim3(kRateThreads), 0, s, out, iters,
                       1.0001f, 0.5f);
  if constexpr (KIND + 1 < kRateKinds) launch_rate<KIND + 1>(kind, out, iters, s);
}

}  // namespace nvfp4_46

extern "C" int nvfp4_46_debug_valu_rate(uint32_t kind, int32_t iters, void *out_f32, void *stream) {
  using namespace nvfp4_46;
  if (!out_f32) return NVFP4_ERR_NULL;
  if (kind >= (uint32_t)kRateKinds || iters <= 0 || iters > (1 << 20)) return NVFP4_ERR_PARAM;
  launch_rate<0>(kind, static_cast<float *>(out_f32), iters, static_cast<hipStream_t>(stream));
  return hipGetLastError() == hipSuccess ? NVFP4_OK : NVFP4_ERR_HIP;
}
