// NVFP4 x NVFP4 matrix product for gfx950: C = alpha_a * alpha_b * A . B^T with both operands
// in the quantizer's rowwise layout over the contraction axis (see include/nvfp4_46.h).
//
// gfx950's block-scaled FP4 matrix instructions take one power-of-two scale per 32 values;
// NVFP4 carries an E4M3 scale (three mantissa bits) per 16, so the operands are expanded on
// the way into the matrix unit instead: value(code) * value(scale) has at most six
// significant bits and lies in [2^-10, 2688], hence is exact in FP16, and the FP16 matrix
// instruction (v_mfma_f32_32x32x16_f16, fp32 accumulation) multiplies exact operands.  The
// only rounding is in the fp32 accumulation and in the final scaling.
//
// Data movement: the operands stay packed (4 bits per value) all the way into registers.
// A workgroup of four waves owns a 256 x 256 tile of C, each wave a 128 x 128 quarter
// (4 x 4 matrix-instruction tiles, 256 accumulator registers per lane).  Per chunk of 128
// contraction steps the workgroup copies 256 rows x 64 bytes of codes and 256 x 8 scale
// bytes of each operand into LDS with coalesced loads (the next chunk's loads are in flight
// while the current one is multiplied); a lane then reads 16 bytes (32 codes) per operand
// tile from LDS and expands them with v_cvt_scalef32_pk_f16_fp4 (x 256, exact) and one
// packed FP16 multiplication by the scale (times 2^-8, built from the scale byte by a
// shift).  Which eight contraction indices a lane feeds to a given matrix instruction is
// the same for A and for B, which is all the sum needs.
//
// Two kernels share this plan: k_gemm (any K that is a multiple of 32; the workgroup stages
// chunks through registers into shared LDS buffers, one barrier per chunk) and k_gemm_dma
// (K a multiple of 128; every wave fills its own LDS with asynchronous global -> LDS copies
// and never meets a barrier).
#include <hip/hip_runtime.h>

#include "codec.hpp"
#include "launch.hpp"
#include "nvfp4_46.h"

namespace nvfp4_46 {

typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kGemmThreads = 256;
constexpr int GT = 256;                  // rows of A (and of B) per workgroup tile
constexpr int GK = 128;                  // contraction steps per LDS chunk
constexpr int kCodeRow = GK / 2 + 16;    // bytes per operand row in LDS: 64 of codes + 16 of padding,
                                         // so that 16 lanes reading 16 bytes from 16 rows hit 16
                                         // different bank groups (80 = 5 * 16, 5 coprime to 16)

// Eight codes (one 32-bit word) times one scale -> eight FP16 values, exactly.
// `sv` is the FP16 with the bit pattern (scale byte << 7), i.e. value(scale) * 2^-8 (also for
// the subnormal scale bytes); the conversion multiplies by 2^8.
NV_DEV h8 expand8(uint32_t word, _Float16 sv) {
  const h2 s = {sv, sv};
  const h2 p0 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(word, 256.0f, 0) * s;
  const h2 p1 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(word, 256.0f, 1) * s;
  const h2 p2 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(word, 256.0f, 2) * s;
  const h2 p3 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(word, 256.0f, 3) * s;
  return h8{p0.x, p0.y, p1.x, p1.y, p2.x, p2.y, p3.x, p3.y};
}

// LDS: two buffers (chunk c is multiplied out of one while chunk c + 1 is written into the
// other), each holding both operands' codes and scales.
struct GemmStage {
  uint8_t codes[2][GT * kCodeRow];   // [A, B][row][80]
  uint4 scales[2][GT];               // [A, B][row] -> the row's 8 scales as FP16 bit patterns
                                     // (byte << 7 = value * 2^-8), ready to multiply with
};
constexpr size_t kGemmLdsBytes = 2 * sizeof(GemmStage);

// What a lane holds of one half chunk (64 contraction steps): per operand tile 16 bytes of
// codes and the two scale bytes that go with them.
struct RawHalf {
  uint4 a[4], b[4];
  uint32_t sa[4], sb[4];
};
struct Frags {
  h8 a[4], b[4];
};

// KFULL: K is a multiple of 128, so every chunk is whole and scale rows are 8-byte aligned.
//
// The main loop is a software pipeline over "steps" of 16 contraction indices (8 per chunk):
// while the 16 matrix instructions of step s run, the lane expands the operands of step
// s + 1 (64 vector instructions, issued in the matrix instructions' shadow).  Per chunk:
//   step 1: read the second half's codes and scales from LDS;
//   step 5: write the next chunk (fetched from global memory one chunk earlier) into the
//           other LDS buffer and start fetching the chunk after it;
//   step 6: barrier (every wave has finished reading this buffer and writing the other),
//           then read the next chunk's first half from LDS;
//   step 7: expand the next chunk's first step.
// So the matrix unit is never left waiting for a barrier, an LDS read or an expansion.
template <bool KFULL, bool OUTF32>
__global__ __launch_bounds__(kGemmThreads) void k_gemm(
    const uint8_t *__restrict__ codes_a, const uint8_t *__restrict__ scales_a,
    const float *__restrict__ alpha_a, const uint8_t *__restrict__ codes_b,
    const uint8_t *__restrict__ scales_b, const float *__restrict__ alpha_b,
    void *__restrict__ out, int64_t M, int64_t N, int64_t K, uint32_t tiles_n, uint32_t sha,
    uint32_t shb) {
  extern __shared__ __align__(16) uint8_t lds_raw[];
  GemmStage *stage = reinterpret_cast<GemmStage *>(lds_raw);

  const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
  const uint32_t r = lane & 31u, g = lane >> 5;        // row within a 32-row tile, half of K
  const uint32_t wm = wave >> 1, wn = wave & 1u;       // the wave's quarter of the tile
  const uint32_t tile_m = blockIdx.x / tiles_n, tile_n = blockIdx.x - tile_m * tiles_n;
  const int64_t m0 = (int64_t)tile_m * GT, n0 = (int64_t)tile_n * GT;
  const int64_t row_codes = K / 2, row_scales = K / 16;

  // ---- global -> registers -> LDS.  Codes: 1024 16-byte pieces per operand and chunk,
  // four per thread (piece = row * 4 + unit, so four lanes read 64 contiguous bytes);
  // scales: thread t fetches row t's eight bytes.  Rows past the end of an operand re-read
  // its last row (their products are never stored).
  uint4 ga[4], gb[4];
  uint2 gsa, gsb;
  const uint32_t ld_row = t >> 2, ld_unit = t & 3u;
  auto clamp_row = [](int64_t row, int64_t n) { return row < n ? row : n - 1; };
  const uint8_t *pa[4], *pb[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    pa[q] = codes_a + clamp_row(m0 + ld_row + 64 * q, M) * row_codes + ld_unit * 16;
    pb[q] = codes_b + clamp_row(n0 + ld_row + 64 * q, N) * row_codes + ld_unit * 16;
  }
  // a row's scale line: the row itself, or row / 16 for an operand quantized in 16x16 tiles
  const uint8_t *psa = scales_a + (clamp_row(m0 + t, M) >> sha) * row_scales;
  const uint8_t *psb = scales_b + (clamp_row(n0 + t, N) >> shb) * row_scales;
  auto fetch = [&](int64_t k0) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      ga[q] = gb[q] = make_uint4(0, 0, 0, 0);
      if (KFULL || k0 + ld_unit * 32 < K) {
        ga[q] = *reinterpret_cast<const uint4 *>(pa[q] + k0 / 2);
        gb[q] = *reinterpret_cast<const uint4 *>(pb[q] + k0 / 2);
      }
    }
    if (KFULL) {
      gsa = *reinterpret_cast<const uint2 *>(psa + k0 / 16);
      gsb = *reinterpret_cast<const uint2 *>(psb + k0 / 16);
    } else {
      // two scale bytes (32 contraction steps) at a time; K is a multiple of 32
      uint32_t wa[4], wb[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        wa[q] = wb[q] = 0;
        if (k0 + 32 * q < K) {
          wa[q] = *reinterpret_cast<const uint16_t *>(psa + k0 / 16 + 2 * q);
          wb[q] = *reinterpret_cast<const uint16_t *>(psb + k0 / 16 + 2 * q);
        }
      }
      gsa = make_uint2(wa[0] | (wa[1] << 16), wa[2] | (wa[3] << 16));
      gsb = make_uint2(wb[0] | (wb[1] << 16), wb[2] | (wb[3] << 16));
    }
  };
  auto stash = [&](GemmStage &st) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const uint32_t off = (ld_row + 64 * q) * kCodeRow + ld_unit * 16;
      *reinterpret_cast<uint4 *>(&st.codes[0][off]) = ga[q];
      *reinterpret_cast<uint4 *>(&st.codes[1][off]) = gb[q];
    }
    // scale bytes -> FP16 bit patterns, two per word
    auto widen = [](uint32_t two_bytes) { return ((two_bytes & 0xffu) << 7) | ((two_bytes & 0xff00u) << 15); };
    st.scales[0][t] = make_uint4(widen(gsa.x), widen(gsa.x >> 16), widen(gsa.y), widen(gsa.y >> 16));
    st.scales[1][t] = make_uint4(widen(gsb.x), widen(gsb.x >> 16), widen(gsb.y), widen(gsb.y >> 16));
  };

  // ---- LDS -> registers: 16 bytes (32 codes, two scale blocks) per operand tile and half
  const uint32_t a_row0 = wm * 128 + r, b_row0 = wn * 128 + r;
  auto read_half = [&](const GemmStage &st, int half, RawHalf &h) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t rowa = a_row0 + 32 * i, rowb = b_row0 + 32 * i;
      h.a[i] = *reinterpret_cast<const uint4 *>(&st.codes[0][rowa * kCodeRow + (2 * half + g) * 16]);
      h.b[i] = *reinterpret_cast<const uint4 *>(&st.codes[1][rowb * kCodeRow + (2 * half + g) * 16]);
      // the lane's two scales of this half (blocks 4*half + 2*g and + 1), one word
      const uint32_t *wa = reinterpret_cast<const uint32_t *>(&st.scales[0][rowa]);
      const uint32_t *wb = reinterpret_cast<const uint32_t *>(&st.scales[1][rowb]);
      h.sa[i] = wa[2 * half + g];
      h.sb[i] = wb[2 * half + g];
    }
  };
  // operands of step s (0..3) of a half: word s of the 16 bytes, scale byte s / 2
  auto expand = [&](const RawHalf &h, int s, Frags &f) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t wa = s == 0 ? h.a[i].x : s == 1 ? h.a[i].y : s == 2 ? h.a[i].z : h.a[i].w;
      const uint32_t wb = s == 0 ? h.b[i].x : s == 1 ? h.b[i].y : s == 2 ? h.b[i].z : h.b[i].w;
      // the block's scale: low or high half of the pair read from LDS
      const h2 pa2 = __builtin_bit_cast(h2, h.sa[i]), pb2 = __builtin_bit_cast(h2, h.sb[i]);
      f.a[i] = expand8(wa, s < 2 ? pa2.x : pa2.y);
      f.b[i] = expand8(wb, s < 2 ? pb2.x : pb2.y);
    }
  };

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  auto mfma16 = [&](const Frags &f) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(f.a[i], f.b[j], acc[i][j], 0, 0, 0);
  };
  // ask the scheduler to issue four vector instructions behind every matrix instruction, and
  // the step's LDS / global accesses one at a time behind the first matrix instructions
  auto interleave = [&](int lds_reads, int lds_writes, int vmem_reads) {
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      if (q < lds_reads) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      if (q < lds_writes) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
      if (q < vmem_reads) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
    }
  };

  const int64_t nchunks = (K + GK - 1) / GK;
  RawHalf h0, h1;
  Frags f0, f1;
  fetch(0);
  stash(stage[0]);
  __syncthreads();
  fetch(nchunks > 1 ? GK : 0);
  read_half(stage[0], 0, h0);
  expand(h0, 0, f0);

  // one chunk; `last` = no chunk follows (nothing to write, read or expand ahead)
  auto chunk = [&](int64_t c, bool last) {
    GemmStage &cur = stage[c & 1], &nxt = stage[(c + 1) & 1];
#pragma unroll
    for (int st = 0; st < 8; ++st) {
      Frags &fc = (st & 1) ? f1 : f0, &fn = (st & 1) ? f0 : f1;
      if (st == 1) read_half(cur, 1, h1);
      if (st == 5 && !last) {
        stash(nxt);
        const int64_t c2 = c + 2 < nchunks ? c + 2 : nchunks - 1;   // past the end: a harmless re-read
        fetch(c2 * GK);
      }
      if (st == 6) {
        // keep each step's instructions on their own side of the barrier
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
        if (!last) read_half(nxt, 0, h0);
      }
      if (st < 7) expand(st < 3 ? h0 : h1, (st + 1) & 3, fn);
      else if (!last) expand(h0, 0, fn);
      mfma16(fc);
      interleave(st == 1 || (st == 6 && !last) ? 16 : 0, st == 5 && !last ? 10 : 0,
                 st == 5 && !last ? 10 : 0);
    }
  };
  for (int64_t c = 0; c + 1 < nchunks; ++c) chunk(c, false);
  chunk(nchunks - 1, true);

  // ---- epilogue: accumulator element v of tile (i, j) is C[32 i + 8 (v / 4) + 4 g + v % 4]
  // [32 j + r] within the wave's quarter
  const float scale = alpha_a[0] * alpha_b[0];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int64_t col = n0 + wn * 128 + 32 * j + r;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int64_t row = m0 + wm * 128 + 32 * i + 8 * (v / 4) + 4 * g + (v % 4);
        if (row < M && col < N) {
          const float c = acc[i][j][v] * scale;
          if (OUTF32)
            static_cast<float *>(out)[row * N + col] = c;
          else
            static_cast<uint16_t *>(out)[row * N + col] = (uint16_t)pack_bf16x2(c, 0.0f);
        }
      }
    }
}

// ----------------------------------------------------------------------------------------
// The same product with wave-private LDS filled by asynchronous global -> LDS loads
// (global_load_lds_dwordx4): no staging registers, no LDS write instructions and no
// workgroup barrier at all.  Each wave copies the 128 rows of A and the 128 rows of B that its
// own quarter of the tile needs (the two waves that share rows each fetch them; operand
// bytes are small) into its own 2 x 18 KiB of LDS:
//   per stage: A codes [128][64 B], B codes [128][64 B], A scales [128][8 B], B scales [128][8 B]
// A load instruction writes its 64 lanes' 16 (or 4) bytes to consecutive LDS addresses, so
// the LDS layout is plain row-major; to keep the later 16-byte reads of 16 lanes on 16
// different bank groups, lane (row, position p) of a copy fetches the row's 16-byte unit
// p ^ ((row >> 2) & 3), and readers look unit u up at position u ^ ((row >> 2) & 3).
// The copies are issued with inline assembly (the compiler then neither reorders LDS reads
// around them nor waits for all of them at every LDS read) and waited for with explicit
// s_waitcnt vmcnt: the kernel issues no other vector-memory loads inside the loop.
// Only for K a multiple of 128 (whole chunks) and K <= 2^24 (32-bit lane offsets).
constexpr uint32_t kDmaStage = 2 * 128 * 64 + 2 * 128 * 8;   // 18432 bytes per wave and stage
constexpr uint32_t kDmaWave = 2 * kDmaStage;
constexpr size_t kGemmDmaLdsBytes = 4 * kDmaWave;   // 147456

// M0 = LDS byte address of lane 0's piece; %1 = the lane's 32-bit byte offset (vector
// register), %2 = the 64-bit base address (scalar register pair).
#define NV_DMA16(lds_sgpr, voff, gbase)                                                       \
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"                          \
               :: "s"(lds_sgpr), "v"(voff), "s"(gbase) : "memory", "m0")
#define NV_DMA4(lds_sgpr, voff, gbase)                                                        \
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dword %1, %2"                            \
               :: "s"(lds_sgpr), "v"(voff), "s"(gbase) : "memory", "m0")

template <bool OUTF32>
__global__ __launch_bounds__(kGemmThreads) void k_gemm_dma(
    const uint8_t *__restrict__ codes_a, const uint8_t *__restrict__ scales_a,
    const float *__restrict__ alpha_a, const uint8_t *__restrict__ codes_b,
    const uint8_t *__restrict__ scales_b, const float *__restrict__ alpha_b,
    void *__restrict__ out, int64_t M, int64_t N, int64_t K, uint32_t tiles_n, uint32_t sha,
    uint32_t shb) {
  extern __shared__ __align__(16) uint8_t lds_raw[];
  const uint32_t t = threadIdx.x, lane = t & 63u;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const uint32_t r = lane & 31u, g = lane >> 5;
  const uint32_t wm = wave >> 1, wn = wave & 1u;
  const uint32_t tile_m = blockIdx.x / tiles_n, tile_n = blockIdx.x - tile_m * tiles_n;
  const int64_t m0 = (int64_t)tile_m * GT + wm * 128, n0 = (int64_t)tile_n * GT + wn * 128;
  const int64_t row_codes = K / 2, row_scales = K / 16;

  const uint8_t *wl = lds_raw + wave * kDmaWave;   // the wave's LDS, for reading
  const uint32_t lds_wave =
      (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)lds_raw + wave * kDmaWave;

  // first rows of the wave's operand slices (a slice that starts past the end re-reads the
  // last row; nothing of it is stored), and each lane's byte offset from there for every
  // copy instruction of a chunk
  const int64_t a_base = m0 < M ? m0 : M - 1, b_base = n0 < N ? n0 : N - 1;
  // (wave-uniform by construction; read through readfirstlane so that they live in scalar
  // registers, which is where the copy instruction takes its base address from)
  auto uniform = [](const uint8_t *p) {
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const uint8_t *>(((uint64_t)hi << 32) | lo);
  };
  const uint8_t *gca = uniform(codes_a + a_base * row_codes), *gcb = uniform(codes_b + b_base * row_codes);
  // (a row's scale line: the row itself, or row / 16 for an operand quantized in 16x16 tiles)
  const uint8_t *gsa = uniform(scales_a + (a_base >> sha) * row_scales);
  const uint8_t *gsb = uniform(scales_b + (b_base >> shb) * row_scales);
  uint32_t oca[8], ocb[8], osa[4], osb[4];
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    const uint32_t row = 16 * q + (lane >> 2), unit = (lane & 3u) ^ ((row >> 2) & 3u);
    const int64_t ra = a_base + row < M ? row : M - 1 - a_base;
    const int64_t rb = b_base + row < N ? row : N - 1 - b_base;
    oca[q] = (uint32_t)(ra * row_codes) + unit * 16;
    ocb[q] = (uint32_t)(rb * row_codes) + unit * 16;
  }
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const uint32_t row = 32 * q + (lane >> 1), half = lane & 1u;
    const int64_t ra = a_base + row < M ? row : M - 1 - a_base;
    const int64_t rb = b_base + row < N ? row : N - 1 - b_base;
    osa[q] = (uint32_t)((((a_base + ra) >> sha) - (a_base >> sha)) * row_scales) + half * 4;
    osb[q] = (uint32_t)((((b_base + rb) >> shb) - (b_base >> shb)) * row_scales) + half * 4;
  }
  // the 24 copy instructions of a chunk, numbered so that they can be issued one at a time
  auto copy_one = [&](int64_t c, uint32_t stage, int n) {
    const uint32_t lds = lds_wave + stage * kDmaStage;
    if (n < 8) NV_DMA16(lds + n * 1024, oca[n], gca + c * (GK / 2));
    else if (n < 16) NV_DMA16(lds + 8192 + (n - 8) * 1024, ocb[n - 8], gcb + c * (GK / 2));
    else if (n < 20) NV_DMA4(lds + 16384 + (n - 16) * 256, osa[n - 16], gsa + c * (GK / 16));
    else NV_DMA4(lds + 17408 + (n - 20) * 256, osb[n - 20], gsb + c * (GK / 16));
  };
  auto copy_chunk = [&](int64_t c, uint32_t stage) {
#pragma unroll
    for (int n = 0; n < 24; ++n) copy_one(c, stage, n);
  };

  // ---- LDS -> registers, one operand tile at a time (u = 0..3: A tiles, 4..7: B tiles)
  const uint32_t swz = (r >> 2) & 3u;
  auto read_tile = [&](uint32_t stage, int half, int u, RawHalf &h) {
    const uint8_t *st = wl + stage * kDmaStage + (u < 4 ? 0 : 8192);
    const uint8_t *sc = wl + stage * kDmaStage + (u < 4 ? 16384 : 17408);
    const uint32_t row = 32 * (u & 3) + r, pos = ((2 * half + g) ^ swz) * 16;
    const uint4 codes = *reinterpret_cast<const uint4 *>(st + row * 64 + pos);
    // the lane's two scale bytes of this half (blocks 4*half + 2*g and + 1), still raw
    const uint32_t two = *reinterpret_cast<const uint16_t *>(sc + row * 8 + 4 * half + 2 * g);
    if (u < 4) { h.a[u] = codes; h.sa[u] = two; } else { h.b[u - 4] = codes; h.sb[u - 4] = two; }
  };
  // operands of step s (0..3) of a half for tile u; at s == 0 the two scale bytes are turned
  // into two FP16 bit patterns (byte << 7) in one word
  auto expand_tile = [&](RawHalf &h, int s, int u, Frags &f) {
    const uint4 &w4 = u < 4 ? h.a[u] : h.b[u - 4];
    uint32_t &sc = u < 4 ? h.sa[u] : h.sb[u - 4];
    if (s == 0) sc = __builtin_amdgcn_perm(0u, sc, 0x0c010c00u) << 7;
    const uint32_t w = s == 0 ? w4.x : s == 1 ? w4.y : s == 2 ? w4.z : w4.w;
    const h2 pair = __builtin_bit_cast(h2, sc);
    const h8 e = expand8(w, s < 2 ? pair.x : pair.y);
    if (u < 4) f.a[u] = e; else f.b[u - 4] = e;
  };

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  const int64_t nchunks = K / GK;
  RawHalf h0, h1;
  Frags f0, f1;
  copy_chunk(0, 0);
  copy_chunk(nchunks > 1 ? 1 : 0, 1);
  asm volatile("s_waitcnt vmcnt(24)" ::: "memory");      // chunk 0 is in LDS
#pragma unroll
  for (int u = 0; u < 8; ++u) read_tile(0, 0, u, h0);
#pragma unroll
  for (int u = 0; u < 8; ++u) expand_tile(h0, 0, u, f0);

  // Chunk c sits in stage c & 1.  A step is eight units of two matrix instructions; unit u
  // also expands operand tile u for the next step and carries the step's share of LDS
  // reads and copy instructions, so that everything issues in the matrix unit's shadow:
  //   step 1        reads the chunk's second half (then the stage is free);
  //   steps 3-5     start the 24 copies of chunk c + 2 into this stage, one per unit;
  //   step 6        waits until only those 24 are outstanding (chunk c + 1 has landed in the
  //                 other stage) and reads its first half;
  //   step 7        expands the next chunk's first step.
  auto chunk = [&](int64_t c, bool last) {
    const uint32_t cur = (uint32_t)c & 1u, nxt = cur ^ 1u;
    const int64_t c2 = c + 2 < nchunks ? c + 2 : nchunks - 1;   // past the end: a harmless re-read
#pragma unroll
    for (int st = 0; st < 8; ++st) {
      Frags &fc = (st & 1) ? f1 : f0, &fn = (st & 1) ? f0 : f1;
      if (st == 3 && !last) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      if (st == 6 && !last) asm volatile("s_waitcnt vmcnt(24)" ::: "memory");
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (st == 1) read_tile(cur, 1, u, h1);
        if (st >= 3 && st <= 5 && !last) copy_one(c2, cur, 8 * (st - 3) + u);
        if (st == 6 && !last) read_tile(nxt, 0, u, h0);
        if (st < 7) expand_tile(st < 3 ? h0 : h1, (st + 1) & 3, u, fn);
        else if (!last) expand_tile(h0, 0, u, fn);
#pragma unroll
        for (int q = 2 * u; q < 2 * u + 2; ++q)
          acc[q >> 2][q & 3] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fc.a[q >> 2], fc.b[q & 3],
                                                                      acc[q >> 2][q & 3], 0, 0, 0);
        const bool reads = st == 1 || (st == 6 && !last);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (reads) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (reads) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };
  for (int64_t c = 0; c + 1 < nchunks; ++c) chunk(c, false);
  chunk(nchunks - 1, true);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");       // nothing may still be writing LDS

  const float scale = alpha_a[0] * alpha_b[0];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int64_t col = n0 + 32 * j + r;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int64_t row = m0 + 32 * i + 8 * (v / 4) + 4 * g + (v % 4);
        if (row < M && col < N) {
          const float c = acc[i][j][v] * scale;
          if (OUTF32)
            static_cast<float *>(out)[row * N + col] = c;
          else
            static_cast<uint16_t *>(out)[row * N + col] = (uint16_t)pack_bf16x2(c, 0.0f);
        }
      }
    }
}

// ----------------------------------------------------------------------------------------
// Few rows of A (a small batch of activations against a weight matrix; the entry point says
// how few).  The product
// is then bound by reading B once from HBM -- which is where four-bit operands pay on this
// chip: 0.5625 bytes per weight instead of 2 -- so the plan changes: every workgroup owns 32
// rows of B (32 columns of C) and all of A, and its waves split the contraction axis (wave w
// takes the chunks of 256 indices with chunk % waves == w); the partial tiles are added
// through LDS at the end in a fixed order.  A is re-read by every workgroup, but it is small
// and stays in L2.
//
// The matrix instruction wants one operand row per lane, but a load instruction whose 64
// lanes address 32 different rows is 64 separate 16-byte requests, and the kernel would be
// bound by their number.  So each wave copies its chunk with asynchronous global -> LDS loads
// in which eight neighbouring lanes fetch the 128 contiguous bytes of one row, into its own
// piece of LDS, and then reads it back a row per lane (16-byte unit u of a row sits at
// position u ^ ((row >> 1) & 7), which spreads 16 rows over 16 bank groups).  With one tile of
// A there is room for two such pieces per wave and the copy of the chunk after next runs
// while a chunk is multiplied; otherwise the next chunk's copy overlaps this chunk's
// arithmetic and the other waves' work.
// MT = number of 32-row tiles of A (1, 2 or 4).  K must be a multiple of 256 and <= 2^24.
constexpr int SK = 256;          // contraction indices per chunk
// Waves per workgroup and staging pieces per wave, for 1, 2 and 4 tiles of A.  Four waves were
// fastest on every weight shape timed (8192 x 8192, 28672 x 8192, 8192 x 28672, 4096 x 4096;
// 2 to 10 waves and 1 to 4 pieces were tried): with one tile of A the workgroup then needs
// 72 KiB of LDS and two of them share a compute unit, so one's start and end overlap the
// other's stream.
constexpr int kSkinnyShape[3][2] = {{4, 2}, {4, 1}, {4, 1}};
constexpr int skinny_waves(int mt) { return kSkinnyShape[mt == 1 ? 0 : mt == 2 ? 1 : 2][0]; }
constexpr int skinny_stages(int mt) { return kSkinnyShape[mt == 1 ? 0 : mt == 2 ? 1 : 2][1]; }
constexpr uint32_t skinny_rows(int mt) { return 32u + 32u * mt; }        // B rows, then A rows
constexpr uint32_t skinny_scale_rows(int mt) { return (skinny_rows(mt) + 63u) / 64u * 64u; }
constexpr uint32_t skinny_stage_bytes(int mt) {
  return skinny_rows(mt) * 128u + skinny_scale_rows(mt) * 16u;
}
constexpr size_t skinny_lds_bytes(int mt) {
  const size_t stages = (size_t)skinny_waves(mt) * skinny_stages(mt) * skinny_stage_bytes(mt);
  const size_t partials = (size_t)(skinny_waves(mt) - 1) * mt * 16 * 64 * sizeof(float);
  return stages > partials ? stages : partials;
}

static_assert(skinny_lds_bytes(1) <= 160 * 1024 && skinny_lds_bytes(2) <= 160 * 1024 &&
              skinny_lds_bytes(4) <= 160 * 1024, "the stages must fit the LDS");

template <int MT, bool OUTF32>
__global__ __launch_bounds__(64 * skinny_waves(MT)) void k_gemm_skinny(
    const uint8_t *__restrict__ codes_a, const uint8_t *__restrict__ scales_a,
    const float *__restrict__ alpha_a, const uint8_t *__restrict__ codes_b,
    const uint8_t *__restrict__ scales_b, const float *__restrict__ alpha_b,
    void *__restrict__ out, int64_t M, int64_t N, int64_t K, uint32_t sha, uint32_t shb,
    uint32_t slabs) {
  constexpr int W = skinny_waves(MT), NST = skinny_stages(MT);
  constexpr uint32_t ROWS = skinny_rows(MT), STAGE = skinny_stage_bytes(MT);
  constexpr int NC = ROWS / 8, NS = skinny_scale_rows(MT) / 64;   // copy instructions per chunk
  extern __shared__ __align__(16) uint8_t lds_raw[];
  const uint32_t t = threadIdx.x, lane = t & 63u;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const uint32_t r = lane & 31u, g = lane >> 5;
  // More than 32 MT rows of A are handled in slabs of 32 MT rows, each by a workgroup of its own.
  // Workgroups go to the chip's eight dies in turn and each die has its own L2, so the slabs
  // of one 32-column strip are consecutive workgroups of one die: B is fetched into one L2.
  const uint32_t xcd = blockIdx.x & 7u, seq = blockIdx.x >> 3;
  const uint32_t slab = seq % slabs, strip = (seq / slabs) * 8 + xcd;
  const int64_t n0 = (int64_t)strip * 32;
  if (n0 >= N) return;                                   // padding of the grid to whole turns
  const int64_t row_codes = K / 2, row_scales = K / 16;
  const int64_t m0 = (int64_t)slab * (32 * MT);
  codes_a += m0 * row_codes;
  scales_a += (m0 >> sha) * row_scales;
  M -= m0;                                               // rows left from this slab's first on
  const uint8_t *wl = lds_raw + wave * (NST * STAGE);
  const uint32_t lds_wave = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)lds_raw +
                            wave * (NST * STAGE);

  // ---- copy instructions.  Codes: instruction q moves rows 8q .. 8q+7 of the stage, lane l
  // the 16-byte unit (l & 7) ^ ((row >> 1) & 7) of row 8q + l / 8; rows 0-31 are B's, the rest
  // A's (rows past the end of an operand re-read its last row).  Scales: one lane per row.
  auto uniform = [](const uint8_t *p) {
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const uint8_t *>(((uint64_t)hi << 32) | lo);
  };
  const int64_t b_base = n0 < N ? n0 : N - 1;
  const uint8_t *gcb = uniform(codes_b + b_base * row_codes), *gca = uniform(codes_a);
  uint32_t oc[NC];
#pragma unroll
  for (int q = 0; q < NC; ++q) {
    const uint32_t row = 8 * q + (lane >> 3), unit = (lane & 7u) ^ ((row >> 1) & 7u);
    int64_t line;
    if (q < 4) line = b_base + row < N ? row : N - 1 - b_base;       // relative to b_base
    else line = (int64_t)(row - 32) < M ? row - 32 : M - 1;
    oc[q] = (uint32_t)(line * row_codes) + unit * 16;
  }
  const uint8_t *ps[NS];
#pragma unroll
  for (int j = 0; j < NS; ++j) {
    const uint32_t row = 64 * j + lane;
    if (row < 32) {
      const int64_t n = n0 + row < N ? n0 + row : N - 1;
      ps[j] = scales_b + (n >> shb) * row_scales;
    } else {
      const int64_t m = (int64_t)(row - 32) < M ? row - 32 : M - 1;
      ps[j] = scales_a + (m >> sha) * row_scales;
    }
  }
  auto copy_chunk = [&](int64_t c, uint32_t stage) {
    const int64_t cc = c < K / SK ? c : K / SK - 1;                  // past the end: a harmless re-read
    const uint32_t lds = lds_wave + stage * STAGE;
    const uint8_t *pb = gcb + cc * (SK / 2), *pa = gca + cc * (SK / 2);
#pragma unroll
    for (int q = 0; q < NC; ++q) {
      if (q < 4) NV_DMA16(lds + q * 1024, oc[q], pb);
      else NV_DMA16(lds + q * 1024, oc[q], pa);
    }
#pragma unroll
    for (int j = 0; j < NS; ++j) {
      const uint8_t *src = ps[j] + cc * (SK / 16);
      asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off"
                   :: "s"(lds + ROWS * 128 + j * 1024), "v"(src) : "memory", "m0");
    }
  };
  constexpr int kCopies = NC + NS;

  // one chunk of one operand row as the lane holds it: 128 codes and their 8 scales, the
  // scales already as FP16 bit patterns (byte << 7), two per word
  struct Raw {
    uint4 c[4];
    uint32_t s[4];
  };
  const uint32_t swz = (r >> 1) & 7u;
  auto read_tile = [&](uint32_t stage, int u, Raw &x) {             // u = 0: B, 1..MT: tiles of A
    const uint8_t *st = wl + stage * STAGE;
    const uint32_t row = 32 * u + r;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      x.c[q] = *reinterpret_cast<const uint4 *>(st + row * 128 + (((4 * g + q) ^ swz) * 16));
    const uint2 sc = *reinterpret_cast<const uint2 *>(st + ROWS * 128 + row * 16 + 8 * g);
    x.s[0] = __builtin_amdgcn_perm(0u, sc.x, 0x0c010c00u) << 7;
    x.s[1] = __builtin_amdgcn_perm(0u, sc.x, 0x0c030c02u) << 7;
    x.s[2] = __builtin_amdgcn_perm(0u, sc.y, 0x0c010c00u) << 7;
    x.s[3] = __builtin_amdgcn_perm(0u, sc.y, 0x0c030c02u) << 7;
  };
  // the eight codes of matrix step s (0..15) of the chunk, expanded with their block's scale
  auto expand = [&](const Raw &x, int s) {
    const uint4 &q = x.c[s >> 2];
    const uint32_t w = (s & 3) == 0 ? q.x : (s & 3) == 1 ? q.y : (s & 3) == 2 ? q.z : q.w;
    const h2 pair = __builtin_bit_cast(h2, x.s[s >> 2]);          // blocks 2 (s / 4) and + 1
    return expand8(w, (s & 2) ? pair.y : pair.x);                  // block s / 2 of the lane's eight
  };

  f32x16 acc[MT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.0f;

  // The wave's chunks are wave, wave + W, ...  Copies are counted by hand (the kernel issues no
  // other vector-memory loads in the loop): before a stage is read, all but the copies
  // issued after it must have landed; before a stage is overwritten, its reads must be back.
  const int64_t nchunks = K / SK;
  int64_t c = wave;
#pragma unroll
  for (int p = 0; p < NST; ++p) copy_chunk(c + W * p, p);
  uint32_t stage = 0;
  while (c < nchunks) {
    // all but the copies of the NST - 1 younger stages must have landed
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"((NST - 1) * kCopies) : "memory");
    Raw rb, ra[MT];
    read_tile(stage, 0, rb);
#pragma unroll
    for (int i = 0; i < MT; ++i) read_tile(stage, 1 + i, ra[i]);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    copy_chunk(c + W * NST, stage);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int s = 0; s < 16; ++s) {
      const h8 fb = expand(rb, s);
#pragma unroll
      for (int i = 0; i < MT; ++i)
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(expand(ra[i], s), fb, acc[i], 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    c += W;
    stage = stage + 1 == (uint32_t)NST ? 0u : stage + 1;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");       // nothing may still be writing LDS
  __syncthreads();                                       // ... of any wave: the stages are reused

  // ---- add the waves' tiles in a fixed order (wave 0 collects), scale, store
  float (*part)[MT][16][64] = reinterpret_cast<float (*)[MT][16][64]>(lds_raw);
  if (wave > 0) {
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) part[wave - 1][i][v][lane] = acc[i][v];
  }
  __syncthreads();
  if (wave == 0) {
    const float scale = alpha_a[0] * alpha_b[0];
    const int64_t col = n0 + r;
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        float sum = acc[i][v];
#pragma unroll
        for (int w = 0; w < W - 1; ++w) sum += part[w][i][v][lane];
        const int64_t row = 32 * i + 8 * (v / 4) + 4 * g + (v % 4);
        if (row < M && col < N) {
          const float cval = sum * scale;
          if (OUTF32)
            static_cast<float *>(out)[(m0 + row) * N + col] = cval;
          else
            static_cast<uint16_t *>(out)[(m0 + row) * N + col] = (uint16_t)pack_bf16x2(cval, 0.0f);
        }
      }
  }
}

// ----------------------------------------------------------------------------------------
// At most 16 rows of A (a decoding batch): the same plan with the 16x16x32 matrix instruction.
// A's tile is 16 rows, so half as much of A is copied, read back and expanded per workgroup,
// and the two 16-column halves of the workgroup's 32 columns of C share each expanded
// fragment of A; per 32 contraction indices a wave issues three expansions and two 4-pass
// matrix instructions where the 32-row plan issues four and two 8-pass ones.
//
// Stage layout per wave: rows 0-31 B, rows 32-47 A (128 code bytes each, 16-byte units
// swizzled as above), then 64 scale lines of 16 bytes (lines 48-63 repeat A's last row).
// Lane l holds row l % 16 of a tile and the 64 codes 64 g .. 64 g + 63 of the chunk,
// g = l / 16 (two 16-byte units); matrix step s (0..7) multiplies codes 64 g + 8 s .. + 7 of
// every lane group, the same for A and B, so which contraction indices meet in one
// instruction is again a permutation shared by both operands.
typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr uint32_t kSkinny16Rows = 48, kSkinny16Stage = kSkinny16Rows * 128 + 64 * 16;   // 7168
constexpr int kSkinny16Waves = 4, kSkinny16Stages = 2;
constexpr size_t kSkinny16LdsBytes = (size_t)kSkinny16Waves * kSkinny16Stages * kSkinny16Stage;
static_assert(kSkinny16LdsBytes <= 160 * 1024 && kSkinny16Stages >= 1, "stages must fit the LDS");
static_assert((size_t)(kSkinny16Waves - 1) * 2 * 4 * 64 * sizeof(float) <= kSkinny16LdsBytes,
              "the partial sums reuse the stages");

template <bool OUTF32>
__global__ __launch_bounds__(64 * kSkinny16Waves) void k_gemm_skinny16(
    const uint8_t *__restrict__ codes_a, const uint8_t *__restrict__ scales_a,
    const float *__restrict__ alpha_a, const uint8_t *__restrict__ codes_b,
    const uint8_t *__restrict__ scales_b, const float *__restrict__ alpha_b,
    void *__restrict__ out, int64_t M, int64_t N, int64_t K, uint32_t sha, uint32_t shb) {
  constexpr int W = kSkinny16Waves, NST = kSkinny16Stages;
  constexpr uint32_t ROWS = kSkinny16Rows, STAGE = kSkinny16Stage;
  constexpr int NC = ROWS / 8;                                     // code copies per chunk
  extern __shared__ __align__(16) uint8_t lds_raw[];
  const uint32_t t = threadIdx.x, lane = t & 63u;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const uint32_t rr = lane & 15u, g = lane >> 4;
  const int64_t n0 = (int64_t)blockIdx.x * 32;
  const int64_t row_codes = K / 2, row_scales = K / 16;
  const uint8_t *wl = lds_raw + wave * (NST * STAGE);
  const uint32_t lds_wave = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)lds_raw +
                            wave * (NST * STAGE);

  auto uniform = [](const uint8_t *p) {
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const uint8_t *>(((uint64_t)hi << 32) | lo);
  };
  const int64_t b_base = n0 < N ? n0 : N - 1;
  const uint8_t *gcb = uniform(codes_b + b_base * row_codes), *gca = uniform(codes_a);
  uint32_t oc[NC];
#pragma unroll
  for (int q = 0; q < NC; ++q) {
    const uint32_t row = 8 * q + (lane >> 3), unit = (lane & 7u) ^ ((row >> 1) & 7u);
    int64_t line;
    if (q < 4) line = b_base + row < N ? row : N - 1 - b_base;       // relative to b_base
    else line = (int64_t)(row - 32) < M ? row - 32 : M - 1;
    oc[q] = (uint32_t)(line * row_codes) + unit * 16;
  }
  const uint8_t *ps;
  if (lane < 32) {
    const int64_t n = n0 + lane < N ? n0 + lane : N - 1;
    ps = scales_b + (n >> shb) * row_scales;
  } else {
    const int64_t m = (int64_t)(lane - 32) < M ? lane - 32 : M - 1;
    ps = scales_a + (m >> sha) * row_scales;
  }
  auto copy_chunk = [&](int64_t c, uint32_t stage) {
    const int64_t cc = c < K / SK ? c : K / SK - 1;                  // past the end: a harmless re-read
    const uint32_t lds = lds_wave + stage * STAGE;
    const uint8_t *pb = gcb + cc * (SK / 2), *pa = gca + cc * (SK / 2);
#pragma unroll
    for (int q = 0; q < NC; ++q) {
      if (q < 4) NV_DMA16(lds + q * 1024, oc[q], pb);
      else NV_DMA16(lds + q * 1024, oc[q], pa);
    }
    const uint8_t *src = ps + cc * (SK / 16);
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off"
                 :: "s"(lds + ROWS * 128), "v"(src) : "memory", "m0");
  };
  constexpr int kCopies = NC + 1;

  // a lane's share of one operand row for one chunk: 64 codes and the scales of their four
  // blocks as FP16 bit patterns (byte << 7), two per word
  struct Raw {
    uint4 c[2];
    uint32_t s[2];
  };
  auto read_tile = [&](uint32_t stage, uint32_t first_row, Raw &x) {
    const uint8_t *st = wl + stage * STAGE;
    const uint32_t row = first_row + rr, swz = (row >> 1) & 7u;
#pragma unroll
    for (int q = 0; q < 2; ++q)
      x.c[q] = *reinterpret_cast<const uint4 *>(st + row * 128 + (((2 * g + q) ^ swz) * 16));
    const uint32_t sc = *reinterpret_cast<const uint32_t *>(st + ROWS * 128 + row * 16 + 4 * g);
    x.s[0] = __builtin_amdgcn_perm(0u, sc, 0x0c010c00u) << 7;
    x.s[1] = __builtin_amdgcn_perm(0u, sc, 0x0c030c02u) << 7;
  };
  auto expand = [&](const Raw &x, int s) {                         // matrix step s = 0..7
    const uint4 &q = x.c[s >> 2];
    const uint32_t w = (s & 3) == 0 ? q.x : (s & 3) == 1 ? q.y : (s & 3) == 2 ? q.z : q.w;
    const h2 pair = __builtin_bit_cast(h2, x.s[s >> 2]);            // blocks 4 g + 2 (s / 4), + 1
    return expand8(w, (s & 2) ? pair.y : pair.x);                    // block 4 g + s / 2
  };

  f32x4 acc[2];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int v = 0; v < 4; ++v) acc[j][v] = 0.0f;

  const int64_t nchunks = K / SK;
  int64_t c = wave;
#pragma unroll
  for (int p = 0; p < NST; ++p) copy_chunk(c + W * p, p);
  uint32_t stage = 0;
  while (c < nchunks) {
    // all but the copies of the NST - 1 younger stages must have landed
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"((NST - 1) * kCopies) : "memory");
    Raw ra, rb[2];
    read_tile(stage, 32, ra);
    read_tile(stage, 0, rb[0]);
    read_tile(stage, 16, rb[1]);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    copy_chunk(c + NST * W, stage);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const h8 fa = expand(ra, s);
#pragma unroll
      for (int j = 0; j < 2; ++j)
        acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fa, expand(rb[j], s), acc[j], 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    c += W;
    stage = stage + 1 == (uint32_t)NST ? 0u : stage + 1;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");       // nothing may still be writing LDS
  __syncthreads();                                       // ... of any wave: the stages are reused

  // ---- add the waves' tiles in a fixed order (wave 0 collects), scale, store
  float (*part)[2][4][64] = reinterpret_cast<float (*)[2][4][64]>(lds_raw);
  if (wave > 0) {
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) part[wave - 1][j][v][lane] = acc[j][v];
  }
  __syncthreads();
  if (wave == 0) {
    const float scale = alpha_a[0] * alpha_b[0];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        float sum = acc[j][v];
#pragma unroll
        for (int w = 0; w < W - 1; ++w) sum += part[w][j][v][lane];
        const int64_t row = 4 * g + v, col = n0 + 16 * j + rr;
        if (row < M && col < N) {
          const float cval = sum * scale;
          if (OUTF32)
            static_cast<float *>(out)[row * N + col] = cval;
          else
            static_cast<uint16_t *>(out)[row * N + col] = (uint16_t)pack_bf16x2(cval, 0.0f);
        }
      }
  }
}

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// The kernels compile side by side when this file is built in parts: NVFP4_46_GEMM_PART =
// 1..4 hold one instantiation of the staged kernel each (by far the slowest to compile),
// 5 the copy-based kernel, 6 the small-batch kernel, 0 the entry point; without the macro
// the file is one self-contained translation unit.
#ifndef NVFP4_46_GEMM_PART
#define NVFP4_46_GEMM_PART (-1)
#endif
#define NVFP4_46_GEMM_HAS(part) (NVFP4_46_GEMM_PART < 0 || NVFP4_46_GEMM_PART == (part))

struct GemmArgs {
  const uint8_t *codes_a, *scales_a;
  const float *alpha_a;
  const uint8_t *codes_b, *scales_b;
  const float *alpha_b;
  void *out;
  int64_t M, N, K;
  uint32_t sha, shb;     // scale rows are shared by 2^sha rows of A, 2^shb rows of B
  bool f32;              // C is fp32 instead of BF16
  hipStream_t stream;
};

// Every run_* raises the kernel's dynamic LDS limit (all three need more than the 64 KiB a
// kernel gets without asking), launches, and returns a status of the C ABI.
template <bool KFULL, bool OUTF32>
int run_gemm_staged(const GemmArgs &a);
int run_gemm_dma(const GemmArgs &a);
int run_gemm_skinny(const GemmArgs &a);

template <typename Kernel, typename... Args>
static int launch_with_lds(Kernel kernel, dim3 grid, dim3 block, size_t lds_bytes, hipStream_t s,
                           Args... args) {
  if (hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                          hipFuncAttributeMaxDynamicSharedMemorySize,
                          (int)lds_bytes) != hipSuccess) {
    return NVFP4_ERR_HIP;
  }
  return launch(kernel, grid, block, lds_bytes, s, args...);
}

static dim3 tile_grid(const GemmArgs &a) {
  const int64_t tiles_m = (a.M + GT - 1) / GT, tiles_n = (a.N + GT - 1) / GT;
  return dim3((uint32_t)(tiles_m * tiles_n));
}

template <bool KFULL, bool OUTF32>
int run_gemm_staged(const GemmArgs &a) {
  return launch_with_lds(k_gemm<KFULL, OUTF32>, tile_grid(a), dim3(kGemmThreads), kGemmLdsBytes,
                         a.stream, a.codes_a, a.scales_a, a.alpha_a, a.codes_b, a.scales_b,
                         a.alpha_b, a.out, a.M, a.N, a.K, (uint32_t)((a.N + GT - 1) / GT), a.sha,
                         a.shb);
}
#if NVFP4_46_GEMM_PART == 0
extern template int run_gemm_staged<false, false>(const GemmArgs &);
extern template int run_gemm_staged<false, true>(const GemmArgs &);
extern template int run_gemm_staged<true, false>(const GemmArgs &);
extern template int run_gemm_staged<true, true>(const GemmArgs &);
#elif NVFP4_46_GEMM_PART >= 1 && NVFP4_46_GEMM_PART <= 4
template int run_gemm_staged<((NVFP4_46_GEMM_PART - 1) / 2 != 0), ((NVFP4_46_GEMM_PART - 1) % 2 != 0)>(
    const GemmArgs &);
#endif

#if NVFP4_46_GEMM_HAS(5)
int run_gemm_dma(const GemmArgs &a) {
  const uint32_t tiles_n = (uint32_t)((a.N + GT - 1) / GT);
  auto go = [&](auto kernel) {
    return launch_with_lds(kernel, tile_grid(a), dim3(kGemmThreads), kGemmDmaLdsBytes, a.stream,
                           a.codes_a, a.scales_a, a.alpha_a, a.codes_b, a.scales_b, a.alpha_b,
                           a.out, a.M, a.N, a.K, tiles_n, a.sha, a.shb);
  };
  return a.f32 ? go(k_gemm_dma<true>) : go(k_gemm_dma<false>);
}
#endif

#if NVFP4_46_GEMM_HAS(6)
// Few rows of A: one workgroup per 32 columns of C, bound by streaming B.
int run_gemm_skinny(const GemmArgs &a) {
  auto go = [&](auto kernel, int mt) {
    const int64_t slabs = (a.M + 32 * mt - 1) / (32 * mt), strips = (a.N + 31) / 32;
    const int64_t grid = (strips + 7) / 8 * 8 * slabs;      // whole turns over the eight dies
    return launch_with_lds(kernel, dim3((uint32_t)grid), dim3(64 * skinny_waves(mt)),
                           skinny_lds_bytes(mt), a.stream, a.codes_a, a.scales_a, a.alpha_a,
                           a.codes_b, a.scales_b, a.alpha_b, a.out, a.M, a.N, a.K, a.sha, a.shb,
                           (uint32_t)slabs);
  };
  if (a.M <= 16) {
    auto go16 = [&](auto kernel) {
      return launch_with_lds(kernel, dim3((uint32_t)((a.N + 31) / 32)), dim3(64 * kSkinny16Waves),
                             kSkinny16LdsBytes, a.stream, a.codes_a, a.scales_a, a.alpha_a,
                             a.codes_b, a.scales_b, a.alpha_b, a.out, a.M, a.N, a.K, a.sha, a.shb);
    };
    return a.f32 ? go16(k_gemm_skinny16<true>) : go16(k_gemm_skinny16<false>);
  }
  if (a.M <= 32) return a.f32 ? go(k_gemm_skinny<1, true>, 1) : go(k_gemm_skinny<1, false>, 1);
  if (a.M <= 64) return a.f32 ? go(k_gemm_skinny<2, true>, 2) : go(k_gemm_skinny<2, false>, 2);
  return a.f32 ? go(k_gemm_skinny<4, true>, 4) : go(k_gemm_skinny<4, false>, 4);
}
#endif

}  // namespace nvfp4_46

#if NVFP4_46_GEMM_PART <= 0

using namespace nvfp4_46;

extern "C" int nvfp4_46_gemm(const void *codes_a, const void *scales_a, const float *alpha_a,
                             const void *codes_b, const void *scales_b, const float *alpha_b,
                             int64_t M, int64_t N, int64_t K, uint32_t out_dtype, uint32_t flags,
                             void *out, void *stream) {
  if (!codes_a || !scales_a || !alpha_a || !codes_b || !scales_b || !alpha_b || !out)
    return NVFP4_ERR_NULL;
  if (M <= 0 || N <= 0 || K <= 0 || (K % 32) != 0) return NVFP4_ERR_SHAPE;
  if (M > (int64_t)1 << 31 || N > (int64_t)1 << 31 || K > (int64_t)1 << 31 ||
      M * K > (int64_t)1 << 40 || N * K > (int64_t)1 << 40 || M * N > (int64_t)1 << 40)
    return NVFP4_ERR_SHAPE;
  if (out_dtype > NVFP4_OUT_F32 || flags > (NVFP4_GEMM_A_TILE_SCALES | NVFP4_GEMM_B_TILE_SCALES))
    return NVFP4_ERR_PARAM;
  if (((flags & NVFP4_GEMM_A_TILE_SCALES) && (M % 16) != 0) ||
      ((flags & NVFP4_GEMM_B_TILE_SCALES) && (N % 16) != 0))
    return NVFP4_ERR_SHAPE;
  if (!aligned16(codes_a) || !aligned16(scales_a) || !aligned16(codes_b) || !aligned16(scales_b) ||
      !aligned16(out))
    return NVFP4_ERR_ALIGN;
  const int64_t tiles_m = (M + GT - 1) / GT, tiles_n = (N + GT - 1) / GT;
  if (tiles_m * tiles_n > (int64_t)1 << 30) return NVFP4_ERR_SHAPE;
  const GemmArgs a{static_cast<const uint8_t *>(codes_a), static_cast<const uint8_t *>(scales_a),
                   alpha_a, static_cast<const uint8_t *>(codes_b),
                   static_cast<const uint8_t *>(scales_b), alpha_b, out, M, N, K,
                   (flags & NVFP4_GEMM_A_TILE_SCALES) ? 4u : 0u,
                   (flags & NVFP4_GEMM_B_TILE_SCALES) ? 4u : 0u, out_dtype == NVFP4_OUT_F32,
                   static_cast<hipStream_t>(stream)};
  const bool offsets_fit = K <= ((int64_t)1 << 24);     // 32-bit lane offsets of the copies
  // The kernel that streams B takes up to 128 rows of A at its best and, in slabs of 128 rows,
  // up to 512 as long as the 128 x 128 tiles of the other kernels would not even fill the
  // chip's 256 compute units once (timed on 8192 x 8192, 28672 x 8192, 8192 x 28672 and
  // 4096 x 4096 weights: with fewer tiles than that, those kernels wait on HBM chunk by chunk).
  const bool few_rows = M <= 128 || (M <= 512 && tiles_m * tiles_n <= 256);
  if (few_rows && (K % SK) == 0 && offsets_fit) return run_gemm_skinny(a);
  // K a multiple of 128: the variant with asynchronous global -> LDS copies
  if ((K % GK) == 0 && offsets_fit) return run_gemm_dma(a);
  if ((K % GK) == 0)
    return a.f32 ? run_gemm_staged<true, true>(a) : run_gemm_staged<true, false>(a);
  return a.f32 ? run_gemm_staged<false, true>(a) : run_gemm_staged<false, false>(a);
}

#endif
