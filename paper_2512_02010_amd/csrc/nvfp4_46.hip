// Kernels and C ABI of libnvfp4_46.so (gfx950).  See include/nvfp4_46.h for the
// contract of every entry point.
//
// Data movement
//   rowwise   A row-major tensor whose rows are multiples of 16 is one flat
//             stream of 16-element blocks, and so are its outputs: block k reads
//             32 bytes at 32k, writes 8 code bytes at 8k and 1 scale byte at k.
//             One lane owns one block (two 128-bit loads, all 16 values in
//             registers, no cross-lane traffic); a wave's 64 lanes cover 2 KiB of
//             contiguous input, 512 B of codes and 64 B of scales.
//   columnwise / both
//             A workgroup stages a 64x128 tile of x in LDS (coalesced 128-bit
//             loads), every lane then reads two adjacent columns x 16 rows from
//             LDS, and the results go back through LDS so that each column's 32
//             code bytes leave as one contiguous run.  When both orientations
//             are wanted the rowwise half is produced from the registers of the
//             staging loads, so x is read from HBM once.
#include <hip/hip_runtime.h>

#include <mutex>

#include "block.hpp"
#include "launch.hpp"
#include "nvfp4_46.h"

// The quantizing kernels exist once per (input type, rounding mode, selection rule, ...):
// several hundred instantiations.  To compile them side by side this file can be built in
// parts: NVFP4_46_PART = 1..6 holds the kernels of one (input type, rounding mode) pair and
// nothing else, NVFP4_46_PART = 0 holds everything else (the entry points included) and
// refers to the six groups as explicit instantiations defined elsewhere.  Without the
// macro the file is one self-contained translation unit.
#ifndef NVFP4_46_PART
#define NVFP4_46_PART (-1)
#endif
#define NVFP4_46_MAIN (NVFP4_46_PART <= 0)

namespace nvfp4_46 {

constexpr int kThreads = 256;
enum : int { kOutCodes = 0, kOutFake = 1, kOutAmax = 2 };

// Launch shapes (workgroups per compute unit; every kernel strides over its input).  Each
// value is the fastest of a timed sweep on 8192 x 8192 tensors.
constexpr int kAmaxUnroll = 8;          // independent 128-bit loads per lane in k_amax_plain
constexpr int kAmaxWgPerCu = 1;         // k_amax_plain: few, long-lived workgroups, each ends
                                        // with a serialising access to the one result word
constexpr int kFlatLongWgPerCu = 6;     // k_flat with outputs: long-lived workgroups (5 ... 8
                                        // timed; 8 leaves no slot for the short ones)
constexpr int kFlatShortRoundsPerCu = 16;  // ... and rounds left to one-round workgroups
constexpr int kFlatAmaxWgPerCu = 2;     // k_flat as the amax pass of the Hadamard transform
constexpr int kAmaxRhtColWgPerCu = 8;   // k_amax_rht_col

// Streaming accesses.  Dequantized BF16 tensors are write-once streams and leave with
// nontemporal stores (dequantize 45 -> 28 us per 8192 x 8192, and their write-back no
// longer competes with the next kernel).  Codes, scales and choice bytes use ordinary
// stores so that the consumer finds them in L2 / the memory-side cache (nontemporal
// stores gain 1.5 us here and cost the following dequantize 4-5 us).  Loads are ordinary
// (nontemporal loads are slower when x is cache-resident and neutral otherwise).
constexpr bool kNtCodes = false;   // codes / scales / choice bytes
constexpr bool kNtBf16 = true;     // dequantized BF16 tensors
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

NV_DEV uint4 load_stream(const uint4 *p) { return *p; }
template <bool NT>
NV_DEV void store_as(uint4 *p, const uint4 &v) {
  if (NT) {
    u32x4 t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, reinterpret_cast<u32x4 *>(p));
  } else {
    *p = v;
  }
}
template <bool NT>
NV_DEV void store_as(uint2 *p, const uint2 &v) {
  if (NT) {
    u32x2 t = {v.x, v.y};
    __builtin_nontemporal_store(t, reinterpret_cast<u32x2 *>(p));
  } else {
    *p = v;
  }
}
template <bool NT>
NV_DEV void store_as(uint8_t *p, uint8_t v) {
  if (NT)
    __builtin_nontemporal_store(v, p);
  else
    *p = v;
}

NV_DEV void unpack16(const uint4 &w0, const uint4 &w1, float (&v)[16]) {
  const uint32_t w[8] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w};
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    v[2 * j] = bf16_lo(w[j]);
    v[2 * j + 1] = bf16_hi(w[j]);
  }
}

// A block as it arrives from memory: two 128-bit pieces of BF16 or four of fp32.
template <bool XF32>
struct RawBlock {
  static constexpr int kPieces = XF32 ? 4 : 2;
  uint4 w[kPieces];
};
template <bool XF32>
NV_DEV void load_block(const uint4 *p, RawBlock<XF32> &r) {
#pragma unroll
  for (int j = 0; j < RawBlock<XF32>::kPieces; ++j) r.w[j] = load_stream(p + j);
}
template <bool XF32>
NV_DEV void unpack16(const RawBlock<XF32> &r, float (&v)[16]) {
  if constexpr (XF32) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      v[4 * j] = u2f(r.w[j].x);
      v[4 * j + 1] = u2f(r.w[j].y);
      v[4 * j + 2] = u2f(r.w[j].z);
      v[4 * j + 3] = u2f(r.w[j].w);
    }
  } else {
    unpack16(r.w[0], r.w[1], v);
  }
}

NV_DEV float wave_max(float m) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
  return m;
}

// Where a reduction kernel leaves its result.  Plain form (scratch == nullptr): `amax_bits` is
// the caller's alpha word, zeroed by a launch before and turned into alpha by a launch after.
// One-launch form: `scratch` is zeroed scratch memory (layout below); the workgroup that
// finishes last applies Eq. (1), writes alpha, and the scratch is all zero again.
//
// Device-scope atomics on one address are carried out one after the other at the memory side
// (about 15-35 ns each here: 256 workgroups that all finish together queued up for 9 of the
// 27 us of a pass over 8192 x 8192).  So the workgroups report in a two-level tree: sixteen
// groups, each with its own maximum and ticket words on cache lines of their own, and the
// last workgroup of a group reports to the top pair.  Two chains of at most ~grid/16 + 16
// atomics replace one of 2 x grid.
struct AmaxFinish {
  uint32_t *scratch;   // kScratchWords words, or nullptr
  float *alpha;
  float fp8_max;
};
constexpr uint32_t kAmaxGroups = 16;
constexpr uint32_t kScratchStride = 32;   // words between two slots: one 128-byte line each
// slot g: maximum of group g; slot 16 + g: its ticket; slot 32: top maximum; slot 33: top ticket
constexpr uint32_t kScratchWords = (2 * kAmaxGroups + 2) * kScratchStride;
NV_DEV uint32_t *scratch_slot(uint32_t *scratch, uint32_t i) { return scratch + i * kScratchStride; }

// Eq. (1): alpha = amax / (6 * fp8_max); an all-zero tensor gets alpha = 1.
NV_DEV float alpha_of(float amax, float fp8_max) {
  return (amax == 0.0f) ? 1.0f : amax / (6.0f * fp8_max);
}

// max into *word, skipped when a plain read already shows a value at least as large (the
// value only ever grows); the returning form, waited for, so that the maximum is in before
// anything the caller does next.
NV_DEV void atomic_max_now(uint32_t *word, uint32_t bits) {
  if (bits > __hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) {
    uint32_t old = __hip_atomic_fetch_max(word, bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(old) : : "memory");
  }
}

// Fold a workgroup's maximum magnitude into the global one.  Bit patterns of non-negative
// floats order like the values, so an integer atomic max is exact and order-free.
// Device-scope atomics are carried out at the one place all compute dies share, so "carried
// out before" needs no cache maintenance, only program order: a workgroup's maximum is in
// before its ticket is drawn, and whoever draws a group's (the grid's) last ticket reads the
// maximum after that.
NV_DEV void publish_amax(float m, uint32_t *amax_bits, const AmaxFinish &fin) {
  __shared__ float wave_part[kThreads / 64];
  m = wave_max(m);
  if ((threadIdx.x & 63) == 0) wave_part[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x != 0) return;
#pragma unroll
  for (int w = 1; w < kThreads / 64; ++w) m = fmaxf(m, wave_part[w]);
  const uint32_t bits = f2u(m);
  if (!fin.scratch) {
    atomic_max_now(amax_bits, bits);
    return;
  }
  const uint32_t groups = gridDim.x < kAmaxGroups ? gridDim.x : kAmaxGroups;
  const uint32_t g = blockIdx.x % groups;
  const uint32_t members = (gridDim.x - g + groups - 1) / groups;     // workgroups b with b % groups == g
  uint32_t *gmax = scratch_slot(fin.scratch, g), *gticket = scratch_slot(fin.scratch, kAmaxGroups + g);
  uint32_t *top = scratch_slot(fin.scratch, 2 * kAmaxGroups), *top_ticket = scratch_slot(fin.scratch, 2 * kAmaxGroups + 1);
  atomic_max_now(gmax, bits);
  if (__hip_atomic_fetch_add(gticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != members - 1) return;
  // last of its group: hand the group's maximum on and leave the group's words zero
  const uint32_t group_bits = __hip_atomic_exchange(gmax, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __hip_atomic_store(gticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  atomic_max_now(top, group_bits);
  if (__hip_atomic_fetch_add(top_ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != groups - 1) return;
  const uint32_t all = __hip_atomic_exchange(top, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __hip_atomic_store(top_ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  *fin.alpha = alpha_of(u2f(all), fin.fp8_max);
}

// ------------------------------------------------------------ tensor scale

#if NVFP4_46_MAIN
__global__ void k_store_u32(uint32_t *p, uint32_t v) { *p = v; }

__global__ void k_finish_alpha(float *alpha, float fp8_max) { *alpha = alpha_of(*alpha, fp8_max); }
#endif

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

// max|x| without the transform: compare magnitudes as integers (15 bits of a BF16 value, 31
// of an fp32 value).  Several independent 128-bit loads per lane are in flight at a time.
template <bool XF32>
__global__ __launch_bounds__(kThreads) void k_amax_plain(const uint4 *__restrict__ x, int64_t n16,
                                                         uint32_t *amax_bits, AmaxFinish fin) {
  u16x2 acc = {0, 0};
  uint32_t acc32 = 0;
  auto fold = [&](const uint4 &w) {
    const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if constexpr (XF32) {
        const uint32_t m = ww[j] & 0x7fffffffu;
        acc32 = m > acc32 ? m : acc32;
      } else {
        uint32_t m = ww[j] & 0x7fff7fffu;
        acc = __builtin_elementwise_max(acc, *reinterpret_cast<u16x2 *>(&m));
      }
    }
  };
  constexpr int U = kAmaxUnroll;
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  for (; i + (U - 1) * stride < n16; i += U * stride) {
    uint4 w[U];
#pragma unroll
    for (int j = 0; j < U; ++j) w[j] = load_stream(x + i + j * stride);
#pragma unroll
    for (int j = 0; j < U; ++j) fold(w[j]);
  }
  for (; i < n16; i += stride) fold(load_stream(x + i));
  const uint32_t top = XF32 ? acc32 : (uint32_t)(acc.x > acc.y ? acc.x : acc.y) << 16;
  publish_amax(u2f(top), amax_bits, fin);
}

// max|y| over the Hadamard-transformed column blocks (16 consecutive rows of one column),
// without LDS: a lane loads one 16-byte piece from each of the 16 rows of a row block -- 8
// BF16 or 4 fp32 columns, a wave's loads cover 1 KiB of each row -- and transforms every
// column in registers.  The signs depend on the row only, so they are flipped in the packed
// words; the factor 1/4 of the transform is applied once to the maximum (scaling by a power
// of two is monotonic, so the maximum of the scaled values is the scaled maximum).
template <bool XF32>
__global__ __launch_bounds__(kThreads) void k_amax_rht_col(const uint4 *__restrict__ x,
                                                           int64_t row_blocks, int64_t pieces_per_row,
                                                           uint64_t rht_seed, uint32_t *amax_bits,
                                                           AmaxFinish fin) {
  const int64_t items = row_blocks * pieces_per_row;
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  float m = 0.0f;
  for (int64_t item = (int64_t)blockIdx.x * kThreads + threadIdx.x; item < items; item += stride) {
    const int64_t rb = item / pieces_per_row, piece = item - rb * pieces_per_row;
    const uint4 *src = x + rb * 16 * pieces_per_row + piece;
    uint4 w[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) w[j] = load_stream(src + j * pieces_per_row);
    const uint32_t sw = rht_sign_word(rht_seed, (uint64_t)rb);
    constexpr uint32_t kSignBits = XF32 ? 0x80000000u : 0x80008000u;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const uint32_t flip = (0u - ((sw >> j) & 1u)) & kSignBits;    // row j of the block
      w[j].x ^= flip;
      w[j].y ^= flip;
      w[j].z ^= flip;
      w[j].w ^= flip;
    }
#pragma unroll
    for (int c = 0; c < (XF32 ? 4 : 8); ++c) {
      float v[16];
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        if constexpr (XF32) {
          v[j] = u2f(c == 0 ? w[j].x : c == 1 ? w[j].y : c == 2 ? w[j].z : w[j].w);
        } else {
          const uint32_t word = (c >> 1) == 0 ? w[j].x : (c >> 1) == 1 ? w[j].y
                              : (c >> 1) == 2 ? w[j].z : w[j].w;
          v[j] = u2f((c & 1) ? (word & 0xffff0000u) : (word << 16));
        }
      }
      // the butterflies of rht16() (strides 1, 2, 4, 8), signs already applied, no scaling
#pragma unroll
      for (int h = 1; h < 16; h <<= 1) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          if ((i & h) == 0) {
            const float a = v[i], b = v[i + h];
            v[i] = a + b;
            v[i + h] = a - b;
          }
        }
      }
#pragma unroll
      for (int j = 0; j < 16; j += 2) m = fmaxf(m, fmaxf(fabsf(v[j]), fabsf(v[j + 1])));
    }
  }
  publish_amax(m * 0.25f, amax_bits, fin);
}

// -------------------------------------------------------- rowwise (flat)

template <bool XF32, int ROUNDING, int SELECT, bool RHT, int OUT>
__global__ __launch_bounds__(kThreads) void k_flat(
    const uint4 *__restrict__ x, const float *__restrict__ alpha_p, uint2 *__restrict__ codes,
    uint8_t *__restrict__ scales, uint8_t *__restrict__ choice, uint4 *__restrict__ out_bf16,
    uint32_t *amax_bits, int64_t nblocks, uint32_t nb_per_row, uint64_t sr_seed,
    uint64_t rht_seed, uint32_t n_long, uint32_t rounds_long, AmaxFinish fin) {
  __shared__ ScaleTable tab;
  // fake-quant only: a wave's 2 KiB of output is turned round in LDS so that each of its
  // two store instructions writes 1 KiB of whole cache lines (streaming stores of half
  // lines are slow), instead of every lane writing its own 32 bytes
  __shared__ uint4 xpose[OUT == kOutFake ? 2 * kThreads : 1];
  // The tensor is cut into rounds of 256 consecutive blocks, dealt to two classes of
  // workgroups: the first n_long workgroups take rounds_long rounds each (w, w + n_long, ...,
  // all below n_long * rounds_long), the others share the remaining rounds (one each, when
  // the launcher sizes the grid for it; in general w', w' + n_short, ...).  A workgroup pays
  // a full memory latency before its first round, with its wave slots idle: the long ones,
  // few enough to be resident all at once, pay it once for most of the tensor, and the short
  // ones, launched as slots fall free, even out the end.  Everything that depends on the
  // round only (base pointers, the number of live lanes) is wave-uniform and stays on the
  // scalar unit; a lane adds its own constant offset.
  const uint32_t tid = threadIdx.x;
  const uint32_t rounds = (uint32_t)((nblocks + kThreads - 1) / kThreads);
  const uint32_t tail = (uint32_t)(nblocks - (int64_t)(rounds - 1) * kThreads);  // 1..256
  // The sign flips of the transform as sixteen XOR masks per lane, in LDS (piece q of lane t at
  // [q][t]: a wave's 128-bit reads are conflict-free).  A lane writes and reads only its own
  // slots, and the LDS operations of one wave execute in order, so no barrier is involved.
  __shared__ uint4 sign_masks[RHT ? 4 : 1][RHT ? kThreads : 1];
  uint32_t B_lane = 0, sign_B = 0xffffffffu;
  if (RHT) B_lane = tid % nb_per_row;
  auto transform = [&](float (&w)[16]) {
    uint32_t mask[16];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const uint4 m = sign_masks[q][tid];
      mask[4 * q] = m.x;
      mask[4 * q + 1] = m.y;
      mask[4 * q + 2] = m.z;
      mask[4 * q + 3] = m.w;
    }
    rht16_masked(w, mask);
  };
  float amax = 0.0f;
  ScaleConsts sc{};

  auto lanes_in_round = [&](uint32_t r) { return (r == rounds - 1) ? tail : (uint32_t)kThreads; };

  // one block, already loaded; `live` = lanes of this round that hold a block (fewer than
  // 256 only in the last round of a ragged tensor)
  using Raw = RawBlock<XF32>;
  auto work = [&](uint32_t r, uint32_t live, const Raw &raw) {
    const int64_t base = (int64_t)r * kThreads;
    float v[16];
    uint32_t u[16];
    unpack16(raw, v);
    if (RHT) {
      // the sign word depends on the block's position in its row only; with the usual
      // shapes a lane meets the same position in every round and keeps its masks
      uint32_t B = (uint32_t)(base % nb_per_row) + B_lane;
      if (B >= nb_per_row) B -= nb_per_row;
      if (B != sign_B) {
        sign_B = B;
        uint32_t mask[16];
        rht_sign_masks(rht_sign_word(rht_seed, B), mask);
#pragma unroll
        for (int q = 0; q < 4; ++q)
          sign_masks[q][tid] = make_uint4(mask[4 * q], mask[4 * q + 1], mask[4 * q + 2], mask[4 * q + 3]);
      }
      transform(v);
    }
    if (OUT == kOutAmax) {
#pragma unroll
      for (int i = 0; i < 16; ++i) amax = fmaxf(amax, fabsf(v[i]));
      return;
    }
    auto random_words = [&](uint32_t (&uu)[16]) {
      const uint64_t q0 = ((uint64_t)base + tid) * 4u;
#pragma unroll
      for (int j = 0; j < 4; ++j) sr_words4(sr_seed, q0 + j, &uu[4 * j]);
    };
    if (ROUNDING != kRTN) random_words(u);
    // the block once more, from memory (a lane without a block of its own holds a copy of
    // the round's last block, as fetch() gave it)
    auto again = [&](float (&w)[16], uint32_t (&uu)[16]) {
      Raw r2;
      load_block<XF32>(x + Raw::kPieces * (base + (tid < live ? tid : live - 1)), r2);
      unpack16(r2, w);
      if (RHT) transform(w);
      if (ROUNDING != kRTN) random_words(uu);
    };
    const BlockResult res = quantize_block<ROUNDING, SELECT>(v, u, sc, tab, again);
    if (OUT == kOutCodes) {
      store_as<kNtCodes>(codes + base + tid, make_uint2(res.lo, res.hi));
      store_as<kNtCodes>(scales + base + tid, (uint8_t)res.scale);
      if (choice) store_as<kNtCodes>(choice + base + tid, (uint8_t)res.four);
    } else {
      float D0[8], D1[8];
      dequant8(res.lo, res.dec, D0);
      dequant8(res.hi, res.dec, D1);
      // lane l of a wave holds 16-byte pieces 2l and 2l+1 of the wave's output and
      // stores pieces l and 64+l; LDS operations of one wave execute in order, so the
      // reads below see the writes above without a barrier
      const uint32_t wave0 = tid & ~63u, lane = tid & 63u;
      uint4 *slot = xpose + 2 * wave0;
      slot[2 * lane] = make_uint4(pack_bf16x2(D0[0], D0[1]), pack_bf16x2(D0[2], D0[3]),
                                  pack_bf16x2(D0[4], D0[5]), pack_bf16x2(D0[6], D0[7]));
      slot[2 * lane + 1] = make_uint4(pack_bf16x2(D1[0], D1[1]), pack_bf16x2(D1[2], D1[3]),
                                      pack_bf16x2(D1[4], D1[5]), pack_bf16x2(D1[6], D1[7]));
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      uint4 *ob = out_bf16 + 2 * (base + wave0);
      if (wave0 + (lane >> 1) < live) store_as<kNtBf16>(ob + lane, slot[lane]);
      if (wave0 + 32 + (lane >> 1) < live) store_as<kNtBf16>(ob + 64 + lane, slot[64 + lane]);
    }
  };

  // Loads run one round ahead of the arithmetic: while a wave works on one block the
  // 128-bit loads of its next block are already in flight (two register sets, used
  // alternately), so a round costs max(memory latency, arithmetic) instead of their sum.
  // The first round's loads also go out before the scale table is built.
  // In the fake-quant kernel lanes without a block still run (their results are not
  // stored), because they store pieces of their neighbours' blocks; elsewhere they skip
  // the round.
  // The loads are unconditional (a conditional load would have to be waited for right
  // where the two control paths join): a round past the workgroup's share re-reads round 0
  // (every workgroup ends with that, so the L2 serves it) and a lane past the end of a ragged
  // last round re-reads that round's last block; what they fetch is never used.
  uint32_t r, step, end;
  if (blockIdx.x < n_long) {
    r = blockIdx.x;
    step = n_long;
    end = n_long * rounds_long;
  } else {
    r = n_long * rounds_long + (blockIdx.x - n_long);
    step = gridDim.x - n_long;
    end = rounds;
  }
  auto fetch = [&](uint32_t next, Raw &raw) {
    const uint32_t rr = next < end ? next : 0u;
    const uint32_t last = lanes_in_round(rr) - 1;
    const uint32_t lane = tid < last ? tid : last;
    const uint4 *xb = x + Raw::kPieces * ((int64_t)rr * kThreads);
    load_block<XF32>(xb + Raw::kPieces * lane, raw);
  };
  auto run = [&](uint32_t r, const Raw &raw) {
    const uint32_t live = lanes_in_round(r);
    if (OUT == kOutFake || tid < live) work(r, live, raw);
  };
  Raw a, b;
  fetch(r, a);
  if (OUT != kOutAmax) sc = build_scale_table(tab, *alpha_p);
  while (r < end) {
    fetch(r + step, b);
    run(r, a);
    r += step;
    if (r >= end) break;
    fetch(r + step, a);
    run(r, b);
    r += step;
  }
  if (OUT == kOutAmax) publish_amax(amax, amax_bits, fin);
}

#if NVFP4_46_MAIN
// One lane per 8 elements: 4 code bytes + the block's scale -> 8 BF16.
__global__ __launch_bounds__(kThreads) void k_dequant_flat(const uint32_t *__restrict__ codes,
                                                           const uint8_t *__restrict__ scales,
                                                           const float *__restrict__ alpha_p,
                                                           uint4 *__restrict__ out, int64_t n8) {
  const float alpha = *alpha_p;
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x; t < n8; t += stride) {
    float dec = e4m3_decode(scales[t >> 1]) * alpha;
    float D[8];
    dequant8(codes[t], dec, D);
    store_as<kNtBf16>(out + t, make_uint4(pack_bf16x2(D[0], D[1]), pack_bf16x2(D[2], D[3]),
                                          pack_bf16x2(D[4], D[5]), pack_bf16x2(D[6], D[7])));
  }
}
#endif

// ------------------------------------------------ columnwise / both (tiled)

constexpr int TR = 64;    // tile rows    (multiple of 16)
constexpr int TC = 128;   // tile columns (multiple of 16)
constexpr int kRowBlocksPerTileRow = TC / 16;          // 16-element row blocks across a tile row
constexpr int kRowBlocksPerTile = TR * TC / 16;
constexpr int kRowBlocksPerLane = kRowBlocksPerTile / kThreads;
constexpr int kColPairs = TC / 2;                      // pairs of adjacent columns
constexpr int kColBlockRows = TR / 16;                 // 16-row blocks down a tile column
constexpr int kPairUnits = kColPairs * kColBlockRows;  // (column pair, row block) units
constexpr int kPairUnitsPerLane = kPairUnits / kThreads;
constexpr int kColItems = TC * kColBlockRows;          // (column, row block) results per tile
constexpr int kColItemsPerLane = kColItems / kThreads;
constexpr int kPieces = TR * TC / 8;                   // 128-bit pieces of a BF16 tile
constexpr int kPiecesPerLane = kPieces / kThreads;
static_assert(TR % 16 == 0 && TC % 16 == 0, "tiles are made of whole blocks both ways");
static_assert(kRowBlocksPerTile % kThreads == 0 && kPairUnits % kThreads == 0 &&
              kColItems % kThreads == 0, "tile work must divide evenly over the workgroup");

struct TileCoord {
  int64_t r0, c0;
  bool valid;
};

// Workgroups are handed to the 8 XCDs round-robin by their index, and each XCD has its own
// L2.  A tile writes only part of every output cache line it touches: 64 of the 128 bytes of
// a row's codes, 32 bytes of a column's, 8 and 4 bytes of the scale lines.  The tiles that
// complete those lines -- horizontal neighbours for the rowwise arrays, vertical neighbours
// for the columnwise ones -- should therefore meet in one L2 while the lines are still
// there.  So the tiles are grouped into super-tiles of sx x sy tiles (8 x 16 when the tensor
// is that large: 1024 x 1024 elements), super-tile S goes to XCD S % 8, and the consecutive
// workgroups of one XCD walk through one super-tile row by row.  (One XCD per tile column,
// top to bottom, merged only the columnwise lines: 66.6 -> 58.6 us for both orientations of
// 8192 x 8192.)
struct TileMap {
  uint32_t sx, sy;   // super-tile width and height in tiles
};

NV_DEV TileCoord tile_of_workgroup(int64_t rows, int64_t cols, TileMap m) {
  const uint32_t nt_r = (uint32_t)((rows + TR - 1) / TR), nt_c = (uint32_t)((cols + TC - 1) / TC);
  const uint32_t per = m.sx * m.sy, nsx = (nt_c + m.sx - 1) / m.sx;
  const uint32_t xcd = blockIdx.x & 7u, slot = blockIdx.x >> 3;
  const uint32_t round = slot / per, within = slot - round * per;
  const uint32_t S = round * 8u + xcd;                      // super-tile, row-major
  const uint32_t sy = S / nsx, sx = S - sy * nsx;
  const uint32_t wy = within / m.sx, wx = within - wy * m.sx;
  const uint32_t tr = sy * m.sy + wy, tc = sx * m.sx + wx;
  return TileCoord{(int64_t)tr * TR, (int64_t)tc * TC, tc < nt_c && tr < nt_r};
}

template <bool XF32, int ROUNDING, int SELECT, bool RHT, bool WANT_ROW, int OUT>
__global__ __launch_bounds__(kThreads) void k_tile(
    const void *__restrict__ x_any, const float *__restrict__ alpha_p,
    uint8_t *__restrict__ codes_row, uint8_t *__restrict__ scales_row,
    uint8_t *__restrict__ choice_row, uint8_t *__restrict__ codes_col,
    uint8_t *__restrict__ scales_col, uint8_t *__restrict__ choice_col,
    uint16_t *__restrict__ out_bf16, int64_t rows, int64_t cols,
    uint64_t sr_seed, uint64_t rht_seed, TileMap map) {
  __shared__ ScaleTable tab;
  // the tile, row-major: one 32-bit word (two BF16) or two (two fp32) per pair of columns
  constexpr int kXW = XF32 ? 2 : 1;
  using Raw = RawBlock<XF32>;
  __shared__ __align__(16) uint32_t tile[TR * TC / 2 * kXW];
  // columnwise results wait here until a whole column segment can leave at once
  __shared__ uint2 stage_codes[OUT == kOutCodes ? kColItems : 1];     // [TC][TR/16]
  __shared__ uint8_t stage_scale[OUT == kOutCodes ? kColItems : 1];   // [TC][TR/16]
  __shared__ uint8_t stage_choice[OUT == kOutCodes ? kColItems : 1];  // [TC][TR/16]

  const TileCoord tcd = tile_of_workgroup(rows, cols, map);
  if (!tcd.valid) return;  // uniform over the workgroup
  const int64_t r0 = tcd.r0, c0 = tcd.c0;
  const int t = threadIdx.x;

  // Only columnwise codes wanted: nothing needs the tile in LDS -- a lane reads its two columns
  // straight from memory, a row at a time (a wave's load covers 256 contiguous bytes of a row).
  constexpr bool kDirect = !WANT_ROW && OUT == kOutCodes;

  // ---- phase 1: global -> LDS (and the rowwise outputs on the way); the loads go out
  // before the scale table is built
  if (!kDirect) {
    constexpr int kElemsPerPiece = XF32 ? 4 : 8;
    Raw w[kRowBlocksPerLane];
#pragma unroll
    for (int j = 0; j < kRowBlocksPerLane; ++j) {
      const int unit = t + j * kThreads;
      const int row = unit / kRowBlocksPerTileRow, rbk = unit % kRowBlocksPerTileRow;
      const int64_t gr = r0 + row, gc = c0 + rbk * 16;
      // (gr * cols + gc) elements into x, counted in 128-bit pieces
      const uint4 *src = static_cast<const uint4 *>(x_any) + (gr * cols + gc) / kElemsPerPiece;
#pragma unroll
      for (int q = 0; q < Raw::kPieces; ++q) {
        w[j].w[q] = make_uint4(0, 0, 0, 0);   // outside the tensor: zeros
        if (gr < rows && gc + q * kElemsPerPiece < cols) w[j].w[q] = src[q];
      }
    }
#pragma unroll
    for (int j = 0; j < kRowBlocksPerLane; ++j) {
      const int unit = t + j * kThreads;
      uint4 *dst = reinterpret_cast<uint4 *>(tile) + unit * Raw::kPieces;
#pragma unroll
      for (int q = 0; q < Raw::kPieces; ++q) dst[q] = w[j].w[q];
    }
  }
  const ScaleConsts sc = build_scale_table(tab, *alpha_p);     // ends with a barrier

  if (WANT_ROW) {
    // the lane's own row blocks, taken back from LDS one at a time (keeps the register
    // footprint of the quantizer to a single block)
    const int64_t nb_per_row = cols / 16;
#pragma unroll 1
    for (int j = 0; j < kRowBlocksPerLane; ++j) {
      const int unit = t + j * kThreads;
      const int row = unit / kRowBlocksPerTileRow, rbk = unit % kRowBlocksPerTileRow;
      const int64_t gr = r0 + row, gc = c0 + rbk * 16;
      if (gr < rows && gc < cols) {
        float v[16];
        uint32_t u[16];
        const int64_t k = gr * nb_per_row + (gc >> 4);
        // the lane's block out of the tile, with its random words
        auto take = [&](float (&w)[16], uint32_t (&uu)[16]) {
          const uint4 *own = reinterpret_cast<const uint4 *>(tile) + unit * Raw::kPieces;
          Raw mine;
#pragma unroll
          for (int q = 0; q < Raw::kPieces; ++q) mine.w[q] = own[q];
          unpack16(mine, w);
          if (ROUNDING != kRTN) {
#pragma unroll
            for (int q = 0; q < 4; ++q) sr_words4(sr_seed, (uint64_t)k * 4u + q, &uu[4 * q]);
          }
        };
        take(v, u);
        BlockResult r = quantize_block<ROUNDING, SELECT>(v, u, sc, tab, take);
        reinterpret_cast<uint2 *>(codes_row)[k] = make_uint2(r.lo, r.hi);
        scales_row[k] = (uint8_t)r.scale;
        if (choice_row) choice_row[k] = (uint8_t)r.four;
      }
    }
  }

  // ---- phase 2: every lane takes two adjacent columns x 16 rows.  A (column pair, row
  // block) unit is read and, for the fake-quant output, rewritten in place by its owner
  // lane only, so no barrier is needed inside this phase.
#pragma unroll 1
  for (int j = 0; j < kPairUnitsPerLane; ++j) {
    const int pu = t + j * kThreads;
    const int cp = pu % kColPairs, rb = pu / kColPairs;
    const int64_t gr = r0 + rb * 16;              // first row of the block
    const int64_t gc = c0 + 2 * cp;               // even column of the pair
    if (gr >= rows || gc >= cols) continue;       // (cols is even, so the pair is in or out together)
    float va[16], vb[16];
    uint32_t ua[16], ub[16];
    // the lane's two column blocks (transformed, with their random words) out of the tile or memory
    auto take = [&](float (&wa)[16], float (&wb)[16], uint32_t (&uua)[16], uint32_t (&uub)[16]) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        if constexpr (XF32) {
          const uint2 pair = kDirect
              ? static_cast<const uint2 *>(x_any)[((gr + i) * cols + gc) >> 1]
              : reinterpret_cast<const uint2 *>(tile)[(rb * 16 + i) * kColPairs + cp];
          wa[i] = u2f(pair.x);
          wb[i] = u2f(pair.y);
        } else {
          const uint32_t pair = kDirect ? static_cast<const uint32_t *>(x_any)[((gr + i) * cols + gc) >> 1]
                                        : tile[(rb * 16 + i) * kColPairs + cp];
          wa[i] = bf16_lo(pair);
          wb[i] = bf16_hi(pair);
        }
      }
      if (RHT) {
        const uint32_t sw = rht_sign_word(rht_seed, (uint64_t)(gr >> 4));
        rht16(wa, sw);
        rht16(wb, sw);
      }
      if (ROUNDING != kRTN) {
        // element (row, col) has flat index g = row*cols + col; the pair (gc, gc+1) shares a
        // Philox call because gc is even and cols is a multiple of 4
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const uint64_t g = (uint64_t)(gr + i) * (uint64_t)cols + (uint64_t)gc;
          uint32_t uu[4];
          sr_words4(sr_seed, g >> 2, uu);
          uua[i] = (g & 2u) ? uu[2] : uu[0];
          uub[i] = (g & 2u) ? uu[3] : uu[1];
        }
      }
    };
    take(va, vb, ua, ub);
    BlockResult ra = quantize_block<ROUNDING, SELECT>(va, ua, sc, tab, [&](float (&w)[16], uint32_t (&uu)[16]) {
      float other[16];
      uint32_t other_u[16];
      take(w, other, uu, other_u);
    });
    BlockResult rbk = quantize_block<ROUNDING, SELECT>(vb, ub, sc, tab, [&](float (&w)[16], uint32_t (&uu)[16]) {
      float other[16];
      uint32_t other_u[16];
      take(other, w, other_u, uu);
    });
    if (OUT == kOutCodes) {
      const int ia = (2 * cp) * kColBlockRows + rb, ib = ia + kColBlockRows;
      stage_codes[ia] = make_uint2(ra.lo, ra.hi);
      stage_codes[ib] = make_uint2(rbk.lo, rbk.hi);
      stage_scale[ia] = (uint8_t)ra.scale;
      stage_scale[ib] = (uint8_t)rbk.scale;
      stage_choice[ia] = (uint8_t)ra.four;
      stage_choice[ib] = (uint8_t)rbk.four;
    } else {
      float Da[16], Db[16];
      {
        float h[8];
        dequant8(ra.lo, ra.dec, h);
#pragma unroll
        for (int i = 0; i < 8; ++i) Da[i] = h[i];
        dequant8(ra.hi, ra.dec, h);
#pragma unroll
        for (int i = 0; i < 8; ++i) Da[8 + i] = h[i];
        dequant8(rbk.lo, rbk.dec, h);
#pragma unroll
        for (int i = 0; i < 8; ++i) Db[i] = h[i];
        dequant8(rbk.hi, rbk.dec, h);
#pragma unroll
        for (int i = 0; i < 8; ++i) Db[8 + i] = h[i];
      }
      // the BF16 pair takes the first word of the pair's slot
#pragma unroll
      for (int i = 0; i < 16; ++i)
        tile[((rb * 16 + i) * kColPairs + cp) * kXW] = pack_bf16x2(Da[i], Db[i]);
    }
  }
  __syncthreads();

  // ---- phase 3: LDS -> global, contiguous runs
  if (OUT == kOutCodes) {
    const int64_t col_codes = rows / 2, col_scales = rows / 16;
#pragma unroll
    for (int j = 0; j < kColItemsPerLane; ++j) {
      const int it = t + j * kThreads;
      const int cl = it / kColBlockRows, rb = it % kColBlockRows;
      const int64_t gc = c0 + cl, gr = r0 + rb * 16;
      if (gc < cols && gr < rows) {
        *reinterpret_cast<uint2 *>(codes_col + gc * col_codes + (gr >> 1)) = stage_codes[it];
        scales_col[gc * col_scales + (gr >> 4)] = stage_scale[it];
        if (choice_col) choice_col[gc * col_scales + (gr >> 4)] = stage_choice[it];
      }
    }
  } else {
#pragma unroll
    for (int j = 0; j < kPiecesPerLane; ++j) {
      const int idx = t + j * kThreads;
      const int row = idx / (TC / 8), seg = idx % (TC / 8);
      const int64_t gr = r0 + row, gc = c0 + seg * 8;
      if (gr < rows && gc < cols) {
        // piece idx = the four column pairs 4*idx .. 4*idx+3 of the tile
        const uint4 piece = XF32 ? make_uint4(tile[8 * idx], tile[8 * idx + 2], tile[8 * idx + 4],
                                              tile[8 * idx + 6])
                                 : reinterpret_cast<const uint4 *>(tile)[idx];
        store_as<kNtBf16>(reinterpret_cast<uint4 *>(out_bf16 + gr * cols + gc), piece);
      }
    }
  }
}

// Columnwise codes/scales -> row-major BF16, through an LDS tile.  TILE2D: the scales are
// per 16x16 tile of the matrix, stored [cols/16][rows/16].
template <bool TILE2D>
__global__ __launch_bounds__(kThreads) void k_dequant_col(const uint8_t *__restrict__ codes,
                                                          const uint8_t *__restrict__ scales,
                                                          const float *__restrict__ alpha_p,
                                                          uint16_t *__restrict__ out, int64_t rows,
                                                          int64_t cols, TileMap map) {
  __shared__ __align__(16) uint16_t tile16[TR * TC];
  const TileCoord tcd = tile_of_workgroup(rows, cols, map);
  if (!tcd.valid) return;
  const int64_t r0 = tcd.r0, c0 = tcd.c0;
  const int t = threadIdx.x;
  const float alpha = *alpha_p;
  const int64_t col_codes = rows / 2, col_scales = rows / 16;
#pragma unroll 1
  for (int j = 0; j < kColItemsPerLane; ++j) {
    const int it = t + j * kThreads;
    const int cl = it / kColBlockRows, rb = it % kColBlockRows;
    const int64_t gc = c0 + cl, gr = r0 + rb * 16;
    if (gc < cols && gr < rows) {
      const uint2 c = *reinterpret_cast<const uint2 *>(codes + gc * col_codes + (gr >> 1));
      const float dec =
          e4m3_decode(scales[(TILE2D ? (gc >> 4) : gc) * col_scales + (gr >> 4)]) * alpha;
      float D[8];
      dequant8(c.x, dec, D);
#pragma unroll
      for (int i = 0; i < 8; ++i) tile16[(rb * 16 + i) * TC + cl] = (uint16_t)pack_bf16x2(D[i], 0.0f);
      dequant8(c.y, dec, D);
#pragma unroll
      for (int i = 0; i < 8; ++i)
        tile16[(rb * 16 + 8 + i) * TC + cl] = (uint16_t)pack_bf16x2(D[i], 0.0f);
    }
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < kPiecesPerLane; ++j) {
    const int idx = t + j * kThreads;
    const int row = idx / (TC / 8), seg = idx % (TC / 8);
    const int64_t gr = r0 + row, gc = c0 + seg * 8;
    if (gr < rows && gc < cols)
      store_as<kNtBf16>(reinterpret_cast<uint4 *>(out + gr * cols + gc),
                        reinterpret_cast<const uint4 *>(tile16)[idx]);
  }
}

// ------------------------------------------------------- 2D (16x16) blocks

// One scale per 16x16 tile (the weight-matrix variant named in Section 4.1).  Sixteen
// adjacent lanes own the sixteen rows of a tile (one row block each); the tile's
// maximum, and the two candidates' errors, are combined across those lanes with XOR
// shuffles.  A tile's error is defined as a row's sixteen terms in the usual fixed order,
// then the sixteen row sums in the same order (strides 4, 2, 1 within each half, then the
// two halves), which is the order of the shuffles 4, 2, 1, 8; for the squared-error rule the
// decision is first tried on cheap row estimates summed the same way and falls back to the
// defined errors when the two sums are too close to call.
// Lane -> (tile, row): lanes 0-15 are the rows of one tile, the next sixteen lanes the
// tile to its right, so four lanes 16 apart read 128 contiguous bytes of one row.

// Sixteen adjacent lanes each hold one row of a 16x16 matrix of 4-bit codes (lo = columns
// 0-7, hi = columns 8-15, column j in bits 4j..4j+3); on return lane j of the sixteen holds
// column j packed the same way (row i in bits 4i..4i+3).  The usual recursive transpose:
// swap the off-diagonal 8x8 blocks between lanes 8 apart, then 4x4 blocks between lanes 4
// apart inside every 8x8 block, and so on down to single codes.
// 8-byte pieces per row of the LDS staging of transposed codes in k_block2d: 16 + 2, so that
// sixteen lanes writing one piece each to sixteen rows fall in different banks
constexpr uint32_t kColStagePitch = 18;

NV_DEV void transpose_codes16(uint32_t &lo, uint32_t &hi) {
  const uint32_t lane = threadIdx.x;
  {
    const bool upper = lane & 8u;
    const uint32_t got = __shfl_xor(upper ? lo : hi, 8, 64);
    if (upper) lo = got; else hi = got;
  }
  auto stage = [&](uint32_t &w, uint32_t bit, uint32_t keep_low, int shift) {
    // keep_low masks the groups a lane with (lane & bit) == 0 keeps in place
    const bool upper = lane & bit;
    const uint32_t give = upper ? (w & keep_low) : ((w >> shift) & keep_low);
    const uint32_t got = __shfl_xor(give, (int)bit, 64);
    w = upper ? ((w & ~keep_low) | got) : ((w & keep_low) | (got << shift));
  };
  stage(lo, 4u, 0x0000ffffu, 16);
  stage(hi, 4u, 0x0000ffffu, 16);
  stage(lo, 2u, 0x00ff00ffu, 8);
  stage(hi, 2u, 0x00ff00ffu, 8);
  stage(lo, 1u, 0x0f0f0f0fu, 4);
  stage(hi, 1u, 0x0f0f0f0fu, 4);
}

template <bool XF32, int ROUNDING, int SELECT, int OUT, bool BY_UNITS>
__global__ __launch_bounds__(kThreads) void k_block2d(
    const void *__restrict__ x_any, const float *__restrict__ alpha_p, uint8_t *__restrict__ codes,
    uint8_t *__restrict__ scales, uint8_t *__restrict__ choice, uint8_t *__restrict__ codes_col,
    uint8_t *__restrict__ scales_col, uint8_t *__restrict__ choice_col,
    uint16_t *__restrict__ out_bf16, int64_t rows, int64_t cols, uint64_t sr_seed) {
  __shared__ ScaleTable tab;
  const ScaleConsts sc = build_scale_table(tab, *alpha_p);
  const uint32_t tid = threadIdx.x, r_in_tile = tid & 15u, grp = tid >> 4;
  // rows, cols <= 2^31 and rows * cols <= 2^40 (checked by the entry point): tile coordinates
  // and tile numbers fit 32 bits
  const uint32_t ncb = (uint32_t)(cols / 16), nrb = (uint32_t)(rows / 16);
  const uint64_t n_tiles = (uint64_t)nrb * ncb;
  constexpr int kCandRounding = ROUNDING == kSRAfterRtnSelect ? kRTN : ROUNDING;
  constexpr int kErr = SELECT == kSel46     ? kErrMseEstimate
                       : SELECT == kSel46Mae ? kErrMae
                       : SELECT == kSel46AbsMax ? kErrAbsMax : kErrNone;
  // Two ways to hand tiles to workgroups (the launcher's grid matches):
  //  * one packing: workgroup id -> sixteen consecutive tiles along a row of tiles, one per group
  //    of sixteen lanes; a row of x is read, and its codes written, 128 contiguous bytes at a
  //    time by the workgroup;
  //  * with the packing for the transposed matrix as well, whose codes are 8 bytes per lane 4 KiB
  //    and more apart (stored like that they cost 1.9x their bytes in HBM writes and 35 us on
  //    8192 x 8192): workgroup id -> a unit of 16 tile rows x 4 tile columns, taken in four
  //    steps of 4 x 4 tiles (wave w: tile row 4 * step + w; its four groups: the tile columns).
  //    The unit's transposed codes (64 rows of the transposed matrix x 16 pieces of 8 bytes) are
  //    gathered in LDS and leave as whole 128-byte lines; row codes leave as 32 contiguous bytes
  //    per store instruction, and id -> unit keeps the four units that share their 128-byte
  //    lines on one die's L2 (ids 8 apart).
  constexpr bool by_units = BY_UNITS;
  static_assert(!BY_UNITS || OUT == kOutCodes, "units are for the transposed packing");
  __shared__ uint2 col_stage[BY_UNITS ? 64 * kColStagePitch : 1];
  const uint32_t wave = tid >> 6, g4 = grp & 3u;
  const uint32_t ncq = (ncb + 3u) / 4u, n_units = ((nrb + 15u) / 16u) * ncq;
  const uint32_t n_ids = by_units ? ((n_units + 31u) / 32u) * 32u : (uint32_t)((n_tiles + 15u) / 16u);
  const uint32_t n_steps = by_units ? 4u : 1u;
  auto tile_body = [&](uint32_t tr, uint32_t tc, uint32_t trl) {
    const uint64_t row = (uint64_t)tr * 16 + r_in_tile;
    const uint64_t first = row * (uint64_t)cols + tc * 16u;  // flat index of the lane's first element
    const uint64_t T = (uint64_t)tr * ncb + tc;
    RawBlock<XF32> raw;
    load_block<XF32>(static_cast<const uint4 *>(x_any) + first / (XF32 ? 4 : 8), raw);
    float v[16];
    uint32_t u[16];
    unpack16(raw, v);
    if (ROUNDING != kRTN) {
#pragma unroll
      for (int j = 0; j < 4; ++j) sr_words4(sr_seed, (uint64_t)(first >> 2) + j, &u[4 * j]);
    }
    float b = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; i += 2) b = fmaxf(fmaxf(b, fabsf(v[i])), fabsf(v[i + 1]));
#pragma unroll
    for (int m = 1; m < 16; m <<= 1) b = fmaxf(b, __shfl_xor(b, m, 64));

    // Eq. (2) for the tile, as for 1x16 blocks (the same for all sixteen lanes of the tile)
    uint32_t S6, S4;
    block_scales(b, sc, S6, S4);
    BlockResult r6{}, r4{};
    float E6 = 0.0f, E4 = 0.0f, enc6 = 0.0f, enc4 = 0.0f;
    if (SELECT != kSelForce4) {
      r6.scale = S6;
      const float4 t = tab.e[r6.scale];
      r6.dec = t.x;
      enc6 = t.y;
      if (!(ROUNDING == kSRAfterRtnSelect && SELECT == kSelForce6))
        E6 = candidate<kCandRounding, kErr>(v, u, t.x, t.y, r6.lo, r6.hi);
    }
    if (SELECT != kSelForce6) {
      r4.scale = S4;
      r4.four = 1u;
      const float4 t = tab.e[r4.scale];
      r4.dec = t.x;
      enc4 = t.y;
      if (!(ROUNDING == kSRAfterRtnSelect && SELECT == kSelForce4))
        E4 = candidate<kCandRounding, kErr>(v, u, t.x, t.y, r4.lo, r4.hi);
    }
    // the sixteen row values -> the tile's, in the fixed order; every lane ends with the same sum
    auto over_tile = [&](float &e6, float &e4) {
      constexpr int order[4] = {4, 2, 1, 8};
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const float o6 = __shfl_xor(e6, order[s], 64), o4 = __shfl_xor(e4, order[s], 64);
        e6 = SELECT == kSel46AbsMax ? fmaxf(e6, o6) : e6 + o6;
        e4 = SELECT == kSel46AbsMax ? fmaxf(e4, o4) : e4 + o4;
      }
    };
    bool four = SELECT == kSelForce4;
    if (SELECT == kSel46Mae || SELECT == kSel46AbsMax) {
      over_tile(E6, E4);      // evaluated as defined
      four = E4 < E6;
    } else if (SELECT == kSel46) {
      // E6, E4 are row estimates (see decide_from_estimates).  Outside the margin of
      // tile_decision_tolerance() the summed estimates order the defined errors; inside it
      // the defined errors are evaluated.  All sixteen lanes hold the same sums and take the
      // same path.
      over_tile(E6, E4);
      const float tol = tile_decision_tolerance(r6.dec, E6, r4.dec, E4);
      const float diff = E4 - E6;
      four = diff < 0.0f;
      if (!(fabsf(diff) > tol)) {
        float e6 = exact_error(v, r6.lo, r6.hi, r6.dec), e4 = exact_error(v, r4.lo, r4.hi, r4.dec);
        over_tile(e6, e4);
        four = e4 < e6;
      }
    }
    BlockResult res = four ? r4 : r6;
    if (ROUNDING == kSRAfterRtnSelect)
      (void)candidate<kSR, kErrNone>(v, u, res.dec, four ? enc4 : enc6, res.lo, res.hi);
    if (OUT == kOutCodes) {
      if (codes) {
        *reinterpret_cast<uint2 *>(codes + first / 2) = make_uint2(res.lo, res.hi);
        if (r_in_tile == 0) {
          scales[T] = (uint8_t)res.scale;
          if (choice) choice[T] = (uint8_t)res.four;
        }
      }
      if (BY_UNITS) {
        // the same tile for the transposed matrix: column (tc*16 + lane) of x is its row
        uint32_t lo = res.lo, hi = res.hi;
        transpose_codes16(lo, hi);
        col_stage[(g4 * 16u + r_in_tile) * kColStagePitch + trl] = make_uint2(lo, hi);
        if (r_in_tile == 0) {
          const uint64_t Tt = (uint64_t)tc * nrb + tr;
          scales_col[Tt] = (uint8_t)res.scale;
          if (choice_col) choice_col[Tt] = (uint8_t)res.four;
        }
      }
    } else {
      float D0[8], D1[8];
      dequant8(res.lo, res.dec, D0);
      dequant8(res.hi, res.dec, D1);
      uint4 *dst = reinterpret_cast<uint4 *>(out_bf16 + first);
      dst[0] = make_uint4(pack_bf16x2(D0[0], D0[1]), pack_bf16x2(D0[2], D0[3]),
                          pack_bf16x2(D0[4], D0[5]), pack_bf16x2(D0[6], D0[7]));
      dst[1] = make_uint4(pack_bf16x2(D1[0], D1[1]), pack_bf16x2(D1[2], D1[3]),
                          pack_bf16x2(D1[4], D1[5]), pack_bf16x2(D1[6], D1[7]));
    }
  };
  for (uint32_t id = blockIdx.x; id < n_ids; id += gridDim.x) {
    // by units: the same for the whole workgroup
    const uint32_t slot = id >> 3, unit = (((slot >> 2) << 3) + (id & 7u)) * 4u + (slot & 3u);
    const uint32_t mr = unit / ncq, cq = unit - mr * ncq;
#pragma unroll 1
    for (uint32_t step = 0; step < n_steps; ++step) {
      uint32_t tr, tc, trl = step * 4u + wave;
      bool live;
      if (by_units) {
        tr = mr * 16u + trl;
        tc = cq * 4u + g4;
        live = unit < n_units && tr < nrb && tc < ncb;
      } else {
        const uint32_t t = id * 16u + grp;
        tr = t / ncb;
        tc = t - tr * ncb;
        live = (uint64_t)id * 16u + grp < n_tiles;
      }
      if (live) tile_body(tr, tc, trl);
      if (by_units && step == 3u) {
        // the unit's 64 rows of the transposed matrix, 16 pieces of 8 bytes each: sixteen
        // consecutive lanes store one 128-byte line
        __syncthreads();
        if (unit < n_units) {
#pragma unroll 1
          for (uint32_t j = 0; j < 4; ++j) {
            const uint32_t piece = tid + j * kThreads, line = piece >> 4, k = piece & 15u;
            const uint64_t col = ((uint64_t)cq * 4 + (line >> 4)) * 16 + (line & 15u);
            const uint32_t tr_k = mr * 16u + k;
            if (col < (uint64_t)cols && tr_k < nrb)
              *reinterpret_cast<uint2 *>(codes_col + col * (uint64_t)(rows / 2) + tr_k * 8u) =
                  col_stage[line * kColStagePitch + k];
          }
        }
        __syncthreads();
      }
    }
  }
}

#if NVFP4_46_MAIN
// 2D-block data -> BF16: one lane per 8 codes; the scale is the tile's.
__global__ __launch_bounds__(kThreads) void k_dequant_2d(const uint32_t *__restrict__ codes,
                                                         const uint8_t *__restrict__ scales,
                                                         const float *__restrict__ alpha_p,
                                                         uint4 *__restrict__ out, int64_t n8,
                                                         int64_t cols) {
  const float alpha = *alpha_p;
  const int64_t per_row = cols / 8, ncb = cols / 16;
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x; t < n8; t += stride) {
    const int64_t row = t / per_row, c8 = t - row * per_row;
    const float dec = e4m3_decode(scales[(row >> 4) * ncb + (c8 >> 1)]) * alpha;
    float D[8];
    dequant8(codes[t], dec, D);
    store_as<kNtBf16>(out + t, make_uint4(pack_bf16x2(D[0], D[1]), pack_bf16x2(D[2], D[3]),
                                          pack_bf16x2(D[4], D[5]), pack_bf16x2(D[6], D[7])));
  }
}

// ------------------------------------------------------------ debug kernels

__global__ void k_dbg_e2m1_rtn(uint32_t first, int64_t n, uint8_t *out) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
    float y = u2f(first + (uint32_t)i);
    out[i] = (uint8_t)(hw_pk_fp4<0>(0u, y, 0.0f) & 15u);
  }
}

__global__ void k_dbg_e4m3(uint32_t first, int64_t n, uint8_t *out) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
    out[i] = (uint8_t)e4m3_encode(u2f(first + (uint32_t)i));
}

__global__ void k_dbg_tables(float *out) {
  const int t = threadIdx.x;
  if (t < 16) {
    float D[8];
    dequant8((uint32_t)t, 1.0f, D);     // code t in nibble 0
    out[t] = D[0];
  }
  if (t < 256) out[16 + t] = e4m3_decode((uint32_t)t & 0x7fu);
}

__global__ void k_dbg_bf16(uint32_t first, uint32_t stride_bits, int64_t n, uint16_t *out) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
    out[i] = (uint16_t)pack_bf16x2(u2f(first + (uint32_t)i * stride_bits), 0.0f);
}

__global__ void k_dbg_e2m1_sr(const float *y, const uint32_t *w, int64_t n, uint8_t *out,
                              uint8_t *out_fast) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
    out[i] = (uint8_t)e2m1_code_of_grid_value(e2m1_sr_value(y[i], sr_uniform_of_word(w[i])));
    float margin = __builtin_inff();
    const uint32_t code = e2m1_sr_code_fast<0>(0u, y[i], ~w[i], (float)w[i], margin) & 0x0fu;
    out_fast[i] = (uint8_t)(code | (margin > kSrMarginAtRisk ? 0u : 0x80u));
  }
}

__global__ void k_dbg_philox(const uint32_t *ctr, uint32_t k0, uint32_t k1, int64_t n,
                             uint32_t *out) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
    Philox4 p = philox4x32_10(ctr[4 * i], ctr[4 * i + 1], ctr[4 * i + 2], ctr[4 * i + 3], k0, k1);
#pragma unroll
    for (int j = 0; j < 4; ++j) out[4 * i + j] = p.w[j];
  }
}

#endif

// ---------------------------------------------------------------- launchers

// Compute units of the device that is current for the calling thread, asked for on every
// call (the library keeps no state, and two devices of one process may differ).
static int compute_units() {
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
    cus = 256;
  return cus;
}

static int grid_for(int64_t work_items, int per_cu) {
  int64_t need = (work_items + kThreads - 1) / kThreads;
  int64_t cap = (int64_t)compute_units() * per_cu;
  if (need < 1) need = 1;
  return (int)(need < cap ? need : cap);
}

// every kernel of this file uses static LDS only
template <typename Kernel, typename... Args>
static int launch(Kernel kernel, dim3 grid, dim3 block, hipStream_t stream, Args... args) {
  return launch(kernel, grid, block, (size_t)0, stream, args...);
}

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

struct FlatArgs {
  bool xf32;        // x holds fp32 values instead of BF16
  const uint4 *x;
  const float *alpha;
  uint2 *codes;
  uint8_t *scales, *choice;
  uint4 *out;
  uint32_t *amax;
  int64_t nblocks;
  uint32_t nb_per_row;
  uint64_t sr_seed, rht_seed;
  hipStream_t stream;
  AmaxFinish fin{nullptr, nullptr, 0.0f};   // the amax pass only
};

template <bool XF32, int ROUNDING, int SELECT, bool RHT, int OUT>
static int launch_flat(const FlatArgs &a) {
  const int64_t rounds = (a.nblocks + kThreads - 1) / kThreads;
  const int cus = compute_units();
  int64_t n_long = 0, rounds_long = 0, grid;
  if (OUT == kOutAmax) {
    // the amax pass ends with one access per workgroup to the one result word: few,
    // long-lived workgroups that stride over the whole tensor
    grid = (int64_t)cus * kFlatAmaxWgPerCu;
    if (grid > rounds) grid = rounds;
  } else {
    n_long = (int64_t)cus * kFlatLongWgPerCu;
    rounds_long = (rounds - (int64_t)cus * kFlatShortRoundsPerCu) / n_long;
    if (rounds_long < 2) n_long = rounds_long = 0;   // a small tensor: one round per workgroup
    grid = n_long + (rounds - n_long * rounds_long);
  }
  if (RHT) {
    // round r starts at block 256*r; if 256 * (a workgroup's stride) is a multiple of the
    // blocks per row, every lane sees one position along the row in all its rounds
    uint32_t g = a.nb_per_row, t = kThreads;
    while (t) { const uint32_t q = g % t; g = t; t = q; }      // gcd(nb_per_row, 256)
    const int64_t period = a.nb_per_row / g;
    if (OUT == kOutAmax) {
      if (period <= grid / 2) grid -= grid % period;
    } else if (n_long && period <= n_long / 2) {
      n_long -= n_long % period;
      rounds_long = (rounds - (int64_t)cus * kFlatShortRoundsPerCu) / n_long;
      grid = n_long + (rounds - n_long * rounds_long);
    }
  }
  return launch(k_flat<XF32, ROUNDING, SELECT, RHT, OUT>, dim3((uint32_t)grid), dim3(kThreads),
                a.stream, a.x, a.alpha, a.codes, a.scales, a.choice, a.out, a.amax, a.nblocks,
                a.nb_per_row, a.sr_seed, a.rht_seed, (uint32_t)n_long, (uint32_t)rounds_long, a.fin);
}

template <bool XF32, int ROUNDING, int SELECT>
static int launch_flat_variant(const FlatArgs &a, bool rht, int out) {
  if (out == kOutCodes) {
    if (rht) return launch_flat<XF32, ROUNDING, SELECT, true, kOutCodes>(a);
    return launch_flat<XF32, ROUNDING, SELECT, false, kOutCodes>(a);
  }
  if (rht) return launch_flat<XF32, ROUNDING, SELECT, true, kOutFake>(a);
  return launch_flat<XF32, ROUNDING, SELECT, false, kOutFake>(a);
}

// All rowwise kernels of one (input type, rounding mode) pair.
template <bool XF32, int ROUNDING>
int run_flat(const FlatArgs &a, uint32_t select, bool rht, int out) {
  if (select == NVFP4_SEL_46_MSE) return launch_flat_variant<XF32, ROUNDING, kSel46>(a, rht, out);
  if (select == NVFP4_SEL_FORCE6) return launch_flat_variant<XF32, ROUNDING, kSelForce6>(a, rht, out);
  if (select == NVFP4_SEL_FORCE4) return launch_flat_variant<XF32, ROUNDING, kSelForce4>(a, rht, out);
  if (select == NVFP4_SEL_46_MAE) return launch_flat_variant<XF32, ROUNDING, kSel46Mae>(a, rht, out);
  return launch_flat_variant<XF32, ROUNDING, kSel46AbsMax>(a, rht, out);
}

struct TileArgs {
  bool xf32;
  const void *x;
  const float *alpha;
  uint8_t *codes_row, *scales_row, *choice_row, *codes_col, *scales_col, *choice_col;
  uint16_t *out;
  int64_t rows, cols;
  uint64_t sr_seed, rht_seed;
  hipStream_t stream;
};

// Super-tiles of 8 x 16 tiles, smaller along an axis that has fewer tiles (a small tensor
// would otherwise launch mostly workgroups without a tile).
static TileMap tile_map(int64_t rows, int64_t cols) {
  const int64_t nt_r = (rows + TR - 1) / TR, nt_c = (cols + TC - 1) / TC;
  return TileMap{(uint32_t)(nt_c < 8 ? nt_c : 8), (uint32_t)(nt_r < 16 ? nt_r : 16)};
}

// Whole turns over the eight XCDs, each turn one super-tile per XCD.
static int tile_grid(int64_t rows, int64_t cols) {
  const TileMap m = tile_map(rows, cols);
  const int64_t nt_r = (rows + TR - 1) / TR, nt_c = (cols + TC - 1) / TC;
  const int64_t supers = ((nt_c + m.sx - 1) / m.sx) * ((nt_r + m.sy - 1) / m.sy);
  return (int)(8 * ((supers + 7) / 8) * m.sx * m.sy);
}

template <bool XF32, int ROUNDING, int SELECT, bool RHT, bool WANT_ROW, int OUT>
static int launch_tile(const TileArgs &a) {
  return launch(k_tile<XF32, ROUNDING, SELECT, RHT, WANT_ROW, OUT>, dim3(tile_grid(a.rows, a.cols)),
                dim3(kThreads), a.stream, a.x, a.alpha, a.codes_row, a.scales_row, a.choice_row,
                a.codes_col, a.scales_col, a.choice_col, a.out, a.rows, a.cols, a.sr_seed,
                a.rht_seed, tile_map(a.rows, a.cols));
}

// variant: 0 = columnwise codes, 1 = columnwise codes + rht, 2 = both orientations,
//          3 = columnwise fake-quant, 4 = columnwise fake-quant + rht
template <bool XF32, int ROUNDING, int SELECT>
static int launch_tile_variant(const TileArgs &a, int variant) {
  switch (variant) {
    case 0: return launch_tile<XF32, ROUNDING, SELECT, false, false, kOutCodes>(a);
    case 1: return launch_tile<XF32, ROUNDING, SELECT, true, false, kOutCodes>(a);
    case 2: return launch_tile<XF32, ROUNDING, SELECT, false, true, kOutCodes>(a);
    case 3: return launch_tile<XF32, ROUNDING, SELECT, false, false, kOutFake>(a);
    default: return launch_tile<XF32, ROUNDING, SELECT, true, false, kOutFake>(a);
  }
}

// All tiled (columnwise / both) kernels of one (input type, rounding mode) pair.
template <bool XF32, int ROUNDING>
int run_tile(const TileArgs &a, uint32_t select, int variant) {
  if (select == NVFP4_SEL_46_MSE) return launch_tile_variant<XF32, ROUNDING, kSel46>(a, variant);
  if (select == NVFP4_SEL_FORCE6) return launch_tile_variant<XF32, ROUNDING, kSelForce6>(a, variant);
  if (select == NVFP4_SEL_FORCE4) return launch_tile_variant<XF32, ROUNDING, kSelForce4>(a, variant);
  if (select == NVFP4_SEL_46_MAE) return launch_tile_variant<XF32, ROUNDING, kSel46Mae>(a, variant);
  return launch_tile_variant<XF32, ROUNDING, kSel46AbsMax>(a, variant);
}

struct Block2dArgs {
  bool xf32;
  const void *x;
  const float *alpha;
  uint8_t *codes, *scales, *choice, *codes_col, *scales_col, *choice_col;
  uint16_t *out;
  int64_t rows, cols;
  uint64_t sr_seed;
  hipStream_t stream;
};

template <bool XF32, int ROUNDING, int SELECT>
static int launch_block2d(const Block2dArgs &a, int out) {
  // ids as the kernel counts them: sixteen tiles each, or - with the transposed packing - units
  // of 16 x 4 tiles in whole groups of 32
  const int64_t tiles = (a.rows / 16) * (a.cols / 16);
  const int64_t units = ((a.rows / 16 + 15) / 16) * ((a.cols / 16 + 3) / 4);
  const int64_t ids = out == kOutCodes && a.codes_col ? ((units + 31) / 32) * 32 : (tiles + 15) / 16;
  const int grid = grid_for(ids * kThreads, 16);
  auto go = [&](auto kernel) {
    return launch(kernel, dim3(grid), dim3(kThreads), a.stream, a.x, a.alpha, a.codes, a.scales,
                  a.choice, a.codes_col, a.scales_col, a.choice_col, a.out, a.rows, a.cols,
                  a.sr_seed);
  };
  if (out == kOutCodes && a.codes_col) return go(k_block2d<XF32, ROUNDING, SELECT, kOutCodes, true>);
  if (out == kOutCodes) return go(k_block2d<XF32, ROUNDING, SELECT, kOutCodes, false>);
  return go(k_block2d<XF32, ROUNDING, SELECT, kOutFake, false>);
}

// All 16x16-tile kernels of one (input type, rounding mode) pair.
template <bool XF32, int ROUNDING>
int run_block2d(const Block2dArgs &a, uint32_t select, int out) {
  if (select == NVFP4_SEL_46_MSE) return launch_block2d<XF32, ROUNDING, kSel46>(a, out);
  if (select == NVFP4_SEL_FORCE6) return launch_block2d<XF32, ROUNDING, kSelForce6>(a, out);
  if (select == NVFP4_SEL_FORCE4) return launch_block2d<XF32, ROUNDING, kSelForce4>(a, out);
  if (select == NVFP4_SEL_46_MAE) return launch_block2d<XF32, ROUNDING, kSel46Mae>(a, out);
  return launch_block2d<XF32, ROUNDING, kSel46AbsMax>(a, out);
}

// One group of kernels = the three run_* templates for one (XF32, ROUNDING) pair.  A part
// that holds a group defines it; the main part, when built apart, only declares them.
#define NVFP4_46_GROUP(KEYWORD, XF32, ROUNDING)                                                 \
  KEYWORD template int run_flat<XF32, ROUNDING>(const FlatArgs &, uint32_t, bool, int);         \
  KEYWORD template int run_tile<XF32, ROUNDING>(const TileArgs &, uint32_t, int);               \
  KEYWORD template int run_block2d<XF32, ROUNDING>(const Block2dArgs &, uint32_t, int);
#if NVFP4_46_PART == 0
NVFP4_46_GROUP(extern, false, kRTN)
NVFP4_46_GROUP(extern, false, kSR)
NVFP4_46_GROUP(extern, false, kSRAfterRtnSelect)
NVFP4_46_GROUP(extern, true, kRTN)
NVFP4_46_GROUP(extern, true, kSR)
NVFP4_46_GROUP(extern, true, kSRAfterRtnSelect)
#elif NVFP4_46_PART >= 1 && NVFP4_46_PART <= 6
static_assert(kRTN == 0 && kSR == 1 && kSRAfterRtnSelect == 2, "parts are numbered by these");
NVFP4_46_GROUP(, ((NVFP4_46_PART - 1) / 3 != 0), ((NVFP4_46_PART - 1) % 3))
#endif

#if NVFP4_46_MAIN
static int rounding_index(uint32_t rounding) {
  return rounding == NVFP4_SR ? kSR : rounding == NVFP4_SR_AFTER_RTN_SELECT ? kSRAfterRtnSelect : kRTN;
}

static int dispatch_flat(const FlatArgs &a, uint32_t rounding, uint32_t select, bool rht, int out) {
  typedef int (*Fn)(const FlatArgs &, uint32_t, bool, int);
  static const Fn table[2][3] = {
      {run_flat<false, kRTN>, run_flat<false, kSR>, run_flat<false, kSRAfterRtnSelect>},
      {run_flat<true, kRTN>, run_flat<true, kSR>, run_flat<true, kSRAfterRtnSelect>}};
  return table[a.xf32][rounding_index(rounding)](a, select, rht, out);
}

static int dispatch_tile(const TileArgs &a, uint32_t rounding, uint32_t select, int variant) {
  typedef int (*Fn)(const TileArgs &, uint32_t, int);
  static const Fn table[2][3] = {
      {run_tile<false, kRTN>, run_tile<false, kSR>, run_tile<false, kSRAfterRtnSelect>},
      {run_tile<true, kRTN>, run_tile<true, kSR>, run_tile<true, kSRAfterRtnSelect>}};
  return table[a.xf32][rounding_index(rounding)](a, select, variant);
}

static int dispatch_block2d(const Block2dArgs &a, uint32_t rounding, uint32_t select, int out) {
  typedef int (*Fn)(const Block2dArgs &, uint32_t, int);
  static const Fn table[2][3] = {
      {run_block2d<false, kRTN>, run_block2d<false, kSR>, run_block2d<false, kSRAfterRtnSelect>},
      {run_block2d<true, kRTN>, run_block2d<true, kSR>, run_block2d<true, kSRAfterRtnSelect>}};
  return table[a.xf32][rounding_index(rounding)](a, select, out);
}

// Checks shared by the entry points that take the parameter block.
static int check_params(const void *x, const nvfp4_46_params *p, bool one_layout_only) {
  if (!x || !p) return NVFP4_ERR_NULL;
  if (p->rows <= 0 || p->cols <= 0) return NVFP4_ERR_SHAPE;
  if (p->layout < 1u || p->layout > 3u) return NVFP4_ERR_PARAM;
  if (one_layout_only && p->layout == 3u) return NVFP4_ERR_PARAM;
  if (p->rounding > NVFP4_SR_AFTER_RTN_SELECT || p->select > NVFP4_SEL_46_ABSMAX || p->rht > 1u ||
      p->block2d > 1u || p->x_dtype > NVFP4_X_F32)
    return NVFP4_ERR_PARAM;
  if (!(p->fp8_max > 0.0f) || !(p->fp8_max <= 448.0f)) return NVFP4_ERR_PARAM;
  if ((p->layout & NVFP4_ROWWISE) && (p->cols % 16) != 0) return NVFP4_ERR_SHAPE;
  if ((p->layout & NVFP4_COLWISE) && ((p->rows % 16) != 0 || (p->cols % 8) != 0))
    return NVFP4_ERR_SHAPE;
  if (p->rows > (int64_t)1 << 31 || p->cols > (int64_t)1 << 31 ||
      p->rows * p->cols > (int64_t)1 << 40)
    return NVFP4_ERR_SHAPE;
  if (!aligned16(x)) return NVFP4_ERR_ALIGN;
  if (p->rht && p->layout == 3u) return NVFP4_ERR_UNSUPPORTED;
  if (p->block2d) {
    if ((p->rows % 16) != 0 || (p->cols % 16) != 0) return NVFP4_ERR_SHAPE;
    if (p->rht) return NVFP4_ERR_UNSUPPORTED;
  }
  return NVFP4_OK;
}

// Eq. (1) for all three entry points.  scratch == nullptr: the reduction runs on the caller's
// alpha word between a zeroing launch and a finishing launch.  Otherwise scratch points at
// kScratchWords zeroed words and one launch does it all (see AmaxFinish).
static int tensor_scale(const void *x, const nvfp4_46_params *p, float *alpha, uint32_t *scratch,
                        hipStream_t s) {
  if (!alpha) return NVFP4_ERR_NULL;
  int rc = check_params(x, p, false);
  if (rc != NVFP4_OK) return rc;
  uint32_t *amax = reinterpret_cast<uint32_t *>(alpha);      // the plain form's running maximum
  const AmaxFinish fin{scratch, alpha, p->fp8_max};
  if (!scratch) {
    rc = launch(k_store_u32, dim3(1), dim3(1), s, amax, 0u);
    if (rc != NVFP4_OK) return rc;
  }
  const int64_t n = p->rows * p->cols;
  const bool xf32 = p->x_dtype == NVFP4_X_F32;
  const uint4 *x4 = static_cast<const uint4 *>(x);
  if (!p->rht) {
    // 128-bit pieces (n is a multiple of 8 by the shape checks)
    const int64_t n16 = xf32 ? n / 4 : n / 8;
    const dim3 grid(grid_for(n16, kAmaxWgPerCu));
    rc = xf32 ? launch(k_amax_plain<true>, grid, dim3(kThreads), s, x4, n16, amax, fin)
              : launch(k_amax_plain<false>, grid, dim3(kThreads), s, x4, n16, amax, fin);
  } else if (p->layout == NVFP4_ROWWISE) {
    FlatArgs a{xf32, x4, nullptr, nullptr, nullptr, nullptr, nullptr, amax,
               n / 16, (uint32_t)(p->cols / 16), 0, p->rht_seed, s, fin};
    rc = xf32 ? launch_flat<true, kRTN, kSel46, true, kOutAmax>(a)
              : launch_flat<false, kRTN, kSel46, true, kOutAmax>(a);
  } else {
    // columnwise blocks (rows % 16 == 0, cols % 8 == 0): 16-byte pieces of 8 BF16 / 4 fp32 columns
    const int64_t row_blocks = p->rows / 16, pieces = xf32 ? p->cols / 4 : p->cols / 8;
    const dim3 grid(grid_for(row_blocks * pieces, kAmaxRhtColWgPerCu));
    rc = xf32 ? launch(k_amax_rht_col<true>, grid, dim3(kThreads), s, x4, row_blocks, pieces,
                       p->rht_seed, amax, fin)
              : launch(k_amax_rht_col<false>, grid, dim3(kThreads), s, x4, row_blocks, pieces,
                       p->rht_seed, amax, fin);
  }
  if (rc != NVFP4_OK || scratch) return rc;
  return launch(k_finish_alpha, dim3(1), dim3(1), s, alpha, p->fp8_max);
}

#endif  // NVFP4_46_MAIN

}  // namespace nvfp4_46

#if NVFP4_46_MAIN

using namespace nvfp4_46;

extern "C" {

int nvfp4_46_tensor_scale(const void *x, const nvfp4_46_params *p, float *alpha, void *stream) {
  return tensor_scale(x, p, alpha, nullptr, static_cast<hipStream_t>(stream));
}

int nvfp4_46_tensor_scale_ws(const void *x, const nvfp4_46_params *p, float *alpha,
                             void *workspace, size_t workspace_bytes, void *stream) {
  if (!workspace) return NVFP4_ERR_NULL;
  if (workspace_bytes < NVFP4_46_TENSOR_SCALE_WS_BYTES) return NVFP4_ERR_PARAM;
  if (!aligned16(workspace)) return NVFP4_ERR_ALIGN;
  return tensor_scale(x, p, alpha, static_cast<uint32_t *>(workspace), static_cast<hipStream_t>(stream));
}

// Scratch of nvfp4_46_tensor_scale_static: the maximum and ticket words of the one-launch
// reduction (see AmaxFinish), 4352 bytes; every GPU the library runs on holds its own copy
// until the process ends.  In host code the array's name only stands for the symbol:
// the device address is looked up once per device and that pointer is what kernels get.
static __device__ __align__(256) uint32_t scratch[kScratchWords];
static_assert(kScratchWords * sizeof(uint32_t) == NVFP4_46_TENSOR_SCALE_WS_BYTES, "header and kernels agree on the scratch size");

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
uint32_t *g_scratch_ptr[kMaxDevices];   // per device; nullptr until that device's first call
}  // namespace

int nvfp4_46_tensor_scale_static(const void *x, const nvfp4_46_params *p, float *alpha, void *stream) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return NVFP4_ERR_HIP;
  uint32_t *ptr;
  {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
      void *sym = nullptr;
      if (hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)) != hipSuccess || !sym) return NVFP4_ERR_HIP;
      g_scratch_ptr[dev] = static_cast<uint32_t *>(sym);
    }
    ptr = g_scratch_ptr[dev];
  }
  return tensor_scale(x, p, alpha, ptr, static_cast<hipStream_t>(stream));
}

int nvfp4_46_quantize(const void *x, const nvfp4_46_params *p, const float *alpha,
                      void *codes_row, void *scales_row, void *codes_col, void *scales_col,
                      void *choice_row, void *choice_col, void *stream) {
  if (!alpha) return NVFP4_ERR_NULL;
  int rc = check_params(x, p, false);
  if (rc != NVFP4_OK) return rc;
  const bool xf32 = p->x_dtype == NVFP4_X_F32;
  const bool want_row = p->layout & NVFP4_ROWWISE, want_col = p->layout & NVFP4_COLWISE;
  if (want_row && (!codes_row || !scales_row)) return NVFP4_ERR_NULL;
  if (want_col && (!codes_col || !scales_col)) return NVFP4_ERR_NULL;
  if (!want_row && (codes_row || scales_row || choice_row)) return NVFP4_ERR_PARAM;
  if (!want_col && (codes_col || scales_col || choice_col)) return NVFP4_ERR_PARAM;
  if (!aligned16(codes_row) || !aligned16(scales_row) || !aligned16(codes_col) ||
      !aligned16(scales_col) || !aligned16(choice_row) || !aligned16(choice_col))
    return NVFP4_ERR_ALIGN;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (p->block2d) {
    Block2dArgs a{xf32, x, alpha, static_cast<uint8_t *>(codes_row),
                  static_cast<uint8_t *>(scales_row), static_cast<uint8_t *>(choice_row),
                  static_cast<uint8_t *>(codes_col), static_cast<uint8_t *>(scales_col),
                  static_cast<uint8_t *>(choice_col), nullptr, p->rows, p->cols, p->sr_seed, s};
    return dispatch_block2d(a, p->rounding, p->select, kOutCodes);
  }
  if (!want_col) {
    FlatArgs a{xf32, static_cast<const uint4 *>(x), alpha, static_cast<uint2 *>(codes_row),
               static_cast<uint8_t *>(scales_row), static_cast<uint8_t *>(choice_row), nullptr,
               nullptr, p->rows * p->cols / 16, (uint32_t)(p->cols / 16), p->sr_seed, p->rht_seed, s};
    return dispatch_flat(a, p->rounding, p->select, p->rht != 0, kOutCodes);
  }
  TileArgs a{xf32, x, alpha, static_cast<uint8_t *>(codes_row),
             static_cast<uint8_t *>(scales_row), static_cast<uint8_t *>(choice_row),
             static_cast<uint8_t *>(codes_col), static_cast<uint8_t *>(scales_col),
             static_cast<uint8_t *>(choice_col), nullptr, p->rows, p->cols, p->sr_seed,
             p->rht_seed, s};
  return dispatch_tile(a, p->rounding, p->select, want_row ? 2 : (p->rht ? 1 : 0));
}

int nvfp4_46_dequantize(const void *codes, const void *scales, const float *alpha, int64_t rows,
                        int64_t cols, uint32_t layout, void *out_bf16, void *stream) {
  if (!codes || !scales || !alpha || !out_bf16) return NVFP4_ERR_NULL;
  if (rows <= 0 || cols <= 0) return NVFP4_ERR_SHAPE;
  if (layout != NVFP4_ROWWISE && layout != NVFP4_COLWISE && layout != NVFP4_BLOCK2D &&
      layout != (NVFP4_BLOCK2D | NVFP4_COLWISE))
    return NVFP4_ERR_PARAM;
  if ((layout & NVFP4_BLOCK2D) && ((rows % 16) != 0 || (cols % 16) != 0)) return NVFP4_ERR_SHAPE;
  if (layout == NVFP4_ROWWISE && (cols % 16) != 0) return NVFP4_ERR_SHAPE;
  if (layout == NVFP4_COLWISE && ((rows % 16) != 0 || (cols % 8) != 0)) return NVFP4_ERR_SHAPE;
  if (rows > (int64_t)1 << 31 || cols > (int64_t)1 << 31 || rows * cols > (int64_t)1 << 40)
    return NVFP4_ERR_SHAPE;
  if (!aligned16(codes) || !aligned16(scales) || !aligned16(out_bf16)) return NVFP4_ERR_ALIGN;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const uint8_t *c8 = static_cast<const uint8_t *>(codes), *s8 = static_cast<const uint8_t *>(scales);
  const int64_t n8 = rows * cols / 8;
  if (layout == NVFP4_BLOCK2D)
    return launch(k_dequant_2d, dim3(grid_for(n8, 16)), dim3(kThreads), s,
                  static_cast<const uint32_t *>(codes), s8, alpha, static_cast<uint4 *>(out_bf16),
                  n8, cols);
  if (layout == NVFP4_ROWWISE)
    return launch(k_dequant_flat, dim3(grid_for(n8, 16)), dim3(kThreads), s,
                  static_cast<const uint32_t *>(codes), s8, alpha, static_cast<uint4 *>(out_bf16),
                  n8);
  if (layout == NVFP4_COLWISE)
    return launch(k_dequant_col<false>, dim3(tile_grid(rows, cols)), dim3(kThreads), s, c8, s8,
                  alpha, static_cast<uint16_t *>(out_bf16), rows, cols, tile_map(rows, cols));
  return launch(k_dequant_col<true>, dim3(tile_grid(rows, cols)), dim3(kThreads), s, c8, s8, alpha,
                static_cast<uint16_t *>(out_bf16), rows, cols, tile_map(rows, cols));
}

int nvfp4_46_fake_quant(const void *x, const nvfp4_46_params *p, const float *alpha,
                        void *out_bf16, void *stream) {
  if (!alpha || !out_bf16) return NVFP4_ERR_NULL;
  int rc = check_params(x, p, true);
  if (rc != NVFP4_OK) return rc;
  const bool xf32 = p->x_dtype == NVFP4_X_F32;
  if (!aligned16(out_bf16)) return NVFP4_ERR_ALIGN;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (p->block2d) {
    Block2dArgs a{xf32, x, alpha, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                  static_cast<uint16_t *>(out_bf16), p->rows, p->cols, p->sr_seed, s};
    return dispatch_block2d(a, p->rounding, p->select, kOutFake);
  }
  if (p->layout == NVFP4_ROWWISE) {
    FlatArgs a{xf32, static_cast<const uint4 *>(x), alpha, nullptr, nullptr, nullptr,
               static_cast<uint4 *>(out_bf16), nullptr, p->rows * p->cols / 16,
               (uint32_t)(p->cols / 16), p->sr_seed, p->rht_seed, s};
    return dispatch_flat(a, p->rounding, p->select, p->rht != 0, kOutFake);
  }
  TileArgs a{xf32, x, alpha, nullptr, nullptr, nullptr, nullptr,
             nullptr, nullptr, static_cast<uint16_t *>(out_bf16), p->rows, p->cols,
             p->sr_seed, p->rht_seed, s};
  return dispatch_tile(a, p->rounding, p->select, p->rht ? 4 : 3);
}

const char *nvfp4_46_status_string(int status) {
  switch (status) {
    case NVFP4_OK: return "ok";
    case NVFP4_ERR_NULL: return "a required pointer is NULL";
    case NVFP4_ERR_SHAPE: return "bad shape (dims must be positive, blocked axis a multiple of 16)";
    case NVFP4_ERR_ALIGN: return "buffer not 16-byte aligned";
    case NVFP4_ERR_PARAM: return "invalid parameter value";
    case NVFP4_ERR_UNSUPPORTED: return "unsupported combination of options";
    case NVFP4_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

int nvfp4_46_debug_e2m1_rtn_range(uint32_t first_bits, int64_t n, void *out_u8, void *stream) {
  if (!out_u8) return NVFP4_ERR_NULL;
  if (n <= 0) return NVFP4_ERR_SHAPE;
  return launch(k_dbg_e2m1_rtn, dim3(grid_for(n, 8)), dim3(kThreads),
                static_cast<hipStream_t>(stream), first_bits, n, static_cast<uint8_t *>(out_u8));
}

int nvfp4_46_debug_e4m3_range(uint32_t first_bits, int64_t n, void *out_u8, void *stream) {
  if (!out_u8) return NVFP4_ERR_NULL;
  if (n <= 0) return NVFP4_ERR_SHAPE;
  return launch(k_dbg_e4m3, dim3(grid_for(n, 8)), dim3(kThreads),
                static_cast<hipStream_t>(stream), first_bits, n, static_cast<uint8_t *>(out_u8));
}

int nvfp4_46_debug_decode_tables(void *out_f32, void *stream) {
  if (!out_f32) return NVFP4_ERR_NULL;
  return launch(k_dbg_tables, dim3(1), dim3(256), static_cast<hipStream_t>(stream),
                static_cast<float *>(out_f32));
}

int nvfp4_46_debug_bf16_range(uint32_t first_bits, uint32_t stride, int64_t n, void *out_u16,
                              void *stream) {
  if (!out_u16) return NVFP4_ERR_NULL;
  if (n <= 0) return NVFP4_ERR_SHAPE;
  return launch(k_dbg_bf16, dim3(grid_for(n, 8)), dim3(kThreads),
                static_cast<hipStream_t>(stream), first_bits, stride, n,
                static_cast<uint16_t *>(out_u16));
}

int nvfp4_46_debug_e2m1_sr(const float *y, const uint32_t *words, int64_t n, void *out_u8,
                           void *out_fast_u8, void *stream) {
  if (!y || !words || !out_u8 || !out_fast_u8) return NVFP4_ERR_NULL;
  if (n <= 0) return NVFP4_ERR_SHAPE;
  return launch(k_dbg_e2m1_sr, dim3(grid_for(n, 8)), dim3(kThreads),
                static_cast<hipStream_t>(stream), y, words, n, static_cast<uint8_t *>(out_u8),
                static_cast<uint8_t *>(out_fast_u8));
}

int nvfp4_46_debug_philox(const uint32_t *ctr, uint32_t key0, uint32_t key1, int64_t n,
                          uint32_t *out, void *stream) {
  if (!ctr || !out) return NVFP4_ERR_NULL;
  if (n <= 0) return NVFP4_ERR_SHAPE;
  return launch(k_dbg_philox, dim3(grid_for(n, 8)), dim3(kThreads),
                static_cast<hipStream_t>(stream), ctr, key0, key1, n, out);
}

}  // extern "C"

#endif  // NVFP4_46_MAIN
