// Measurement aid, not part of Algorithm 1: what the matrix cores of this part deliver when nothing else is
// in the way.  Every wave runs the instruction mix of the contraction kernel's inner loop - eight 32x32
// accumulators, four "row" and two "column" operand fragments, two fragment sets used in turn - with all
// operands resident in registers: no LDS, no memory, no barrier.  With all-zero operands the result is the
// part's issue-limited rate; with random operands it is the rate the part sustains once its clock has
// settled under a bit-toggling load, which is the ceiling any real contraction on such data runs under.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_mfma.hip.h"
#include "lds_plan.h"

namespace flashdp {

// pattern 0: zeros; 1: pseudo-random bf16 values in (-2, 2) made from a hash of the lane and fragment index;
// 4: the values of 1 with the instructions in boustrophedon order (consecutive instructions of a wave share one
// operand fragment); 5: the values of 1 with one and the same operand pair for every instruction; 6: pseudo-random
// values with eight different exponents (2^-7 .. 2) instead of two.  4-6 answer whether the rate on random data
// depends on how operands are delivered or on the values themselves.  7: the values of 1 through
// v_mfma_f32_16x16x32_bf16 (two per 32x32x16 instruction of the other patterns: the same FLOPs, half the reuse of
// an operand element inside the instruction); 9: the same instruction on zeros (its issue-limited rate).
// (one instantiation per pattern: in a single kernel with a run-time switch the patterns disturbed each other's code)
template <int pattern>
__global__ __launch_bounds__(512, 2) void mfma_probe_kernel(int iters, float* __restrict__ sink) {
  const uint32_t gid = blockIdx.x * 512u + threadIdx.x;
  s16x8_t fa[2][4], fb[2][2];
  auto fill = [&](s16x8_t& f, uint32_t salt) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      uint32_t h = (gid * 0x9E3779B9u) ^ (salt * 0x85EBCA6Bu) ^ ((uint32_t)e * 0xC2B2AE35u);
      h ^= h >> 15; h *= 0x2C1B3C6Du; h ^= h >> 12; h *= 0x297A2D39u; h ^= h >> 15;
      // sign and 7 mantissa bits from the hash, exponent of 0.5 .. 2 (pattern 6: of 2^-7 .. 2)
      const uint32_t ex = pattern == 6 ? 120u + ((h >> 16) % 8u) : 126u + ((h >> 16) % 2u);
      const uint32_t bits = (h & 0x8000u) | (ex << 7) | (h & 0x7Fu);
      f[e] = (pattern && pattern != 9) ? (short)bits : (short)0;   // (10, 11: random)
    }
  };
#pragma unroll
  for (int s = 0; s < 2; ++s) {
#pragma unroll
    for (int i = 0; i < 4; ++i) fill(fa[s][i], 16u * s + i);
#pragma unroll
    for (int j = 0; j < 2; ++j) fill(fb[s][j], 16u * s + 8u + j);
  }
  f32x16_t acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
  if constexpr (pattern == 4) {
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int jj = 0; jj < 2; ++jj) {
            const int j = (i & 1) ? 1 - jj : jj;
            acc[i][j] = mfma32<DT_BF16>(fb[s][j], fa[s][i], acc[i][j]);
          }
    }
  } else if constexpr (pattern == 10 || pattern == 11) {
    // 16x16x32 on random operands with the accumulators updated in place (inline assembly), held in the
    // accumulation registers (10) or in ordinary vector registers (11)
    typedef float f32x4_t __attribute__((ext_vector_type(4)));
    f32x4_t small[4][2][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int h = 0; h < 2; ++h) small[i][j][h] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
              if constexpr (pattern == 10) asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(small[i][j][h]) : "v"(fb[s][j]), "v"(fa[s][i]));
              else asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(small[i][j][h]) : "v"(fb[s][j]), "v"(fa[s][i]));
            }
    }
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[i][j][e] += small[i][j][h][e];
  } else if constexpr (pattern == 7 || pattern == 9) {
    typedef float f32x4_t __attribute__((ext_vector_type(4)));
    f32x4_t small[4][2][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int h = 0; h < 2; ++h) small[i][j][h] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int h = 0; h < 2; ++h)
              small[i][j][h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, fb[s][j]), __builtin_bit_cast(bf16x8_t, fa[s][i]),
                                                                       small[i][j][h], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[i][j][e] += small[i][j][h][e];
  } else if constexpr (pattern == 5) {
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j) acc[i][j] = mfma32<DT_BF16>(fb[0][0], fa[0][0], acc[i][j]);
    }
  } else {
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j) acc[i][j] = mfma32<DT_BF16>(fb[s][j], fa[s][i], acc[i][j]);
    }
  }
  float t = 0.0f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) t += acc[i][j][e];
  if (t == 12345.678f) sink[0] = t;   // keeps the loop alive; never true for these operands
}

// The same instruction mix with the operand fragments coming from LDS through the transposed reads of the
// contraction kernel (a 32 KB stage filled once with zeros or pseudo-random values, re-read every k-tile):
// matrix cores + LDS traffic, still no memory loads and no barrier in the loop.
// RANDOM: pseudo-random instead of zero operands.  FORM 0: 32x32x16; 1: 16x16x32 (two per 32x32x16 instruction);
// 2: 16x16x32 with a third fewer fragment reads (the X fragments are read once, not every k-step): what a tiling with
// 128 x 128 per wave would save in LDS traffic.
template <bool RANDOM, int FORM>
__global__ __launch_bounds__(512, 2) void mfma_lds_probe_kernel(int iters, float* __restrict__ sink) {
  extern __shared__ __attribute__((aligned(16))) unsigned short lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave % 2, wave_n = wave / 2;
  for (int e = tid; e < lds_plan::STAGE_ELEMS; e += 512) {
    uint32_t h = ((uint32_t)e * 0x9E3779B9u) ^ (blockIdx.x * 0x85EBCA6Bu);
    h ^= h >> 15; h *= 0x2C1B3C6Du; h ^= h >> 12; h *= 0x297A2D39u; h ^= h >> 15;
    const uint32_t bits = (h & 0x8000u) | ((126u + ((h >> 16) % 2u)) << 7) | (h & 0x7Fu);
    lds[e] = RANDOM ? (unsigned short)bits : (unsigned short)0;
  }
  __syncthreads();
  int a_rd[4], b_rd[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) a_rd[i] = lds_plan::frag_offset(lane, wave_m * 4 + i);
#pragma unroll
  for (int j = 0; j < 2; ++j) b_rd[j] = lds_plan::OPERAND_ELEMS + lds_plan::frag_offset(lane, wave_n * 2 + j);
  s16x8_t fa[2][4], fb[2][2];
  auto load_frags = [&](int ks, s16x8_t* pfa, s16x8_t* pfb) {
    const unsigned short* base = lds + ks * 16 * lds_plan::ROW;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const s16x4_t lo = lds_read_tr(base + a_rd[i]);
      const s16x4_t hi = lds_read_tr(base + a_rd[i] + 4 * lds_plan::ROW);
      pfa[i] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const s16x4_t lo = lds_read_tr(base + b_rd[j]);
      const s16x4_t hi = lds_read_tr(base + b_rd[j] + 4 * lds_plan::ROW);
      pfb[j] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
  };
  auto load_a_frags = [&](int ks, s16x8_t* pfa) {
    const unsigned short* base = lds + ks * 16 * lds_plan::ROW;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const s16x4_t lo = lds_read_tr(base + a_rd[i]);
      const s16x4_t hi = lds_read_tr(base + a_rd[i] + 4 * lds_plan::ROW);
      pfa[i] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
  };
  f32x16_t acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
  load_frags(0, fa[0], fb[0]);
  load_frags(1, fa[1], fb[1]);
  if constexpr (FORM != 0) {   // the same fragment traffic feeding 16x16x32 instructions, two per 32x32x16 one
    typedef float f32x4_t __attribute__((ext_vector_type(4)));
    f32x4_t small[4][2][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int h = 0; h < 2; ++h) small[i][j][h] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
    for (int it = 0; it < iters; ++it) {
      static_for<2>([&](auto ks_c) {
        constexpr int ks = decltype(ks_c)::value;
        if constexpr (FORM == 2) load_a_frags(ks ^ 1, fa[ks ^ 1]); else load_frags(ks ^ 1, fa[ks ^ 1], fb[ks ^ 1]);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int h = 0; h < 2; ++h)
              small[i][j][h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, fb[ks][j]), __builtin_bit_cast(bf16x8_t, fa[ks][i]),
                                                                       small[i][j][h], 0, 0, 0);
        sched_interleave<0, 16, FORM == 2 ? 8 : 12, 0, 0>();
      });
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[i][j][e] += small[i][j][h][e];
  } else {
  for (int it = 0; it < iters; ++it) {
    static_for<2>([&](auto ks_c) {
      constexpr int ks = decltype(ks_c)::value;
      load_frags(ks ^ 1, fa[ks ^ 1], fb[ks ^ 1]);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = mfma32<DT_BF16>(fb[ks][j], fa[ks][i], acc[i][j]);
      sched_interleave<0, 8, 12, 0, 0>();
    });
  }
  }
  float t = 0.0f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) t += acc[i][j][e];
  if (t == 12345.678f) sink[0] = t;
}

}  // namespace flashdp
