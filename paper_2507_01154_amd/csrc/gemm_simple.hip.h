// Generic (any shape, any supported storage type) version of the per-sample contraction of Algorithm 1,
// on the vector ALUs with fp32 accumulation: used for fp32 inputs and for 16-bit inputs whose feature
// dimensions are not multiples of 8.  Same three modes and the same outputs as the matrix-core kernel.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_mfma.hip.h"

namespace flashdp {

template <int DT>
__device__ __forceinline__ float load_elem(const void* p, size_t idx) {
  if constexpr (DT == DT_F32) {
    return ((const float*)p)[idx];
  } else if constexpr (DT == DT_BF16) {
    return __builtin_bit_cast(float, (uint32_t)((const unsigned short*)p)[idx] << 16);
  } else {
    return (float)((const _Float16*)p)[idx];
  }
}

// The value of v as the scratch keeps it (rounded to bfloat16 for 16-bit inputs, unchanged for fp32): the
// squared norm of the scratch schedule is taken of these, so that the clip factor bounds what is summed.
template <int DT>
__device__ __forceinline__ float as_parked(float v) {
  if constexpr (DT == DT_F32) {
    return v;
  } else {
    return __builtin_bit_cast(float, (uint32_t)to_16bit<DT_BF16>(v) << 16);
  }
}

template <int DT>
__device__ __forceinline__ void store_scratch(void* p, size_t idx, float v) {
  if constexpr (DT == DT_F32) {
    ((float*)p)[idx] = v;
  } else {
    ((unsigned short*)p)[idx] = to_16bit<DT_BF16>(v);   // bfloat16 scratch for both 16-bit input types (range)
  }
}

// 64x64 output tile, 16-deep k steps, 256 threads, 4x4 outputs per thread.
template <int MODE, int DT>
__global__ __launch_bounds__(256) void gemm_simple_kernel(const GemmArgs a) {
  constexpr int BM = 64, BN = 64, BK = 16;
  __shared__ float As[BK][BM + 4];
  __shared__ float Bs[BK][BN + 4];
  __shared__ float red[4];
  const int tid = threadIdx.x;
  const int tiles = a.tiles_m * a.tiles_n;
  const int item = blockIdx.x;
  const int sample0 = (MODE == MODE_ACCUM) ? 0 : item / tiles;
  const int n_samples = (MODE == MODE_ACCUM) ? a.B : 1;
  const int tile = (MODE == MODE_ACCUM) ? item : item - sample0 * tiles;
  const int tm = tile / a.tiles_n, tn = tile - tm * a.tiles_n;
  const int m0 = tm * BM, n0 = tn * BN;
  const int ty = tid / 16, tx = tid % 16;   // thread owns rows m0 + 4*ty + 0..3, cols n0 + 4*tx + 0..3

  float acc[4][4];
  float tot[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) { acc[i][j] = 0.0f; tot[i][j] = 0.0f; }

  for (int s = 0; s < n_samples; ++s) {
    const size_t xa = (size_t)(sample0 + s) * a.T * a.D;
    const size_t xb = (size_t)(sample0 + s) * a.T * a.P;
    for (int t0 = 0; t0 < a.T; t0 += BK) {
      // 16 x 64 elements per operand, 4 per thread: row = e / 64, col = e % 64 with e = tid + 256 * q
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int e = tid + 256 * q, r = e / 64, c = e % 64;
        const int t = t0 + r;
        As[r][c] = (t < a.T && m0 + c < a.D) ? load_elem<DT>(a.dY, xa + (size_t)t * a.D + m0 + c) : 0.0f;
        Bs[r][c] = (t < a.T && n0 + c < a.P) ? load_elem<DT>(a.X, xb + (size_t)t * a.P + n0 + c) : 0.0f;
      }
      __syncthreads();
#pragma unroll
      for (int kk = 0; kk < BK; ++kk) {
        float av[4], bv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) av[i] = As[kk][4 * ty + i];
#pragma unroll
        for (int j = 0; j < 4; ++j) bv[j] = Bs[kk][4 * tx + j];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
      }
      __syncthreads();
    }
    if constexpr (MODE == MODE_ACCUM) {
      const float c = a.factors ? a.factors[s] : 1.0f;
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) { tot[i][j] = fmaf(c, acc[i][j], tot[i][j]); acc[i][j] = 0.0f; }
    }
  }

  if constexpr (MODE == MODE_NORM || MODE == MODE_SPILL) {
    float ss = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float g = (MODE == MODE_SPILL) ? as_parked<DT>(acc[i][j]) : acc[i][j];
        ss = fmaf(g, g, ss);
      }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    if (tid == 0) a.partials[(size_t)sample0 * tiles + tile] = (red[0] + red[1]) + (red[2] + red[3]);
    if constexpr (MODE == MODE_SPILL) {
      const size_t base = (size_t)sample0 * a.D * a.P;
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int row = m0 + 4 * ty + i, col = n0 + 4 * tx + j;
          if (row < a.D && col < a.P) store_scratch<DT>(a.scratch, base + (size_t)row * a.P + col, acc[i][j]);
        }
    }
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int row = m0 + 4 * ty + i, col = n0 + 4 * tx + j;
        if (row < a.D && col < a.P) {
          if constexpr (MODE == MODE_MATERIALIZE) {
            ((float*)a.scratch)[(size_t)sample0 * a.D * a.P + (size_t)row * a.P + col] = acc[i][j];
          } else {
            float* po = a.out + (size_t)row * a.P + col;
            *po = a.accumulate ? *po + tot[i][j] : tot[i][j];
          }
        }
      }
  }
}

}  // namespace flashdp
