// Per-sample gradient norms WITHOUT forming the gradient: the "ghost clipping" route the paper cites among
// the implicit methods (Section 2, related work; Figure "compare" (c)).  For one sample
//
//   ||dY^T X||_F^2 = sum_{t,t'} (x_t . x_t') (dy_t . dy_t') = < X X^T , dY dY^T >_F ,
//
// two T x T Gram matrices and their elementwise dot product.  Built as a measured comparison schedule: its
// cost is 2 T^2 (P + D) per sample (half of that here, both Gram matrices being symmetric) against
// 2 T P D for the gradient itself, so it pays only for short sequences - the trade the paper's Table 1
// discussion describes.  The clip factors it yields feed the same clipped batch accumulation as the
// two-pass schedule.
//
// A workgroup owns one 128 x 128 block (bi <= bj) of both Gram matrices of one sample: it runs the X
// contraction over P into one set of accumulators, the dY contraction over D into a second set with the
// same register layout, multiplies the two elementwise, reduces, and writes one partial (weighted 2 for
// off-diagonal blocks).  Here the reduction index (p resp. d) is the contiguous one, so the matrix-core
// operands are plain 16-byte LDS reads (lane l: row l % 32, k = 8 * (l / 32) .. + 7) and no transpose is needed.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_mfma.hip.h"
#include "gemm_simple.hip.h"

namespace flashdp {

struct GramArgs {
  const void* X;    // [B][T][P]
  const void* dY;   // [B][T][D]
  int B, T, P, D;
  int nb;           // ceil(T / block)
  int n_tri;        // nb * (nb + 1) / 2 blocks on or above the diagonal
  float* partials;  // [B][n_tri]
};

// r = bj * (bj + 1) / 2 + bi with bi <= bj
__device__ __forceinline__ void tri_decode(int r, int* bi, int* bj) {
  int j = (int)((sqrtf(8.0f * (float)r + 1.0f) - 1.0f) * 0.5f);
  while (j * (j + 1) / 2 > r) --j;
  while ((j + 1) * (j + 2) / 2 <= r) ++j;
  *bj = j;
  *bi = r - j * (j + 1) / 2;
}

struct GramCfg {
  static constexpr int BT = 128, BK = 64, NT = 256;
  static constexpr int LD = BK + 8;                 // 144-byte rows: 16 consecutive rows read 16 distinct 16-byte bank groups
  static constexpr int STAGE = BT * LD;             // elements per operand per stage
  static constexpr int LDS_BYTES = 2 * 2 * STAGE * 2;
  static constexpr int CH = BT * BK / 8 / NT;       // 16-byte chunks per thread per operand per k-tile
};

template <int DT>
__global__ __launch_bounds__(GramCfg::NT, 2) void gram_norm_mfma_kernel(const GramArgs a) {
  constexpr int BT = GramCfg::BT, BK = GramCfg::BK, NT = GramCfg::NT, LD = GramCfg::LD, CH = GramCfg::CH;
  extern __shared__ __attribute__((aligned(16))) unsigned short lds[];
  unsigned short* const As = lds;                        // [2][BT][LD]  rows of block bi
  unsigned short* const Bs = lds + 2 * GramCfg::STAGE;   // [2][BT][LD]  rows of block bj

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave & 1, wave_n = wave >> 1;
  const int item = xcd_remap(blockIdx.x, a.B * a.n_tri);
  const int sample = item / a.n_tri;
  int bi, bj;
  tri_decode(item - sample * a.n_tri, &bi, &bj);

  const int ld_row = tid >> 3, ld_kc = tid & 7;          // thread copies chunk ld_kc of rows ld_row + 32 j
  const int lds_w = ld_row * LD + ld_kc * 8;
  const int fr_a = (wave_m * 64 + (lane & 31)) * LD + 8 * (lane >> 5);
  const int fr_b = (wave_n * 64 + (lane & 31)) * LD + 8 * (lane >> 5);

  f32x16_t acc[2][2][2];   // [which Gram matrix][i][j]
#pragma unroll
  for (int g = 0; g < 2; ++g)
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[g][i][j][e] = 0.0f;

  static_for<2>([&](auto g_c) {
    constexpr int g = decltype(g_c)::value;
    const int K = g == 0 ? a.P : a.D;
    const char* base = (const char*)(g == 0 ? a.X : a.dY) + (size_t)sample * a.T * K * 2;
    const uint32_t bytes = (uint32_t)a.T * (uint32_t)K * 2u;   // rows >= T lie beyond it and read zeros
    const __amdgpu_buffer_rsrc_t rs = make_rsrc(base, bytes);
    const uint32_t off_a = (uint32_t)((bi * BT + ld_row) * K + ld_kc * 8) * 2u;
    const uint32_t off_b = (uint32_t)((bj * BT + ld_row) * K + ld_kc * 8) * 2u;
    const uint32_t rstep = (uint32_t)(32 * K) * 2u;
    const int nk = (K + BK - 1) / BK;
    u32x4_t ra[CH], rb[CH];
    auto load_global = [&](int kt) {
      // a chunk whose columns lie beyond K (K is a multiple of 8: all in or all out) is sent past the
      // buffer's end and reads zeros; so does every chunk of a k-tile past the last one
      const bool ok = kt * BK + ld_kc * 8 < K;
      const uint32_t ko = (uint32_t)(kt * BK) * 2u;
#pragma unroll
      for (int j = 0; j < CH; ++j) {
        ra[j] = __builtin_amdgcn_raw_buffer_load_b128(rs, ok ? (int)(off_a + ko + j * rstep) : (int)0x80000000u, 0, 0);
        rb[j] = __builtin_amdgcn_raw_buffer_load_b128(rs, ok ? (int)(off_b + ko + j * rstep) : (int)0x80000000u, 0, 0);
      }
    };
    auto store_lds = [&](int stage) {
#pragma unroll
      for (int j = 0; j < CH; ++j) {
        *(u32x4_t*)(As + stage * GramCfg::STAGE + lds_w + j * 32 * LD) = ra[j];
        *(u32x4_t*)(Bs + stage * GramCfg::STAGE + lds_w + j * 32 * LD) = rb[j];
      }
    };
    __syncthreads();   // the previous Gram matrix's last reads are done before stage 0 is overwritten
    load_global(0);
    store_lds(0);
    load_global(1);
    __syncthreads();
    // fragments are double-buffered in registers: the reads of k-step ks + 1 go out before the matrix-core
    // instructions of k-step ks (the first reads of the next k-tile right after the barrier)
    constexpr int KS = BK / 16;
    s16x8_t fa[2][2], fb[2][2];
    auto load_frags = [&](int stage, int ks, s16x8_t* pfa, s16x8_t* pfb) {
      const unsigned short* pa = As + stage * GramCfg::STAGE + fr_a + ks * 16;
      const unsigned short* pb = Bs + stage * GramCfg::STAGE + fr_b + ks * 16;
#pragma unroll
      for (int i = 0; i < 2; ++i) pfa[i] = *(const s16x8_t*)(pa + i * 32 * LD);
#pragma unroll
      for (int j = 0; j < 2; ++j) pfb[j] = *(const s16x8_t*)(pb + j * 32 * LD);
    };
    load_frags(0, 0, fa[0], fb[0]);
    for (int kt = 0; kt < nk; ++kt) {
      const int cur = kt & 1;
      static_for<KS>([&](auto ks_c) {
        constexpr int ks = decltype(ks_c)::value;
        constexpr int cb = ks & 1, nb = cb ^ 1;
        constexpr bool copy = ks == 0;
        if constexpr (ks + 1 < KS) {
          load_frags(cur, ks + 1, fa[nb], fb[nb]);
        } else {
          __syncthreads();   // tile kt + 1 is in LDS and every wave has read the last fragments of tile kt
          load_frags(cur ^ 1, 0, fa[nb], fb[nb]);
        }
        if constexpr (copy) {
          store_lds(cur ^ 1);     // tile kt + 1 (in registers since the last trip) to the other stage
          load_global(kt + 2);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j) acc[g][i][j] = mfma32<DT>(fa[cb][i], fb[cb][j], acc[g][i][j]);
        sched_interleave<0, 4, 4, copy ? 2 * CH : 0, copy ? 2 * CH : 0>();
      });
    }
  });

  // <X X^T, dY dY^T> over this block: both accumulator sets have the same element -> register mapping
  float ss = 0.0f;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) ss = fmaf(acc[0][i][j][e], acc[1][i][j][e], ss);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
  float* red = (float*)lds;   // operand tiles are dead: the main loop ended with a barrier
  if (lane == 0) red[wave] = ss;
  __syncthreads();
  if (tid == 0) {
    const float tot = (red[0] + red[1]) + (red[2] + red[3]);
    a.partials[(size_t)sample * a.n_tri + (item - sample * a.n_tri)] = (bi == bj) ? tot : 2.0f * tot;
  }
}

// Any shape and storage type, vector ALUs: 64 x 64 block of both Gram matrices, 4 x 4 entries per thread.
template <int DT>
__global__ __launch_bounds__(256) void gram_norm_simple_kernel(const GramArgs a) {
  constexpr int BT = 64, BK = 16;
  __shared__ float As[BK][BT + 4];
  __shared__ float Bs[BK][BT + 4];
  __shared__ float red[4];
  const int tid = threadIdx.x;
  const int item = blockIdx.x;
  const int sample = item / a.n_tri;
  int bi, bj;
  tri_decode(item - sample * a.n_tri, &bi, &bj);
  const int ty = tid / 16, tx = tid % 16;

  float acc[2][4][4];
#pragma unroll
  for (int g = 0; g < 2; ++g)
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[g][i][j] = 0.0f;

#pragma unroll
  for (int g = 0; g < 2; ++g) {
    const int K = g == 0 ? a.P : a.D;
    const void* src = g == 0 ? a.X : a.dY;
    const size_t base = (size_t)sample * a.T * K;
    for (int k0 = 0; k0 < K; k0 += BK) {
      // 64 rows x 16 k per operand, 4 elements per thread; stored k-major
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int e = tid + 256 * q, r = e / BK, c = e % BK;
        const int ta = bi * BT + r, tb = bj * BT + r, k = k0 + c;
        As[c][r] = (ta < a.T && k < K) ? load_elem<DT>(src, base + (size_t)ta * K + k) : 0.0f;
        Bs[c][r] = (tb < a.T && k < K) ? load_elem<DT>(src, base + (size_t)tb * K + k) : 0.0f;
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
          for (int j = 0; j < 4; ++j) acc[g][i][j] = fmaf(av[i], bv[j], acc[g][i][j]);
      }
      __syncthreads();
    }
  }
  float ss = 0.0f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) ss = fmaf(acc[0][i][j], acc[1][i][j], ss);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
  if ((tid & 63) == 0) red[tid >> 6] = ss;
  __syncthreads();
  if (tid == 0) {
    const float tot = (red[0] + red[1]) + (red[2] + red[3]);
    a.partials[(size_t)sample * a.n_tri + (item - sample * a.n_tri)] = (bi == bj) ? tot : 2.0f * tot;
  }
}

}  // namespace flashdp
