// Per-sample weight-gradient contraction for fp32 inputs on the gfx950 matrix cores
// (v_mfma_f32_32x32x2_f32, fp32 in, fp32 accumulate): the fp32 counterpart of gemm_mfma.hip.h, same
// modes, same tiling (256x256 output tile, 8 waves of 128x64, two LDS stages), same workgroup -> tile map.
//
// Operands: lane l of the instruction holds A[r = l % 32][k = l / 32] and B[k = l / 32][c = l % 32], one
// float each.  The LDS tiles are stored as in HBM (rows = t), so a fragment is one 4-byte LDS read per lane:
// row (2 ks + l / 32), column (block + l % 32): 32 consecutive floats per half-wave, and with a row pitch
// of 32 floats mod 64 the two half-waves fall in disjoint banks.  No transpose is needed for 32-bit data.
// As in the 16-bit kernel the X fragment is the row operand, so a lane owns one output row and, per four
// accumulator registers, four consecutive output columns (16-byte stores).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_mfma.hip.h"

namespace flashdp {

struct F32Cfg {
  static constexpr int BM = 256, BN = 256, BK = 16, WAVES_M = 2, WAVES_N = 4, NT = 512;
  static constexpr int TM = 128, TN = 64, FM = 4, FN = 2;
  static constexpr int LDA = BM + 32, LDB = BN + 32;               // floats; 288 = 32 mod 64
  static constexpr int A_STAGE = BK * LDA, B_STAGE = BK * LDB;     // floats per stage
  static constexpr int LDS_BYTES = 2 * (A_STAGE + B_STAGE) * 4;    // 73 728
  static constexpr int CPR = BM / 4;                               // 16-byte chunks per row
  static constexpr int RSTEP = NT / CPR;                           // rows covered by one pass of the workgroup
  static constexpr int CA = BK / RSTEP, CB = BK / RSTEP;           // chunks per thread per k-tile
  static constexpr int KS = BK / 2;                                // matrix-core k-steps per k-tile
};

template <int MODE>
__global__ __launch_bounds__(512, 2) void gemm_mfma_f32_kernel(const GemmArgs a) {
  using C = F32Cfg;
  constexpr int FM = C::FM, FN = C::FN, LDA = C::LDA, LDB = C::LDB, KS = C::KS;
  extern __shared__ __attribute__((aligned(16))) float ldsf[];
  float* const As = ldsf;                     // [2][BK][LDA]
  float* const Bs = ldsf + 2 * C::A_STAGE;    // [2][BK][LDB]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave % C::WAVES_M, wave_n = wave / C::WAVES_M;
  const int tiles = a.tiles_m * a.tiles_n;
  int sample0 = 0, tile;
  if constexpr (MODE == MODE_ACCUM) {
    tile = xcd_remap(blockIdx.x, tiles);
  } else {
    if (!shared_block_item(blockIdx.x, tiles, a.B, &sample0, &tile)) return;   // the whole workgroup, before any barrier
  }
  const int n_samples = (MODE == MODE_ACCUM) ? a.B : 1;
  int tm, tn;
  tile_coords<8>(tile, a.tiles_m, a.tiles_n, &tm, &tn);
  const int m0 = tm * C::BM, n0 = tn * C::BN;

  // global -> LDS copy plan (16-byte chunks of 4 floats; out-of-range columns are sent beyond num_records)
  const int c_row = tid / C::CPR, c_cc = tid % C::CPR;
  const bool a_ok = m0 + c_cc * 4 < a.D, b_ok = n0 + c_cc * 4 < a.P;
  const uint32_t a_off0 = a_ok ? (uint32_t)(c_row * a.D + m0 + c_cc * 4) * 4u : 0x80000000u;
  const uint32_t b_off0 = b_ok ? (uint32_t)(c_row * a.P + n0 + c_cc * 4) * 4u : 0x80000000u;
  const uint32_t a_rstep = (uint32_t)(C::RSTEP * a.D) * 4u, b_rstep = (uint32_t)(C::RSTEP * a.P) * 4u;
  const uint32_t a_kstep = (uint32_t)(C::BK * a.D) * 4u, b_kstep = (uint32_t)(C::BK * a.P) * 4u;
  const uint32_t a_bytes = (uint32_t)a.T * (uint32_t)a.D * 4u, b_bytes = (uint32_t)a.T * (uint32_t)a.P * 4u;
  const int a_lds_w = c_row * LDA + c_cc * 4, b_lds_w = c_row * LDB + c_cc * 4;

  const int kt_per_sample = (a.T + C::BK - 1) / C::BK;
  const int nk = kt_per_sample * n_samples;

  u32x4_t ra[C::CA], rb[C::CB];
  int ld_s = 0, ld_kt = 0;   // fetch cursor; parks past the end on rows >= T, which read as zeros
  auto load_global = [&]() {
    const char* pa = (const char*)a.dY + (size_t)(sample0 + ld_s) * a_bytes;
    const char* pb = (const char*)a.X + (size_t)(sample0 + ld_s) * b_bytes;
    const __amdgpu_buffer_rsrc_t rsa = make_rsrc(pa, a_bytes), rsb = make_rsrc(pb, b_bytes);
    const uint32_t ao = a_off0 + (uint32_t)ld_kt * a_kstep, bo = b_off0 + (uint32_t)ld_kt * b_kstep;
#pragma unroll
    for (int j = 0; j < C::CA; ++j) ra[j] = __builtin_amdgcn_raw_buffer_load_b128(rsa, (int)(ao + j * a_rstep), 0, 0);
#pragma unroll
    for (int j = 0; j < C::CB; ++j) rb[j] = __builtin_amdgcn_raw_buffer_load_b128(rsb, (int)(bo + j * b_rstep), 0, 0);
    ld_kt += 1;
    const bool wrap = ld_kt >= kt_per_sample && ld_s + 1 < n_samples;
    ld_s = wrap ? ld_s + 1 : ld_s;
    ld_kt = wrap ? 0 : ld_kt;
  };
  auto store_lds = [&](int stage) {
    float* pa = As + stage * C::A_STAGE + a_lds_w;
    float* pb = Bs + stage * C::B_STAGE + b_lds_w;
#pragma unroll
    for (int j = 0; j < C::CA; ++j) *(u32x4_t*)(pa + j * C::RSTEP * LDA) = ra[j];
#pragma unroll
    for (int j = 0; j < C::CB; ++j) *(u32x4_t*)(pb + j * C::RSTEP * LDB) = rb[j];
  };

  // fragment read plan: lane -> row (l / 32) of the 2-row k-step, column (l % 32) of the 32-wide block
  const int a_lds_r = (lane >> 5) * LDA + wave_m * C::TM + (lane & 31);
  const int b_lds_r = (lane >> 5) * LDB + wave_n * C::TN + (lane & 31);
  float fa[2][FM], fb[2][FN];
  auto load_frags = [&](int stage, int ks, float* pfa, float* pfb) {
    const float* pa = As + stage * C::A_STAGE + a_lds_r + ks * 2 * LDA;
    const float* pb = Bs + stage * C::B_STAGE + b_lds_r + ks * 2 * LDB;
#pragma unroll
    for (int i = 0; i < FM; ++i) pfa[i] = pa[i * 32];
#pragma unroll
    for (int j = 0; j < FN; ++j) pfb[j] = pb[j * 32];
  };

  f32x16_t acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  load_global();
  store_lds(0);
  load_global();
  __syncthreads();
  load_frags(0, 0, fa[0], fb[0]);

  for (int k = 0; k < nk; ++k) {
    const int cur = k & 1;
    static_for<KS>([&](auto ks_c) {
      constexpr int ks = decltype(ks_c)::value;
      constexpr int cb = ks & 1, nb = cb ^ 1;
      if constexpr (ks + 1 < KS) {
        load_frags(cur, ks + 1, fa[nb], fb[nb]);
      } else {
        __syncthreads();   // tile k+1 is in LDS, and every wave has read the last fragments of tile k
        load_frags(cur ^ 1, 0, fa[nb], fb[nb]);
      }
      constexpr bool do_store = ks == KS / 2 - 1, do_fetch = ks == KS - 2;
      if constexpr (do_store) store_lds(cur ^ 1);
      if constexpr (do_fetch) load_global();
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fb[cb][j], fa[cb][i], acc[i][j], 0, 0, 0);
      // keep the fragment reads of the next k-step (and the tile copy) between this k-step's matrix-core
      // instructions instead of in front of the ones that consume them
      sched_interleave<0, FM * FN, FM + FN, do_store ? C::CA + C::CB : 0, do_fetch ? C::CA + C::CB : 0>();
    });
    if constexpr (MODE == MODE_ACCUM) {
      // sample boundary: keep acc = sum_{j<=i} (c_j / c_i) G_j (see the 16-bit kernel)
      if (a.factors != nullptr && (k + 1) % kt_per_sample == 0) {
        const int s = k / kt_per_sample;
        const float ratio = (s + 1 < n_samples) ? a.factors[s] / a.factors[s + 1] : a.factors[s];
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
          for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] *= ratio;
      }
    }
  }
  __syncthreads();

  // epilogue.  acc[i][j][4q + r] = G[m0 + wave_m*TM + 32i + lane%32][n0 + wave_n*TN + 32j + 8q + 4(lane/32) + r]
  const int row_base = m0 + wave_m * C::TM + (lane & 31);
  const int col_base = n0 + wave_n * C::TN + 4 * (lane >> 5);
  if constexpr (MODE == MODE_NORM || MODE == MODE_SPILL) {
    float ss = 0.0f;
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) ss = fmaf(acc[i][j][e], acc[i][j][e], ss);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
    float* red = ldsf;
    if (lane == 0) red[wave] = ss;
    __syncthreads();
    if (tid == 0) {
      float tot = 0.0f;
      for (int w = 0; w < C::NT / 64; ++w) tot += red[w];
      a.partials[(size_t)sample0 * tiles + tile] = tot;
    }
  }
  if constexpr (MODE != MODE_NORM) {
    float* obase = a.out;
    if constexpr (MODE == MODE_SPILL || MODE == MODE_MATERIALIZE) obase = (float*)a.scratch + (size_t)sample0 * a.D * a.P;
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      const int row = row_base + i * 32;
      if (row >= a.D) continue;
      float* prow = obase + (size_t)row * a.P;
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int col = col_base + j * 32 + 8 * q;
          if (col < a.P) {   // P is a multiple of 4 on this path: a 4-column group is all in or all out
            float4 v = make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
            if (MODE == MODE_ACCUM && a.accumulate) {
              const float4 o = *(const float4*)(prow + col);
              v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w;
            }
            *(float4*)(prow + col) = v;
          }
        }
    }
  }
}

}  // namespace flashdp
