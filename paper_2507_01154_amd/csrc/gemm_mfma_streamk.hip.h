// Non-private weight gradient out = sum_i dY_i^T X_i (Appendix B.1, Eq. "batched-grad") with the work balanced
// over the chip whatever the tile count: the comparator the DP path is held against, so that its ratio is not
// flattered by a plain GEMM whose last round of workgroups runs half empty (400 tiles of 256x256 on 256 CUs).
//
// Same tile, ring of direct-to-LDS loads, fragment reads and matrix-core loop as gemm_mfma_dma_kernel in its
// batch-accumulating mode; what differs is who computes what.  The output is cut into blocks of 32 tiles (8 tile
// rows x 4 tile columns, the group that shares 12 operand panels in one XCD's L2).  A block costs nk k-tiles of
// time on the 32 CUs of one XCD (nk = all samples' k-tiles, one after the other).  The 8 XCDs are each dealt the
// same number of (block, k-tile) units, a contiguous range: an XCD walks its range block by block, its 32 workgroups
// in step on the 32 tiles of the block over the same k-range, so the L2 sharing of the per-sample kernel is kept,
// while a block at the edge of a range is cut along the reduction index between neighbouring XCDs.  A tile whose
// whole reduction ran in one piece is stored straight to out; pieces of a cut tile go to fp32 partial tiles and a
// small second kernel adds them in a fixed order (no atomics: bit-repeatable).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_mfma_dma.hip.h"
#include "streamk_plan.h"

namespace flashdp {

struct StreamKArgs {
  const void* X;        // [B][T][P]
  const void* dY;       // [B][T][D]
  int B, T, P, D;
  int tiles_m, tiles_n;
  int n_blocks;         // ceil(tiles / 32)
  int nk_pad;           // k-tiles per output tile over the whole batch, rounded up to a multiple of the ring depth
  int units_per_xcd;    // (block, k-tile) units per range, a multiple of the ring depth
  float* out;           // [D][P]
  float* partial;       // [STREAMK_SLOTS][32][256][256] fp32 pieces of cut tiles
};

// Which partial slots make up each cut block, in the order of the reduction index (filled by the host with the
// same walk the kernel does).
struct StreamKCuts {
  int n;
  int block[STREAMK_MAX_CUT];
  int count[STREAMK_MAX_CUT];
  int slot[STREAMK_MAX_CUT][STREAMK_XCDS];
};

template <typename Cfg, int DT>
__global__ __launch_bounds__(Cfg::NT, Cfg::WAVES_PER_EU) void gemm_mfma_streamk_kernel(const StreamKArgs a) {
  constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, FM = Cfg::FM, FN = Cfg::FN, STAGES = Cfg::STAGES;
  constexpr int ROW = 256;
  extern __shared__ __attribute__((aligned(16))) unsigned short lds[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wave_m = wave % Cfg::WAVES_M, wave_n = wave / Cfg::WAVES_M;
  const int xcd = blockIdx.x & 7, w = blockIdx.x >> 3;
  const int tiles = a.tiles_m * a.tiles_n;

  const int d_row = lds_plan::load_row(wave, lane);
  const int d_chunk = lds_plan::load_chunk(wave, lane);
  const uint32_t a_half = (uint32_t)(16 * a.D) * 2u, b_half = (uint32_t)(16 * a.P) * 2u;
  const uint32_t a_kstep = (uint32_t)(BK * a.D) * 2u, b_kstep = (uint32_t)(BK * a.P) * 2u;
  const uint32_t a_bytes = (uint32_t)a.T * (uint32_t)a.D * 2u, b_bytes = (uint32_t)a.T * (uint32_t)a.P * 2u;
  const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned short*)lds;
  const int kt_per_sample = (a.T + BK - 1) / BK;

  int a_rd[FM], b_rd[FN];
#pragma unroll
  for (int i = 0; i < FM; ++i) a_rd[i] = lds_plan::frag_offset(lane, wave_m * FM + i);
#pragma unroll
  for (int j = 0; j < FN; ++j) b_rd[j] = Cfg::A_ELEMS + lds_plan::frag_offset(lane, wave_n * FN + j);

  streamk_walk(xcd, a.n_blocks, a.nk_pad, a.units_per_xcd, [&](const StreamKPiece& pc) {
    const int tile = pc.block * STREAMK_WG_PER_XCD + w;
    if (tile >= tiles) return;   // a ragged last block: this workgroup has no tile in it (uniform over the workgroup)
    int tm, tn;
    tile_coords<8>(tile, a.tiles_m, a.tiles_n, &tm, &tn);
    const int m0 = tm * BM, n0 = tn * BN;
    const bool a_ok = m0 + d_chunk * 8 < a.D;
    const bool b_ok = n0 + d_chunk * 8 < a.P;
    const uint32_t a_off0 = a_ok ? (uint32_t)(d_row * a.D + m0 + d_chunk * 8) * 2u : 0x80000000u;
    const uint32_t b_off0 = b_ok ? (uint32_t)(d_row * a.P + n0 + d_chunk * 8) * 2u : 0x80000000u;

    // Fetch cursor: starts at k-tile k0 of the batch-long reduction; past the last sample it parks on rows >= T.
    int ld_s = pc.k0 / kt_per_sample;
    ld_s = ld_s < a.B ? ld_s : a.B - 1;
    int ld_kt = pc.k0 - ld_s * kt_per_sample;
    auto issue_loads = [&](int stage) {
      const char* pa = (const char*)a.dY + (size_t)ld_s * a_bytes;
      const char* pb = (const char*)a.X + (size_t)ld_s * b_bytes;
      const u32x4_t rsa = make_rsrc_words(pa, a_bytes), rsb = make_rsrc_words(pb, b_bytes);
      const uint32_t ao = a_off0 + (uint32_t)ld_kt * a_kstep, bo = b_off0 + (uint32_t)ld_kt * b_kstep;
      load_to_lds(rsa, ao, lds_base + lds_plan::load_dst_bytes(stage, 0, wave, 0));
      load_to_lds(rsa, ao + a_half, lds_base + lds_plan::load_dst_bytes(stage, 0, wave, 1));
      load_to_lds(rsb, bo, lds_base + lds_plan::load_dst_bytes(stage, 1, wave, 0));
      load_to_lds(rsb, bo + b_half, lds_base + lds_plan::load_dst_bytes(stage, 1, wave, 1));
      ld_kt += 1;
      const bool wrap = ld_kt >= kt_per_sample && ld_s + 1 < a.B;
      ld_s = wrap ? ld_s + 1 : ld_s;
      ld_kt = wrap ? 0 : ld_kt;
    };

    f32x16_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    s16x8_t fa[2][FM], fb[2][FN];
    auto load_frags = [&](int stage, int ks, s16x8_t* pfa, s16x8_t* pfb) {
      const unsigned short* base = lds + stage * Cfg::STAGE_ELEMS + ks * 16 * ROW;
#pragma unroll
      for (int i = 0; i < FM; ++i) {
        const s16x4_t lo = lds_read_tr(base + a_rd[i]);
        const s16x4_t hi = lds_read_tr(base + a_rd[i] + 4 * ROW);
        pfa[i] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      }
#pragma unroll
      for (int j = 0; j < FN; ++j) {
        const s16x4_t lo = lds_read_tr(base + b_rd[j]);
        const s16x4_t hi = lds_read_tr(base + b_rd[j] + 4 * ROW);
        pfb[j] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      }
    };

#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s) issue_loads(s);
    wait_loads_outstanding<4 * (STAGES - 2)>();   // the first k-tile has landed (and the previous piece's stores are done)
    __syncthreads();
    load_frags(0, 0, fa[0], fb[0]);

    constexpr int N_MMA = FM * FN, N_RD = 2 * (FM + FN);
    auto k_tile = [&](auto cur_c) {
      constexpr int cur = decltype(cur_c)::value;
      constexpr int nxt = (cur + 1) % STAGES, refill = (cur + STAGES - 1) % STAGES;
      load_frags(cur, 1, fa[1], fb[1]);
      issue_loads(refill);
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) acc[i][j] = mfma32<DT>(fb[0][j], fa[0][i], acc[i][j]);
      sched_interleave<0, N_MMA, N_RD, 0, 0>();
      wait_loads_outstanding<4 * (STAGES - 2)>();
      __syncthreads();
      load_frags(nxt, 0, fa[0], fb[0]);
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) acc[i][j] = mfma32<DT>(fb[1][j], fa[1][i], acc[i][j]);
      sched_interleave<0, N_MMA, N_RD, 0, 0>();
    };
    // k1 - k0 is a multiple of the ring depth (range boundaries and nk_pad are); the k-tiles between the true end
    // of the reduction and nk_pad read the zeros the parked loads deliver.  The loads issued past k1 land in stages
    // nobody reads again before the next piece's own loads replace them.
    for (int k = pc.k0; k < pc.k1; k += STAGES) {
      static_for<STAGES>([&](auto s_c) { k_tile(s_c); });
    }
    wait_loads_outstanding<0>();
    __syncthreads();   // every wave is done with the ring before the next piece refills it

    // acc[i][j][4q + r] = G[m0 + wave_m*TM + 32i + lane%32][n0 + wave_n*TN + 32j + 8q + 4(lane/32) + r]
    const int r_in = wave_m * Cfg::TM + (lane & 31), c_in = wave_n * Cfg::TN + 4 * (lane >> 5);
    if (pc.slot < 0) {
#pragma unroll
      for (int i = 0; i < FM; ++i) {
        const int row = m0 + r_in + i * 32;
        if (row >= a.D) continue;
        float* prow = a.out + (size_t)row * a.P;
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int col = n0 + c_in + j * 32 + 8 * q;
            if (col < a.P) *(float4*)(prow + col) = make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
          }
      }
    } else {
      float* pt = a.partial + ((size_t)pc.slot * STREAMK_WG_PER_XCD + w) * (BM * BN);
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q)
            *(float4*)(pt + (size_t)(r_in + i * 32) * BN + c_in + j * 32 + 8 * q) =
                make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
    }
  });
}

// out tile = sum of its pieces, in the order of the reduction index.  grid = (cut blocks * 32), 256 threads.
__global__ __launch_bounds__(256) void streamk_fixup_kernel(const StreamKArgs a, const StreamKCuts cuts) {
  constexpr int BM = 256, BN = 256;
  const int c = blockIdx.x / STREAMK_WG_PER_XCD, w = blockIdx.x % STREAMK_WG_PER_XCD;
  const int tiles = a.tiles_m * a.tiles_n;
  const int tile = cuts.block[c] * STREAMK_WG_PER_XCD + w;
  if (tile >= tiles) return;
  int tm, tn;
  tile_coords<8>(tile, a.tiles_m, a.tiles_n, &tm, &tn);
  const int m0 = tm * BM, n0 = tn * BN;
  const int n = cuts.count[c];
  for (int e = threadIdx.x; e < BM * BN / 4; e += 256) {
    const int r = e / (BN / 4), cc = (e % (BN / 4)) * 4;
    const int row = m0 + r, col = n0 + cc;
    if (row >= a.D || col >= a.P) continue;   // P is a multiple of 8 on this path: a group of 4 is all in or all out
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int p = 0; p < n; ++p) {
      const float4 v = *(const float4*)(a.partial + ((size_t)cuts.slot[c][p] * STREAMK_WG_PER_XCD + w) * (BM * BN) + (size_t)r * BN + cc);
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    *(float4*)(a.out + (size_t)row * a.P + col) = s;
  }
}

}  // namespace flashdp
