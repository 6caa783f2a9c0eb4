// Non-private weight gradient out = sum_i dY_i^T X_i (Appendix B.1, Eq. "batched-grad") with the work balanced
// over the chip whatever the tile count: the comparator the DP path is held against, so that its ratio is not
// flattered by a plain GEMM whose last round of workgroups runs half empty (400 tiles of 256x256 on 256 CUs).
//
// Same tile, ring of direct-to-LDS loads, fragment reads and matrix-core loop as gemm_mfma_dma16_kernel in its
// batch-accumulating mode (the loop itself is shared: contract16); what differs is who computes what.  The output is cut into blocks of 32 tiles (8 tile
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

#include "gemm_mfma_dma16.hip.h"
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
__global__ __launch_bounds__(Cfg::NT, Cfg::WAVES_PER_EU) __attribute__((amdgpu_num_vgpr(DMA16_VGPR_ATTR))) void gemm_mfma_streamk_kernel(const StreamKArgs a) {
  constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK;
  extern __shared__ __attribute__((aligned(16))) unsigned short lds[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wave_m = wave % Cfg::WAVES_M, wave_n = wave / Cfg::WAVES_M;
  const int xcd = blockIdx.x & 7, w = blockIdx.x >> 3;
  const int tiles = a.tiles_m * a.tiles_n;

  const int d_row = lds_plan16::load_row(wave, lane);
  const int d_chunk = lds_plan16::load_chunk(wave, lane);
  const uint32_t a_half = (uint32_t)(16 * a.D) * 2u, b_half = (uint32_t)(16 * a.P) * 2u;
  const uint32_t a_kstep = (uint32_t)(BK * a.D) * 2u, b_kstep = (uint32_t)(BK * a.P) * 2u;
  const uint32_t a_bytes = (uint32_t)a.T * (uint32_t)a.D * 2u, b_bytes = (uint32_t)a.T * (uint32_t)a.P * 2u;
  const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned short*)lds;
  const int kt_per_sample = (a.T + BK - 1) / BK;

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
      load_to_lds(rsa, ao, lds_base + lds_plan16::load_dst_bytes(stage, 0, wave, 0));
      load_to_lds(rsa, ao + a_half, lds_base + lds_plan16::load_dst_bytes(stage, 0, wave, 1));
      load_to_lds(rsb, bo, lds_base + lds_plan16::load_dst_bytes(stage, 1, wave, 0));
      load_to_lds(rsb, bo + b_half, lds_base + lds_plan16::load_dst_bytes(stage, 1, wave, 1));
      ld_kt += 1;
      const bool wrap = ld_kt >= kt_per_sample && ld_s + 1 < a.B;
      ld_s = wrap ? ld_s + 1 : ld_s;
      ld_kt = wrap ? 0 : ld_kt;
    };

    // k1 - k0 is a multiple of the ring depth (range boundaries and nk_pad are); the k-tiles between the true end
    // of the reduction and nk_pad read the zeros the parked loads deliver.  The main loop returns with every load
    // landed and the workgroup past a barrier: the next piece may refill the ring at once.
    f32x4_t acc[8][4];
    contract16<Cfg, DT>(acc, lds_base, lane, wave_m, wave_n, pc.k1 - pc.k0, issue_loads, [](int) {}, []() {});

    // acc[i][j][r] = G[m0 + wave_m*128 + 16 i + lane%16][n0 + wave_n*64 + 16 j + 4 (lane/16) + r]
    const int r_in = wave_m * 128 + (lane & 15), c_in = wave_n * 64 + 4 * (lane >> 4);
    if (pc.slot < 0) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int row = m0 + r_in + i * 16;
        if (row >= a.D) continue;
        float* prow = a.out + (size_t)row * a.P;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int col = n0 + c_in + j * 16;
          if (col < a.P) *(float4*)(prow + col) = make_float4(acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]);
        }
      }
    } else {
      float* pt = a.partial + ((size_t)pc.slot * STREAMK_WG_PER_XCD + w) * (BM * BN);
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          *(float4*)(pt + (size_t)(r_in + i * 16) * BN + c_in + j * 16) = make_float4(acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]);
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
