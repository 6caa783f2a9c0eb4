// The per-sample contraction of Algorithm 1 (direct-to-LDS pipeline of gemm_mfma_dma_kernel) for tiles other than
// 256 x 256: 384 x 192 and 192 x 384, eight waves of 96 x 96 (3 x 3 matrix-core blocks) each.
//
// Why.  Every work item (sample, tile) of a per-sample pass is equally long, so a pass takes
// ceil(items / compute units) rounds.  A layer of 3072 x 768 at B = 8 is 288 items of 256 x 256 - two rounds, the
// second for 32 stragglers - but exactly 256 items of 384 x 192: one round of items 9/8 as long.  The host picks the
// shape with the fewest tile-rounds; for large layers that is always 256 x 256 (less padding, and the measured
// kernel), these shapes are for layers with a few hundred work items.
//
// What differs from gemm_mfma_dma_kernel: rows of 768 or 384 bytes do not divide the 1 KB a direct load writes, so
// every lane has its own (row, chunk) per load instruction, and the k-tile's 24 + 12 loads are dealt round-robin to
// the 8 waves, five instructions each with four of the forty fetching nothing (see shaped_plan.h, which also has the
// bank swizzle for the two row pitches).  The main loop, the waits, the fragment reads and the epilogue are the same.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_mfma_dma.hip.h"
#include "shaped_plan.h"

namespace flashdp {

template <int BM_, int BN_, int WAVES_M_, int WAVES_N_, int STAGES_>
struct ShapedCfg {
  static constexpr int BM = BM_, BN = BN_, BK = 32, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_, STAGES = STAGES_;
  static constexpr int WAVES_PER_EU = 2;
  static constexpr int NT = 64 * WAVES_M * WAVES_N;
  static constexpr int TM = BM / WAVES_M, TN = BN / WAVES_N, FM = TM / 32, FN = TN / 32;
  static constexpr int A_ELEMS = BK * BM, B_ELEMS = BK * BN, STAGE_ELEMS = A_ELEMS + B_ELEMS;
  static constexpr int SLOTS = (BM / 16 + 7) / 8 + (BN / 16 + 7) / 8;
  static constexpr int LOAD_BYTES = STAGES * STAGE_ELEMS * 2 + 1024 * 8;   // ring + the spare 1 KB per wave
  static constexpr int EPILOGUE_BYTES = BM * (BN + 8) * 2 + 64;
  static constexpr int LDS_BYTES = LOAD_BYTES > EPILOGUE_BYTES ? LOAD_BYTES : EPILOGUE_BYTES;
  static_assert(NT == 512 && BK == shaped_plan::TILE_ROWS && WAVES_M * WAVES_N == shaped_plan::WAVES, "eight waves, 32-deep k-tiles");
  static_assert(BM % 64 == 0 && BN % 64 == 0 && TM % 32 == 0 && TN % 32 == 0, "tile shape");
  static_assert(STAGE_ELEMS == shaped_plan::stage_elems(BM, BN) && SLOTS == shaped_plan::slots(BM, BN) &&
                LOAD_BYTES == (int)shaped_plan::lds_bytes_for_loads(BM, BN, STAGES), "shaped_plan.h describes this tile");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS per workgroup");
  static_assert(STAGES >= 3 && STAGES <= 4 && SLOTS * (STAGES - 1) < 64, "stages");
};

template <int N>
__device__ __forceinline__ void wait_loads_outstanding_n() {
  static_assert(N >= 0 && N < 64, "count");
  asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

template <typename Cfg, int MODE, int DT>
__global__ __launch_bounds__(Cfg::NT, Cfg::WAVES_PER_EU) void gemm_mfma_dma_shaped_kernel(const GemmArgs a) {
  static_assert(MODE != MODE_ACCUM, "per-sample passes only");
  constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, FM = Cfg::FM, FN = Cfg::FN, STAGES = Cfg::STAGES, SLOTS = Cfg::SLOTS;
  extern __shared__ __attribute__((aligned(16))) unsigned short lds[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wave_m = wave % Cfg::WAVES_M, wave_n = wave / Cfg::WAVES_M;

  const int tiles = a.tiles_m * a.tiles_n;
  int sample0 = 0, tile;
  if (!shared_block_item(blockIdx.x, tiles, a.B, &sample0, &tile)) return;   // the whole workgroup, before any barrier
  int tm, tn;
  tile_coords<8>(tile, a.tiles_m, a.tiles_n, &tm, &tn);
  const int m0 = tm * BM, n0 = tn * BN;

  // ---- direct-load plan: per instruction slot, the lane's byte offset inside a sample at k-tile 0 (an out-of-range
  // column, and the slot that loads nothing, are sent to 2 GiB, beyond num_records, and read 0), the operand, the
  // step per k-tile and the LDS destination inside a stage.
  const uint32_t a_kstep = (uint32_t)(BK * a.D) * 2u, b_kstep = (uint32_t)(BK * a.P) * 2u;
  const uint32_t a_bytes = (uint32_t)a.T * (uint32_t)a.D * 2u, b_bytes = (uint32_t)a.T * (uint32_t)a.P * 2u;
  const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned short*)lds;
  uint32_t off0[SLOTS];     // per lane
  uint32_t dst0[SLOTS];     // per wave: LDS destination in stage 0, or the spare 1 KB of this wave
  uint32_t in_ring[SLOTS];  // per wave: all ones if the instruction loads something (its destination moves with the stage)
#pragma unroll
  for (int j = 0; j < SLOTS; ++j) {
    const int op = shaped_plan::slot_operand(BM, BN, j);
    const int n = shaped_plan::slot_index(BM, BN, wave, j);
    const int w = op == 0 ? BM : BN, ld = op == 0 ? a.D : a.P, c0 = op == 0 ? m0 : n0;
    const int row = shaped_plan::lane_row(w, n < 0 ? 0 : n, lane), chunk = shaped_plan::lane_chunk(w, n < 0 ? 0 : n, lane);
    const bool ok = n >= 0 && c0 + chunk * 8 < ld;
    off0[j] = ok ? (uint32_t)(row * ld + c0 + chunk * 8) * 2u : 0x80000000u;
    dst0[j] = __builtin_amdgcn_readfirstlane(lds_base + shaped_plan::slot_dst_bytes(BM, BN, STAGES, 0, wave, j));
    in_ring[j] = __builtin_amdgcn_readfirstlane(n >= 0 ? 0xFFFFFFFFu : 0u);
  }

  const int kt_per_sample = (a.T + BK - 1) / BK;
  const int nk = kt_per_sample;
  const char* const pa = (const char*)a.dY + (size_t)sample0 * a_bytes;
  const char* const pb = (const char*)a.X + (size_t)sample0 * b_bytes;
  const u32x4_t rsa = make_rsrc_words(pa, a_bytes), rsb = make_rsrc_words(pb, b_bytes);

  // Loads past the last k-tile point at rows >= T, fetch nothing and write zeros into a dead stage.
  int ld_kt = 0;
  auto issue_loads = [&](int stage) {
#pragma unroll
    for (int j = 0; j < SLOTS; ++j) {
      const bool is_a = shaped_plan::slot_operand(BM, BN, j) == 0;   // known at compile time
      const uint32_t dst = dst0[j] + ((uint32_t)(stage * Cfg::STAGE_ELEMS * 2) & in_ring[j]);
      load_to_lds(is_a ? rsa : rsb, off0[j] + (uint32_t)ld_kt * (is_a ? a_kstep : b_kstep), dst);
    }
    ld_kt += 1;
  };

  // ---- fragment read plan
  int a_rd[FM], b_rd[FN];
#pragma unroll
  for (int i = 0; i < FM; ++i) a_rd[i] = shaped_plan::frag_offset(lane, wave_m * FM + i, BM);
#pragma unroll
  for (int j = 0; j < FN; ++j) b_rd[j] = Cfg::A_ELEMS + shaped_plan::frag_offset(lane, wave_n * FN + j, BN);

  f32x16_t acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  static_assert(BK / 16 == 2, "two k-steps per tile");
  s16x8_t fa[2][FM], fb[2][FN];
  auto load_frags = [&](int stage, int ks, s16x8_t* pfa, s16x8_t* pfb) {
    const unsigned short* base = lds + stage * Cfg::STAGE_ELEMS;
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      const s16x4_t lo = lds_read_tr(base + a_rd[i] + ks * 16 * BM);
      const s16x4_t hi = lds_read_tr(base + a_rd[i] + ks * 16 * BM + 4 * BM);
      pfa[i] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
#pragma unroll
    for (int j = 0; j < FN; ++j) {
      const s16x4_t lo = lds_read_tr(base + b_rd[j] + ks * 16 * BN);
      const s16x4_t hi = lds_read_tr(base + b_rd[j] + ks * 16 * BN + 4 * BN);
      pfb[j] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
  };

  constexpr int LANDED = SLOTS * (STAGES - 2);   // loads complete in order: at most this many outstanding = the next k-tile is in
#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s) issue_loads(s);
  wait_loads_outstanding_n<LANDED>();
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
    wait_loads_outstanding_n<LANDED>();
    __syncthreads();
    load_frags(nxt, 0, fa[0], fb[0]);
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j) acc[i][j] = mfma32<DT>(fb[1][j], fa[1][i], acc[i][j]);
    sched_interleave<0, N_MMA, N_RD, 0, 0>();
  };
  for (int k = 0; k < nk; k += STAGES) {
    static_for<STAGES>([&](auto s_c) { k_tile(s_c); });
  }
  wait_loads_outstanding_n<0>();   // parked loads still write (zeros) into LDS: let them finish before LDS is reused
  __syncthreads();

  tile_epilogue<Cfg, MODE, DT>(a, acc, lds, m0, n0, sample0, tile, tiles);
}

}  // namespace flashdp
