// The per-sample contraction of Algorithm 1 with the operand tiles going from HBM to LDS directly
// (buffer_load ... lds), never through registers: same tile shape, fragment reads, matrix-core
// instructions and epilogue as gemm_mfma_kernel, a different main-loop pipeline.
//
// Direct loads.  One buffer_load_dwordx4 ... lds of a wave writes 1 KB of LDS: lane L's 16 bytes land at
// M0 + 16 L, wherever in memory the lane's own offset points (measured on gfx950; lanes whose offset is
// outside the buffer write zeros).  A 32 (t) x 256 operand tile is 32 rows of 512 bytes, so one instruction
// fills two whole rows and each of the 8 waves issues two per operand per k-tile.  LDS rows cannot be padded
// (the 1 KB is contiguous), so bank conflicts of the transposed fragment reads - which touch rows t..t+3 at
// the same 64-byte column window - are avoided by a swizzle instead: the 16-byte chunk c of row t is kept at
// chunk position c ^ ((t & 3) << 2).  The swizzle costs nothing on the way in (the lane that fills position p
// simply fetches chunk p ^ ((t & 3) << 2) from memory) and one XOR in the fragment address.
//
// Pipeline.  STAGES LDS stages; the loads of k-tile k + STAGES - 1 are issued at the top of k-tile k, into
// the stage k-tile k - 1 was read from (free since the barrier that ended it).  The compiler does not model
// these loads (inline assembly), so the waits are written by hand: memory loads complete in order, hence
// "at most 4 (STAGES - 2) outstanding" = the loads of k-tile k + 1 have landed; then the one barrier per
// k-tile makes them visible to every wave.  Loads past the last k-tile are issued all the same: they point at
// rows >= T, fetch nothing, write zeros into a dead stage and keep the outstanding-load count uniform.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_mfma.hip.h"
#include "lds_plan.h"

namespace flashdp {

template <int STAGES_>
struct DmaCfg {
  static constexpr int BM = 256, BN = 256, BK = 32, WAVES_M = 2, WAVES_N = 4, STAGES = STAGES_;
  static constexpr int WAVES_PER_EU = 2;
  static constexpr int NT = 64 * WAVES_M * WAVES_N;
  static constexpr int TM = BM / WAVES_M, TN = BN / WAVES_N, FM = TM / 32, FN = TN / 32;
  static constexpr int A_ELEMS = BK * BM, B_ELEMS = BK * BN, STAGE_ELEMS = A_ELEMS + B_ELEMS;
  static_assert(A_ELEMS == lds_plan::OPERAND_ELEMS && B_ELEMS == lds_plan::OPERAND_ELEMS && STAGE_ELEMS == lds_plan::STAGE_ELEMS &&
                BM == lds_plan::ROW && BK == lds_plan::TILE_ROWS, "the index arithmetic in lds_plan.h is written for this tile");
  static constexpr int OPERAND_BYTES = STAGES * STAGE_ELEMS * 2;
  static constexpr int EPILOGUE_BYTES = BM * (BN + 8) * 2 + 64;
  static constexpr int LDS_BYTES = OPERAND_BYTES > EPILOGUE_BYTES ? OPERAND_BYTES : EPILOGUE_BYTES;
  static_assert(BM == 256 && BN == 256 && NT == 512 && BK == 32, "the load plan below is written for 8 waves, 512-byte rows, 32 rows");
  static_assert(STAGES >= 3 && STAGES <= 4, "stages");
};

// 128-bit buffer descriptor in scalar registers: base, stride 0, num_records = bytes, raw 32-bit format
__device__ __forceinline__ u32x4_t make_rsrc_words(const void* base, uint32_t bytes) {
  const uint64_t p = (uint64_t)base;
  u32x4_t r = {(uint32_t)p, (uint32_t)(p >> 32) & 0xFFFFu, bytes, 0x00020000u};
  return r;
}

// M0 (the LDS destination of a direct load) is written inside the statement and named as clobbered; the
// compiler flags any mention of that register, which is exactly what is meant here.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
// One wave-wide 1 KB direct load: lane L's 16 bytes at buffer offset voff go to LDS byte address lds_base + 16 L.
__device__ __forceinline__ void load_to_lds(const u32x4_t rsrc, uint32_t voff, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
               :: "s"(lds_base), "v"(voff), "s"(rsrc) : "memory", "m0");
}
#pragma clang diagnostic pop

template <int N>
__device__ __forceinline__ void wait_loads_outstanding() {
  static_assert(N == 0 || N == 4 || N == 8 || N == 24, "count");
  if constexpr (N == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  if constexpr (N == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
  if constexpr (N == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
  if constexpr (N == 24) asm volatile("s_waitcnt vmcnt(24)" ::: "memory");
}

// TRACE (measurement aid, off in every instantiation the library computes with): the workgroup also records where
// its time goes - constant-rate timestamps (100 MHz) at its start, when its first k-tile has landed, at the end of
// the main loop, when the epilogue has issued its stores and when they are acknowledged; the shader-clock cycles the
// main loop took (so that the clock the part actually ran at can be read off); and which XCD / CU it ran on.
template <typename Cfg, int MODE, int DT, bool TRACE = false>
__global__ __launch_bounds__(Cfg::NT, Cfg::WAVES_PER_EU) void gemm_mfma_dma_kernel(const GemmArgs a) {
  constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, FM = Cfg::FM, FN = Cfg::FN, STAGES = Cfg::STAGES;
  constexpr int ROW = 256;   // elements per LDS row of either operand (BM == BN == 256)
  extern __shared__ __attribute__((aligned(16))) unsigned short lds[];
  unsigned long long t_start = 0, t_first = 0, t_loop = 0, t_issued = 0, c_first = 0, c_loop = 0;
  if constexpr (TRACE) t_start = __builtin_amdgcn_s_memrealtime();

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wave_m = wave % Cfg::WAVES_M, wave_n = wave / Cfg::WAVES_M;

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
  const int m0 = tm * BM, n0 = tn * BN;

  // ---- direct-load plan: this wave fills rows 2 wave, 2 wave + 1 (first instruction) and 16 more (second)
  const int d_row = lds_plan::load_row(wave, lane);
  const int d_chunk = lds_plan::load_chunk(wave, lane);   // the chunk of the row this lane fetches (swizzle)
  const bool a_ok = m0 + d_chunk * 8 < a.D;
  const bool b_ok = n0 + d_chunk * 8 < a.P;
  // byte offsets inside one sample; an out-of-range column is sent to 2 GiB, beyond num_records, and reads 0
  const uint32_t a_off0 = a_ok ? (uint32_t)(d_row * a.D + m0 + d_chunk * 8) * 2u : 0x80000000u;
  const uint32_t b_off0 = b_ok ? (uint32_t)(d_row * a.P + n0 + d_chunk * 8) * 2u : 0x80000000u;
  const uint32_t a_half = (uint32_t)(16 * a.D) * 2u, b_half = (uint32_t)(16 * a.P) * 2u;
  const uint32_t a_kstep = (uint32_t)(BK * a.D) * 2u, b_kstep = (uint32_t)(BK * a.P) * 2u;
  const uint32_t a_bytes = (uint32_t)a.T * (uint32_t)a.D * 2u, b_bytes = (uint32_t)a.T * (uint32_t)a.P * 2u;
  const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned short*)lds;

  const int kt_per_sample = (a.T + BK - 1) / BK;
  const int nk = kt_per_sample * n_samples;

  // Fetch cursor, as in gemm_mfma_kernel: past the last tile it parks on rows >= T of the last sample.
  int ld_s = 0, ld_kt = 0;
  auto issue_loads = [&](int stage) {
    const char* pa = (const char*)a.dY + (size_t)(sample0 + ld_s) * a_bytes;
    const char* pb = (const char*)a.X + (size_t)(sample0 + ld_s) * b_bytes;
    const u32x4_t rsa = make_rsrc_words(pa, a_bytes), rsb = make_rsrc_words(pb, b_bytes);
    const uint32_t ao = a_off0 + (uint32_t)ld_kt * a_kstep, bo = b_off0 + (uint32_t)ld_kt * b_kstep;
    load_to_lds(rsa, ao, lds_base + lds_plan::load_dst_bytes(stage, 0, wave, 0));
    load_to_lds(rsa, ao + a_half, lds_base + lds_plan::load_dst_bytes(stage, 0, wave, 1));
    load_to_lds(rsb, bo, lds_base + lds_plan::load_dst_bytes(stage, 1, wave, 0));
    load_to_lds(rsb, bo + b_half, lds_base + lds_plan::load_dst_bytes(stage, 1, wave, 1));
    ld_kt += 1;
    const bool wrap = ld_kt >= kt_per_sample && ld_s + 1 < n_samples;
    ld_s = wrap ? ld_s + 1 : ld_s;
    ld_kt = wrap ? 0 : ld_kt;
  };

  // ---- fragment read plan: as in gemm_mfma_kernel, with the 32-column block index XORed by (row & 3)
  int a_rd[FM], b_rd[FN];
#pragma unroll
  for (int i = 0; i < FM; ++i) a_rd[i] = lds_plan::frag_offset(lane, wave_m * FM + i);
#pragma unroll
  for (int j = 0; j < FN; ++j) b_rd[j] = Cfg::A_ELEMS + lds_plan::frag_offset(lane, wave_n * FN + j);

  f32x16_t acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  constexpr int KS = BK / 16;
  static_assert(KS == 2, "two k-steps per tile");
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
  wait_loads_outstanding<4 * (STAGES - 2)>();   // k-tile 0 has landed
  __syncthreads();
  if constexpr (TRACE) { t_first = __builtin_amdgcn_s_memrealtime(); c_first = __builtin_amdgcn_s_memtime(); }
  load_frags(0, 0, fa[0], fb[0]);

  constexpr int N_MMA = FM * FN, N_RD = 2 * (FM + FN);
  // One k-tile, computed from LDS stage `cur` (compile-time).
  auto k_tile = [&](int k, auto cur_c) {
    constexpr int cur = decltype(cur_c)::value;
    constexpr int nxt = (cur + 1) % STAGES, refill = (cur + STAGES - 1) % STAGES;
    // k-step 0: fragments of k-step 1; refill the stage the previous k-tile was read from
    load_frags(cur, 1, fa[1], fb[1]);
    issue_loads(refill);
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j) acc[i][j] = mfma32<DT>(fb[0][j], fa[0][i], acc[i][j]);
    sched_interleave<0, N_MMA, N_RD, 0, 0>();
    // k-step 1: k-tile k+1 is in LDS once every wave's loads of it have landed
    wait_loads_outstanding<4 * (STAGES - 2)>();
    __syncthreads();
    load_frags(nxt, 0, fa[0], fb[0]);
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j) acc[i][j] = mfma32<DT>(fb[1][j], fa[1][i], acc[i][j]);
    sched_interleave<0, N_MMA, N_RD, 0, 0>();
    if constexpr (MODE == MODE_ACCUM) {
      // sample boundary: rescale so that acc always holds sum_{j<=i} (c_j / c_i) G_j (see gemm_mfma_kernel)
      if (a.factors != nullptr && k < nk && (k + 1) % kt_per_sample == 0) {
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
  };
  // STAGES k-tiles per trip so that every LDS stage index is a compile-time constant; a tile count that is
  // not a multiple runs up to STAGES - 1 extra k-tiles on the zeros the parked loads deliver.
  for (int k = 0; k < nk; k += STAGES) {
    static_for<STAGES>([&](auto s_c) { k_tile(k + decltype(s_c)::value, s_c); });
  }
  wait_loads_outstanding<0>();   // parked loads still write (zeros) into LDS: let them finish before LDS is reused
  __syncthreads();
  if constexpr (TRACE) { t_loop = __builtin_amdgcn_s_memrealtime(); c_loop = __builtin_amdgcn_s_memtime(); }

  tile_epilogue<Cfg, MODE, DT>(a, acc, lds, m0, n0, sample0, tile, tiles);
  if constexpr (TRACE) {
    t_issued = __builtin_amdgcn_s_memrealtime();
    wait_loads_outstanding<0>();
    const unsigned long long t_end = __builtin_amdgcn_s_memrealtime();
    if (tid == 0) {
      uint32_t hw_id, xcc_id;
      asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw_id));
      asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc_id));
      unsigned long long* p = a.trace + (size_t)blockIdx.x * 8;
      p[0] = t_start; p[1] = t_first; p[2] = t_loop; p[3] = t_issued; p[4] = t_end;
      p[5] = ((unsigned long long)(xcc_id & 0xFu) << 32) | hw_id;
      p[6] = c_loop - c_first;
      p[7] = 1;   // entry written (workgroups beyond the last work item write nothing)
    }
  }
}

}  // namespace flashdp
