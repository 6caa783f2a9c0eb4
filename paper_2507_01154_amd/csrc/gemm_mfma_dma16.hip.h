// The per-sample contraction of Algorithm 1, direct-to-LDS pipeline of gemm_mfma_dma_kernel, built on
// v_mfma_f32_16x16x32 instead of v_mfma_f32_32x32x16.
//
// Why.  On N(0,1) operands this part is held at its power limit, and what the matrix cores sustain there depends on
// the instruction: on register-resident random operands the 32x32x16 form runs at 0.72-0.77 of the nominal peak, the
// 16x16x32 form at 0.81-0.89 (0.66-0.70 against 0.81 with the kernel's LDS fragment reads; flashdp_mfma_probe
// patterns 1/7 and 3/8) - half as many accumulator updates per multiply-add.  Same FLOPs, same tile (256 x 256,
// 8 waves of 128 x 64, 32-deep k-tiles in a ring of 4 LDS stages), same direct loads, same one barrier per k-tile.
//
// What differs.  The instruction consumes a whole 32-deep k-tile, and a lane holds operand[r = lane % 16]
// [k = 8 (lane / 16) + 0..7], so the fragment reads and the LDS swizzle are those of lds_plan16.h.  A wave's 128 x 64
// is 8 x 4 blocks of 16 x 16 (32 accumulators of 4 registers).  Holding all 12 operand fragments of a k-tile twice over
// (to read the next tile's while this one's are multiplied) would take 96 registers; instead a k-tile is walked in
// four quadrants (4 dY fragments x 2 X fragments, 8 instructions each) in an order that lets every half-set of
// fragments be overwritten as soon as its last quadrant has been issued: lo x lo, lo x hi, hi x hi, hi x lo on even
// k-tiles and lo x hi, lo x lo, hi x lo, hi x hi on odd ones, 48 fragment registers in all, each read issued one
// quadrant ahead of its use.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_mfma_dma.hip.h"
#include "lds_plan16.h"

namespace flashdp {

typedef float f32x4_t __attribute__((ext_vector_type(4)));

// Register cap of the kernel: 232 (the attribute counts in units of two on this target).  Two of its waves per SIMD
// then leave 48 of the 512 registers for one wave of the streaming aggregation of the overlapped schedule.
#define DMA16_VGPR_ATTR 116

// The main loop is written instruction by instruction (inline assembly, every statement volatile, so the order below
// is the order issued).  Left to the compiler, the 32 four-register accumulators wandered through the register file
// from k-tile to k-tile (the instruction's destination need not be its addend) and the kernel needed 250 registers,
// too many to leave room for a wave of the streaming aggregation beside two of its own.  Here every accumulator is
// updated in place, which also means that the compiler neither sees the LDS reads (the waits for them are written
// by hand, like those for the direct loads: LDS reads complete in order) nor inserts the wait states the matrix-core
// pipeline asks for between an instruction and a vector-ALU access to its result (idle instructions are placed by
// hand where the accumulators are zeroed, rescaled and handed to the epilogue; inside the loop an accumulator is
// touched once per 32 instructions).
template <int DT>
__device__ __forceinline__ void mfma16_inplace(f32x4_t& c, const s16x8_t& a, const s16x8_t& b) {
  if constexpr (DT == DT_BF16) {
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(c) : "v"(a), "v"(b));
  } else {
    asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+v"(c) : "v"(a), "v"(b));
  }
}

// one transposed 64-bit LDS read at byte address `addr` + OFF (OFF < 65536: the instruction's offset field)
template <int OFF>
__device__ __forceinline__ s16x4_t lds_read_tr_at(uint32_t addr) {
  static_assert(OFF >= 0 && OFF < 65536, "offset field");
  s16x4_t d;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(d) : "v"(addr), "n"(OFF) : "memory");
  return d;
}

template <int N>
__device__ __forceinline__ void wait_lds_reads_outstanding() {
  static_assert(N >= 0 && N <= 15, "count");
  asm volatile("s_waitcnt lgkmcnt(%0)" :: "n"(N) : "memory");
}

__device__ __forceinline__ void matrix_core_results_settle() {   // 32 idle issue cycles
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
}

// What a workgroup does with its finished tile (the 16 x 16 block layout of tile_epilogue).  acc[i][j][r] =
// G[m0 + wave_m*128 + 16 i + lane%16][n0 + wave_n*64 + 16 j + 4 (lane/16) + r].  The caller has ended its main loop
// with a barrier: the operand tiles in LDS are dead and LDS is reused for the reduction and the staging.
template <typename Cfg, int MODE, int DT>
__device__ __forceinline__ void tile_epilogue16(const GemmArgs& a, f32x4_t (&acc)[8][4], unsigned short* lds,
                                                int m0, int n0, int sample0, int tile, int tiles) {
  constexpr int BM = Cfg::BM, BN = Cfg::BN, NT = Cfg::NT;
  static_assert(BM == 256 && BN == 256 && Cfg::WAVES_M == 2 && Cfg::WAVES_N == 4, "8 waves of 128 x 64");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave % Cfg::WAVES_M, wave_n = wave / Cfg::WAVES_M;
  const int row_l = wave_m * 128 + (lane & 15);            // + 16 i
  const int col_l = wave_n * 64 + 4 * (lane >> 4);         // + 16 j
  if constexpr (MODE == MODE_NORM || MODE == MODE_SPILL) {
    constexpr int EP = BN + 8;                               // staging pitch in elements: 16-byte aligned rows
    static_assert(BM * EP * 2 + 64 <= Cfg::LDS_BYTES, "epilogue staging must fit in the operand buffers");
    float* red = (float*)(lds + BM * EP);
    float ss = 0.0f;
    if constexpr (MODE == MODE_SPILL) {
      // the norm is taken of the tile as parked (after the rounding to bfloat16), see tile_epilogue
      unsigned short* st = lds + row_l * EP + col_l;
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          uint2 v;
          v.x = pack2_16bit<DT_BF16>(acc[i][j][0], acc[i][j][1]);
          v.y = pack2_16bit<DT_BF16>(acc[i][j][2], acc[i][j][3]);
          const float r0 = __builtin_bit_cast(float, v.x << 16), r1 = __builtin_bit_cast(float, v.x & 0xFFFF0000u);
          const float r2 = __builtin_bit_cast(float, v.y << 16), r3 = __builtin_bit_cast(float, v.y & 0xFFFF0000u);
          ss = fmaf(r0, r0, ss); ss = fmaf(r1, r1, ss); ss = fmaf(r2, r2, ss); ss = fmaf(r3, r3, ss);
          *(uint2*)(st + (i * 16) * EP + j * 16) = v;
        }
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int e = 0; e < 4; ++e) ss = fmaf(acc[i][j][e], acc[i][j][e], ss);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
    if (lane == 0) red[wave] = ss;
    __syncthreads();
    if (tid == 0) {
      float tot = 0.0f;
      for (int w = 0; w < NT / 64; ++w) tot += red[w];
      a.partials[(size_t)sample0 * tiles + tile] = tot;
    }
    if constexpr (MODE == MODE_SPILL) {
      unsigned short* sc = (unsigned short*)a.scratch + (size_t)sample0 * a.D * a.P;
      constexpr int CPR = BN / 8;
#pragma unroll
      for (int it = 0; it < BM * CPR / NT; ++it) {
        const int c = tid + it * NT;
        const int r = c / CPR, cc = c % CPR;
        const int row = m0 + r, col = n0 + cc * 8;
        if (row < a.D && col < a.P)   // P is a multiple of 8 on this path: a chunk is all in or all out
          __builtin_nontemporal_store(*(const u32x4_t*)(lds + r * EP + cc * 8), (u32x4_t*)(sc + (size_t)row * a.P + col));
      }
    }
  } else {
    float* obase = a.out;
    if constexpr (MODE == MODE_MATERIALIZE) obase = (float*)a.scratch + (size_t)sample0 * a.D * a.P;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int row = m0 + row_l + i * 16;
      if (row >= a.D) continue;
      float* prow = obase + (size_t)row * a.P;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int col = n0 + col_l + j * 16;
        if (col < a.P) {   // P is a multiple of 8 and col of 4: the four columns are all in or all out
          float4 v = make_float4(acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]);
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

// The main loop: contracts nk k-tiles (rounded up to a multiple of the ring depth; the surplus runs on the zeros that
// loads past the end deliver) into acc.  issue_loads(stage) enqueues the four direct loads of the next k-tile of the
// caller's stream of k-tiles into LDS stage `stage` (it is called STAGES - 1 times up front, then once per k-tile);
// after_tile(k) runs behind k-tile k (the batch-accumulating mode rescales there).  On return every load and LDS
// read has completed, the matrix-core results have settled and the workgroup has passed a barrier: LDS is free.
// first_tile_landed() is called once, when k-tile 0 is in LDS (a hook for the traced instantiation).
template <typename Cfg, int DT, typename IssueLoads, typename AfterTile, typename FirstLanded>
__device__ __forceinline__ void contract16(f32x4_t (&acc)[8][4], uint32_t lds_base, int lane, int wave_m, int wave_n, int nk,
                                           IssueLoads&& issue_loads, AfterTile&& after_tile, FirstLanded&& first_tile_landed) {
  constexpr int STAGES = Cfg::STAGES, ROW = 256;
  static_assert(Cfg::BK == 32 && STAGES == 4 && STAGES == lds_plan16::STAGES && Cfg::BM == 256 && Cfg::BN == 256,
                "one 16x16x32 k-step per k-tile; k-tiles are walked in pairs");
  // ---- fragment read plan: LDS byte addresses (stage 0) of the 8 dY blocks (rows of the wave's 128) and the 4 X
  // blocks (its 64 columns) of 16; a stage adds 16 KB and the second read of a fragment 4 tile rows, both through the
  // offset field
  uint32_t a_rd[8], b_rd[4];
#pragma unroll
  for (int i = 0; i < 8; ++i) a_rd[i] = lds_base + 2u * (uint32_t)lds_plan16::frag_offset(lane, wave_m * 8 + i);
#pragma unroll
  for (int j = 0; j < 4; ++j) b_rd[j] = lds_base + 2u * (uint32_t)(lds_plan16::tile_base(0, 1) + lds_plan16::frag_offset(lane, wave_n * 4 + j));
  constexpr int STAGE_BYTES = lds_plan16::OPERAND_ELEMS * 2, SECOND = 4 * ROW * 2;

#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};

  // Operand fragments.  dY: the lower and upper four block rows.  X: the half that a k-tile uses in its first and last
  // quadrant ("outer": columns 0-1 of even k-tiles in Bx, columns 2-3 of odd ones in Bz) and the half it uses in its
  // two middle quadrants ("inner": By, columns 2-3 of even k-tiles, 0-1 of odd ones).  56 registers.
  s16x8_t Alo[4], Ahi[4], Bx[2], By[2], Bz[2];
  // fragment f (0..3) of the lower (half = 0) or upper half of the wave's dY blocks, resp. fragment f (0..1) of a half
  // of its X blocks, from LDS stage `stage`: two reads each
  auto read_a = [&](auto stage_c, auto half_c, auto f_c, s16x8_t* dst) {
    constexpr int stage = decltype(stage_c)::value, half = decltype(half_c)::value, f = decltype(f_c)::value;
    const s16x4_t lo = lds_read_tr_at<stage * STAGE_BYTES>(a_rd[4 * half + f]);
    const s16x4_t hi = lds_read_tr_at<stage * STAGE_BYTES + SECOND>(a_rd[4 * half + f]);
    dst[f] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  };
  auto read_b = [&](auto stage_c, auto half_c, auto f_c, s16x8_t* dst) {
    constexpr int stage = decltype(stage_c)::value, half = decltype(half_c)::value, f = decltype(f_c)::value;
    const s16x4_t lo = lds_read_tr_at<stage * STAGE_BYTES>(b_rd[2 * half + f]);
    const s16x4_t hi = lds_read_tr_at<stage * STAGE_BYTES + SECOND>(b_rd[2 * half + f]);
    dst[f] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  };
  // One quadrant: 4 dY fragments (block rows i0..i0+3) x 2 X fragments (block columns j0, j0+1); `after(m)` runs
  // behind instruction m (0..7) and issues reads for later quadrants.  Every fragment is read two quadrants before
  // its first use (one and a half for the outer X half), so a quadrant waits once, at its start, until at most
  // ALLOWED reads are outstanding: the reads issued during the previous quadrant (LDS reads complete in order).
  auto quadrant = [&](auto allowed_c, const s16x8_t* A, int i0, const s16x8_t* B, int j0, auto&& after) {
    constexpr int ALLOWED = decltype(allowed_c)::value;
    if constexpr (ALLOWED >= 0) wait_lds_reads_outstanding<ALLOWED>();
    static_for<8>([&](auto m_c) {
      constexpr int m = decltype(m_c)::value, i = m / 2, j = m % 2;
      mfma16_inplace<DT>(acc[i0 + i][j0 + j], B[j], A[i]);
      after(m_c);
    });
  };
  using c0 = std::integral_constant<int, 0>;
  using c1 = std::integral_constant<int, 1>;
  using c4 = std::integral_constant<int, 4>;
  using c8 = std::integral_constant<int, 8>;
  using cnone = std::integral_constant<int, -1>;

#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s) issue_loads(s);
  wait_loads_outstanding<4 * (STAGES - 2)>();   // k-tile 0 has landed
  __builtin_amdgcn_s_barrier();
  first_tile_landed();
  // the reads an odd k-tile would have issued for k-tile 0 in its third (outer X, dY lo) and fourth (inner X) quadrant
  static_for<2>([&](auto f_c) { read_b(c0{}, c0{}, f_c, Bx); });
  static_for<4>([&](auto f_c) { read_a(c0{}, c0{}, f_c, Alo); });
  static_for<2>([&](auto f_c) { read_b(c0{}, c1{}, f_c, By); });
  asm volatile("s_nop 7" ::: "memory");   // the zeroed accumulators are vector-ALU results

  // One k-tile from LDS stage `cur`.  PARITY 0 (even): outer X half = columns 0-1 (OUT = Bx), the next tile's goes to
  // Bz; PARITY 1 (odd): outer = columns 2-3 (OUT = Bz), the next tile's goes to Bx.  Quadrants: lo x outer,
  // lo x inner, hi x inner, hi x outer.  Reads issued: the tile's own dY hi in the first quadrant (used in the third);
  // after the barrier in the third, the next tile's outer X half and dY lo (used in its first); in the fourth, the
  // next tile's inner X half (used in its second).  The ring is refilled in the first quadrant: the stage k-tile
  // k - 1 was read from is free since the barrier inside that tile (every read of it was issued before).
  auto k_tile = [&](int k, auto cur_c, auto parity_c) {
    constexpr int cur = decltype(cur_c)::value, PARITY = decltype(parity_c)::value;
    constexpr int nxt = (cur + 1) % STAGES, refill = (cur + STAGES - 1) % STAGES;
    using ccur = std::integral_constant<int, cur>;
    using cnxt = std::integral_constant<int, nxt>;
    using couter = std::integral_constant<int, PARITY>;          // which X half is the outer one of this tile
    using cinner = std::integral_constant<int, 1 - PARITY>;
    s16x8_t* const OUT = PARITY == 0 ? Bx : Bz;
    s16x8_t* const NEXT_OUT = PARITY == 0 ? Bz : Bx;
    constexpr int j_out = 2 * PARITY, j_in = 2 - 2 * PARITY;
    quadrant(c4{}, Alo, 0, OUT, j_out, [&](auto m_c) {          // behind it: the 4 reads of the previous quadrant
      if constexpr (decltype(m_c)::value < 4) read_a(ccur{}, c1{}, m_c, Ahi);
      if constexpr (decltype(m_c)::value == 5) issue_loads(refill);
    });
    quadrant(c8{}, Alo, 0, By, j_in, [&](auto m_c) {});         // behind it: the 8 reads of the first quadrant
    wait_loads_outstanding<4 * (STAGES - 2)>();   // k-tile k+1 is in LDS once every wave's loads of it have landed
    quadrant(c0{}, Ahi, 4, By, j_in, [&](auto m_c) {            // nothing was read in the second quadrant
      constexpr int m = decltype(m_c)::value;
      if constexpr (m == 0) __builtin_amdgcn_s_barrier();
      if constexpr (m < 2) read_b(cnxt{}, cinner{}, m_c, NEXT_OUT);   // the next tile's outer half is this tile's inner side
      if constexpr (m >= 2 && m < 6) read_a(cnxt{}, c0{}, std::integral_constant<int, m - 2>{}, Alo);
    });
    quadrant(cnone{}, Ahi, 4, OUT, j_out, [&](auto m_c) {
      if constexpr (decltype(m_c)::value < 2) read_b(cnxt{}, couter{}, m_c, By);   // and its inner half this tile's outer side
    });
    after_tile(k);
  };
  // STAGES k-tiles per trip so that every LDS stage index is a compile-time constant
  for (int k = 0; k < nk; k += STAGES) {
    k_tile(k, std::integral_constant<int, 0>{}, c0{});
    k_tile(k + 1, std::integral_constant<int, 1>{}, c1{});
    k_tile(k + 2, std::integral_constant<int, 2>{}, c0{});
    k_tile(k + 3, std::integral_constant<int, 3>{}, c1{});
  }
  wait_loads_outstanding<0>();       // parked loads still write (zeros) into LDS: let them finish before LDS is reused
  wait_lds_reads_outstanding<0>();   // and so do the reads issued for a k-tile that does not exist
  matrix_core_results_settle();
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

template <typename Cfg, int MODE, int DT, bool TRACE = false>
__global__ __launch_bounds__(Cfg::NT, Cfg::WAVES_PER_EU) __attribute__((amdgpu_num_vgpr(DMA16_VGPR_ATTR))) void gemm_mfma_dma16_kernel(const GemmArgs a) {
  constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK;
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

  // ---- direct-load plan (as gemm_mfma_dma_kernel, with this kernel's swizzle and ring layout)
  const int d_row = lds_plan16::load_row(wave, lane);
  const int d_chunk = lds_plan16::load_chunk(wave, lane);
  const bool a_ok = m0 + d_chunk * 8 < a.D;
  const bool b_ok = n0 + d_chunk * 8 < a.P;
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
    load_to_lds(rsa, ao, lds_base + lds_plan16::load_dst_bytes(stage, 0, wave, 0));
    load_to_lds(rsa, ao + a_half, lds_base + lds_plan16::load_dst_bytes(stage, 0, wave, 1));
    load_to_lds(rsb, bo, lds_base + lds_plan16::load_dst_bytes(stage, 1, wave, 0));
    load_to_lds(rsb, bo + b_half, lds_base + lds_plan16::load_dst_bytes(stage, 1, wave, 1));
    ld_kt += 1;
    const bool wrap = ld_kt >= kt_per_sample && ld_s + 1 < n_samples;
    ld_s = wrap ? ld_s + 1 : ld_s;
    ld_kt = wrap ? 0 : ld_kt;
  };

  f32x4_t acc[8][4];
  auto after_tile = [&](int k) {
    if constexpr (MODE == MODE_ACCUM) {
      // sample boundary: rescale so that acc always holds sum_{j<=i} (c_j / c_i) G_j (see gemm_mfma_kernel)
      if (a.factors != nullptr && k < nk && (k + 1) % kt_per_sample == 0) {
        const int s = k / kt_per_sample;
        const float ratio = (s + 1 < n_samples) ? a.factors[s] / a.factors[s + 1] : a.factors[s];
        matrix_core_results_settle();
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            acc[i][j] *= ratio;
            asm volatile("" : "+v"(acc[i][j]));   // the product is formed here, in front of the idle cycles below
          }
        matrix_core_results_settle();
      }
    }
  };
  contract16<Cfg, DT>(acc, lds_base, lane, wave_m, wave_n, nk, issue_loads, after_tile, [&]() {
    if constexpr (TRACE) { t_first = __builtin_amdgcn_s_memrealtime(); c_first = __builtin_amdgcn_s_memtime(); }
  });
  if constexpr (TRACE) { t_loop = __builtin_amdgcn_s_memrealtime(); c_loop = __builtin_amdgcn_s_memtime(); }

  tile_epilogue16<Cfg, MODE, DT>(a, acc, lds, m0, n0, sample0, tile, tiles);
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
