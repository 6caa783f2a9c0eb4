// Per-sample weight-gradient contraction on the gfx950 matrix cores.
//
// Steps of Algorithm 1 covered here: load tiles of dY and X from HBM to on-chip memory, compute the
// per-sample gradient tile B_G = sum_T B_dY^T B_X, and the intra-block reduction of its squared norm
// (one scalar per workgroup).  Depending on MODE the tile is then dropped (norm pass), parked in the
// 16-bit scratch (single-compute schedule), or - with the clip factors already known - accumulated
// over the batch as sum_i c_i G_i (second pass; with c == 1 this is the non-private Eq. "batched-grad").
//
// Operand layout.  out[m][n] = sum_t dY[t][m] * X[t][n]: both operands have the reduction index t as the
// slow dimension and m (= d_out) resp. n (= d_in) contiguous.  Tiles are copied to LDS as they are
// (rows = t), 16 bytes per lane and coalesced along m / n.  The matrix-core operand wants, per lane,
// eight consecutive t for one m; the LDS transpose read ds_read_b64_tr_b16 delivers exactly that from
// the t-major tile: within 16 lanes, lane s supplies the address of 4 contiguous 16-bit values and lane
// i receives element (i % 4) of lanes (i / 4), (i / 4) + 4, (i / 4) + 8, (i / 4) + 12.  So lane s points
// at row (s / 4), column 4 * (s % 4) of a 4 (t) x 16 (m) block and lane i gets column i for 4 rows.
//
// v_mfma_f32_32x32x16 (bf16 or f16): lane l holds A[r = l % 32][k = 8 * (l / 32) + 0..7], likewise B with
// c = l % 32; accumulator register j of lane l is C[row = 8 * (j / 4) + 4 * (l / 32) + (j % 4)][col = l % 32].
// The X fragment is passed as the first (row) operand and the dY fragment as the second, i.e. the
// instruction forms the transposed block: lane l then owns output row m = l % 32 and, in registers
// 4q..4q+3, four CONSECUTIVE output columns n = 8q + 4 * (l / 32) + 0..3, which the epilogue packs into one
// 8-byte LDS write (the bfloat16 tile is staged in LDS and leaves the chip in whole 512-byte rows: partial
// cache lines from direct stores measured slower) or one 16-byte global store (fp32 output).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

namespace flashdp {

// Compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>).
template <typename F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// Issue-order hints for one phase of the main loop: after each matrix-core instruction, let its share of
// the phase's LDS reads / LDS writes / global loads issue (they run in the shadow of the 32-cycle MFMA).
template <int I, int N_MMA, int N_RD, int N_WR, int N_VM>
__device__ __forceinline__ void sched_interleave() {
  if constexpr (I < N_MMA) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    constexpr int rd = (N_RD + N_MMA - 1 - I) / N_MMA;
    constexpr int wr = (N_WR + N_MMA - 1 - I) / N_MMA;
    constexpr int vm = (N_VM + N_MMA - 1 - I) / N_MMA;
    if constexpr (rd > 0) __builtin_amdgcn_sched_group_barrier(0x100, rd, 0);
    if constexpr (wr > 0) __builtin_amdgcn_sched_group_barrier(0x200, wr, 0);
    if constexpr (vm > 0) __builtin_amdgcn_sched_group_barrier(0x020, vm, 0);
    sched_interleave<I + 1, N_MMA, N_RD, N_WR, N_VM>();
  }
}

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

// NORM: squared norm only.  SPILL: squared norm + 16-bit tile to the scratch.  ACCUM: sum over the batch with
// clip factors.  MATERIALIZE: the fp32 per-sample gradient itself to the scratch, nothing else (stage 1 of the
// explicit four-stage flow of Appendix B.2, built as a measured comparison).
enum : int { MODE_NORM = 0, MODE_SPILL = 1, MODE_ACCUM = 2, MODE_MATERIALIZE = 3 };
enum : int { DT_BF16 = 0, DT_F32 = 1, DT_F16 = 2 };

struct GemmArgs {
  const void* X;         // [B][T][P]
  const void* dY;        // [B][T][D]
  int B, T, P, D;
  int tiles_m, tiles_n;  // ceil(D / BM), ceil(P / BN)
  float* partials;       // [B][tiles_m * tiles_n] squared-norm partial sums (NORM, SPILL)
  void* scratch;         // [B][D][P] bfloat16 (SPILL, also for fp16 inputs), fp32 (SPILL of fp32 inputs, MATERIALIZE)
  const float* factors;  // [B] clip factors (ACCUM); nullptr = all ones
  float* out;            // [D][P] (ACCUM)
  int accumulate;        // ACCUM: add to what out holds (gradient accumulation over micro-batches) instead of overwriting
  unsigned long long* trace;   // measurement aid (traced instantiation of the direct-to-LDS kernel only): 8 words per workgroup
};

template <int BM_, int BN_, int BK_, int WAVES_M_, int WAVES_N_, int WAVES_PER_EU_ = 0>
struct TileCfg {
  // waves per SIMD the register allocation must allow (0: whatever one workgroup per CU needs)
  static constexpr int WAVES_PER_EU = WAVES_PER_EU_ ? WAVES_PER_EU_ : (WAVES_M_ * WAVES_N_ + 3) / 4;
  static constexpr int BM = BM_, BN = BN_, BK = BK_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
  static constexpr int NT = 64 * WAVES_M * WAVES_N;
  static constexpr int TM = BM / WAVES_M, TN = BN / WAVES_N;   // per-wave tile
  static constexpr int FM = TM / 32, FN = TN / 32;             // 32x32 blocks per wave
  static constexpr int PAD = 32;                               // row stride = 64 bytes mod 256: 4 consecutive rows hit 4 bank windows
  static constexpr int LDA = BM + PAD, LDB = BN + PAD;         // LDS row strides in elements
  static constexpr int A_STAGE = BK * LDA, B_STAGE = BK * LDB; // elements per stage
  static constexpr int OPERAND_BYTES = 2 * (A_STAGE + B_STAGE) * 2;
  static constexpr int EPILOGUE_BYTES = BM * (BN + 8) * 2 + 64;   // staged 16-bit output tile + per-wave partial sums
  static constexpr int LDS_BYTES = OPERAND_BYTES > EPILOGUE_BYTES ? OPERAND_BYTES : EPILOGUE_BYTES;
  static constexpr int CA = BK * BM / 8 / NT, CB = BK * BN / 8 / NT;   // 16-byte chunks per thread per k-tile
  static_assert(BK % 16 == 0 && TM % 32 == 0 && TN % 32 == 0, "tile shape");
  static_assert((BK * BM / 8) % NT == 0 && (BK * BN / 8) % NT == 0, "copy shape");
  static_assert(NT % (BM / 8) == 0 && NT % (BN / 8) == 0, "copy rows");
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}

template <int DT>
__device__ __forceinline__ f32x16_t mfma32(const s16x8_t a, const s16x8_t b, const f32x16_t c) {
  if constexpr (DT == DT_BF16) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
  } else {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
  }
}

__device__ __forceinline__ s16x4_t lds_read_tr(const unsigned short* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(p));
}

template <int DT>
__device__ __forceinline__ unsigned short to_16bit(float v) {
  if constexpr (DT == DT_BF16) {
    return __builtin_bit_cast(unsigned short, (__bf16)v);
  } else {
    return __builtin_bit_cast(unsigned short, (_Float16)v);
  }
}

typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));

template <int DT>
__device__ __forceinline__ uint32_t pack2_16bit(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  if constexpr (DT == DT_BF16) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
  } else {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2_t));
  }
}

// Workgroup id -> logical work item, so that the workgroups resident on one XCD (ids congruent mod 8)
// cover a contiguous range of work items and share operand panels in that XCD's L2.
__device__ __forceinline__ int xcd_remap(int bid, int total) {
  const int per = total >> 3, rem = total & 7;
  const int xcd = bid & 7, idx = bid >> 3;
  return xcd < rem ? xcd * (per + 1) + idx : rem * (per + 1) + (xcd - rem) * per + idx;
}

// Per-sample passes: the work items (sample, tile), sample-major, are handed out in blocks of 32 consecutive items
// (in the band order of tile_coords below 32 consecutive tiles are 8 tile rows x 4 tile columns: 12 operand panels
// for 32 tiles), block q to XCD q % 8.  Workgroup ids congruent mod 8 share an XCD, so the 32 workgroups resident on
// an XCD are one such block and share its panels in that XCD's L2, and the eight XCDs work on eight consecutive
// blocks - almost always of the same sample - at the same time: one sample's operands (tens of MB) stay in the
// memory-side cache shared by the XCDs for as long as they are needed.  (One sample per XCD made eight working sets
// compete for that cache; an eighth of every sample per XCD cut the blocks of 32 into pieces.)
// Blocks run across sample boundaries, so only the very last block can be short.  (Cutting the blocks per sample
// left a short block at the end of every sample; with an even number of blocks per sample those all went to the
// same four XCDs, which then idled: 36 tiles per sample - blocks of 32 and 4 - ran at 0.56 of the rate.)
// The grid is 8 * ceil(blocks / 8) * 32 workgroups; those beyond the last item return false and exit at once.
constexpr int SHARE_BLOCK = 32;
__host__ __device__ __forceinline__ int64_t shared_block_grid(int tiles, int B) {
  const int64_t blocks = ((int64_t)B * tiles + SHARE_BLOCK - 1) / SHARE_BLOCK;
  return 8 * ((blocks + 7) / 8) * SHARE_BLOCK;
}
__device__ __forceinline__ bool shared_block_item(int bid, int tiles, int B, int* sample, int* tile) {
  const int xcd = bid & 7, idx = bid >> 3;
  const int q = 8 * (idx / SHARE_BLOCK) + xcd, w = idx % SHARE_BLOCK;
  const int g = q * SHARE_BLOCK + w;   // < grid < 2^31 (checked at launch)
  const int s = g / tiles;
  *sample = s;
  *tile = g - s * tiles;
  return g < B * tiles;
}

// Tiles are walked in bands of GROUP_M tile rows, column by column inside a band, so that consecutive
// work items reuse the same dY panel (rows) and neighbouring X panels.
template <int GROUP_M>
__device__ __forceinline__ void tile_coords(int t, int tiles_m, int tiles_n, int* tm, int* tn) {
  const int band = GROUP_M * tiles_n;
  const int g = t / band;
  const int first = g * GROUP_M;
  const int rows = min(tiles_m - first, GROUP_M);
  const int r = t - g * band;
  *tm = first + r % rows;
  *tn = r / rows;
}

// What a workgroup does with its finished tile.  acc[i][j][4q + r] =
// G[m0 + wave_m*TM + 32i + lane%32][n0 + wave_n*TN + 32j + 8q + 4(lane/32) + r].  The caller has ended its main
// loop with a barrier: the operand tiles in LDS are dead and LDS is reused for the reduction and the staging.
template <typename Cfg, int MODE, int DT>
__device__ __forceinline__ void tile_epilogue(const GemmArgs& a, f32x16_t (&acc)[Cfg::FM][Cfg::FN], unsigned short* lds,
                                              int m0, int n0, int sample0, int tile, int tiles) {
  constexpr int BM = Cfg::BM, BN = Cfg::BN, NT = Cfg::NT, FM = Cfg::FM, FN = Cfg::FN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave % Cfg::WAVES_M, wave_n = wave / Cfg::WAVES_M;
  const int row_base = m0 + wave_m * Cfg::TM + (lane & 31);
  const int col_base = n0 + wave_n * Cfg::TN + 4 * (lane >> 5);
  if constexpr (MODE == MODE_NORM || MODE == MODE_SPILL) {
    // intra-block reduction of the squared norm: lane chain -> wave shuffle -> LDS across waves.
    // Rows/columns beyond D/P were loaded as zeros and add nothing.
    // The operand tiles are dead after the barrier that follows the main loop; LDS now stages the
    // 16-bit tile (row pitch BN + 8 elements) so that it leaves the chip in full rows, and holds the
    // per-wave partial sums behind it.
    constexpr int EP = BN + 8;                               // pitch in elements: 16-byte aligned rows
    static_assert(BM * EP * 2 + 64 <= Cfg::LDS_BYTES, "epilogue staging must fit in the operand buffers");
    float* red = (float*)(lds + BM * EP);
    float ss = 0.0f;
    if constexpr (MODE == MODE_SPILL) {
      // The norm is taken of the tile AS PARKED (after the rounding to bfloat16), not of the fp32 accumulators:
      // the clip factor then bounds the norm of exactly what the aggregation sums, so that every clipped
      // per-sample contribution is <= C (the sensitivity bound of Algorithm 1) and not C (1 + 2^-9).
      unsigned short* st = lds + (wave_m * Cfg::TM + (lane & 31)) * EP + wave_n * Cfg::TN + 4 * (lane >> 5);
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            uint2 v;
            // the scratch is bfloat16 for fp16 inputs too: a per-sample gradient before clipping has no
            // bound, and fp16's range (65504) would turn a large one into inf
            v.x = pack2_16bit<DT_BF16>(acc[i][j][4 * q], acc[i][j][4 * q + 1]);
            v.y = pack2_16bit<DT_BF16>(acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
            const float r0 = __builtin_bit_cast(float, v.x << 16), r1 = __builtin_bit_cast(float, v.x & 0xFFFF0000u);
            const float r2 = __builtin_bit_cast(float, v.y << 16), r3 = __builtin_bit_cast(float, v.y & 0xFFFF0000u);
            ss = fmaf(r0, r0, ss); ss = fmaf(r1, r1, ss); ss = fmaf(r2, r2, ss); ss = fmaf(r3, r3, ss);
            *(uint2*)(st + (i * 32) * EP + j * 32 + 8 * q) = v;
          }
    } else {
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
          for (int e = 0; e < 16; ++e) ss = fmaf(acc[i][j][e], acc[i][j][e], ss);
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
      // 16 bytes per lane, BN/8 lanes per row: every store instruction writes whole 2*BN-byte rows
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
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      const int row = row_base + i * 32;
      if (row >= a.D) continue;
      float* obase = a.out;
      if constexpr (MODE == MODE_MATERIALIZE) obase = (float*)a.scratch + (size_t)sample0 * a.D * a.P;
      float* prow = obase + (size_t)row * a.P;
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int col = col_base + j * 32 + 8 * q;
          if (col < a.P) {
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

template <typename Cfg, int MODE, int DT>
__global__ __launch_bounds__(Cfg::NT, Cfg::WAVES_PER_EU) void gemm_mfma_kernel(const GemmArgs a) {
  constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, NT = Cfg::NT;
  constexpr int FM = Cfg::FM, FN = Cfg::FN, LDA = Cfg::LDA, LDB = Cfg::LDB;
  constexpr int CA = Cfg::CA, CB = Cfg::CB;
  extern __shared__ __attribute__((aligned(16))) unsigned short lds[];
  unsigned short* const As = lds;                       // [2][BK][LDA]
  unsigned short* const Bs = lds + 2 * Cfg::A_STAGE;    // [2][BK][LDB]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave % Cfg::WAVES_M, wave_n = wave / Cfg::WAVES_M;

  const int tiles = a.tiles_m * a.tiles_n;
  const int total = (MODE == MODE_ACCUM) ? tiles : tiles * a.B;
  const int item = xcd_remap(blockIdx.x, total);
  const int sample0 = (MODE == MODE_ACCUM) ? 0 : item / tiles;
  const int n_samples = (MODE == MODE_ACCUM) ? a.B : 1;
  const int tile = (MODE == MODE_ACCUM) ? item : item - sample0 * tiles;
  int tm, tn;
  tile_coords<8>(tile, a.tiles_m, a.tiles_n, &tm, &tn);
  const int m0 = tm * BM, n0 = tn * BN;

  // ---- global -> LDS copy plan: thread owns chunk column cc of rows r0, r0 + NT/(BM/8), ...
  constexpr int A_CPR = BM / 8, B_CPR = BN / 8;           // chunks per row
  constexpr int A_RSTEP = NT / A_CPR, B_RSTEP = NT / B_CPR;
  const int a_row = tid / A_CPR, a_cc = tid % A_CPR;
  const int b_row = tid / B_CPR, b_cc = tid % B_CPR;
  const bool a_ok = m0 + a_cc * 8 < a.D;
  const bool b_ok = n0 + b_cc * 8 < a.P;
  // byte offsets inside one sample; an out-of-range column is sent to 2 GiB, beyond num_records, and reads 0
  const uint32_t a_off0 = a_ok ? (uint32_t)(a_row * a.D + m0 + a_cc * 8) * 2u : 0x80000000u;
  const uint32_t b_off0 = b_ok ? (uint32_t)(b_row * a.P + n0 + b_cc * 8) * 2u : 0x80000000u;
  const uint32_t a_rstep = (uint32_t)(A_RSTEP * a.D) * 2u, b_rstep = (uint32_t)(B_RSTEP * a.P) * 2u;
  const uint32_t a_kstep = (uint32_t)(BK * a.D) * 2u, b_kstep = (uint32_t)(BK * a.P) * 2u;
  const uint32_t a_bytes = (uint32_t)a.T * (uint32_t)a.D * 2u, b_bytes = (uint32_t)a.T * (uint32_t)a.P * 2u;
  const int a_lds_w = a_row * LDA + a_cc * 8, b_lds_w = b_row * LDB + b_cc * 8;   // element offsets in a stage

  const int kt_per_sample = (a.T + BK - 1) / BK;
  const int nk = kt_per_sample * n_samples;

  u32x4_t ra[CA], rb[CB];
  // Fetch cursor: (sample, k-tile) of the next tile to load.  Past the last tile it parks on the last
  // sample with k-tile index >= kt_per_sample, where every row is >= T and the buffer loads return zeros,
  // so the main loop can prefetch unconditionally (no branches in its body).
  int ld_s = 0, ld_kt = 0;
  auto load_global = [&]() {
    const char* pa = (const char*)a.dY + (size_t)(sample0 + ld_s) * a_bytes;
    const char* pb = (const char*)a.X + (size_t)(sample0 + ld_s) * b_bytes;
    const __amdgpu_buffer_rsrc_t rsa = make_rsrc(pa, a_bytes), rsb = make_rsrc(pb, b_bytes);
    const uint32_t ao = a_off0 + (uint32_t)ld_kt * a_kstep, bo = b_off0 + (uint32_t)ld_kt * b_kstep;
#pragma unroll
    for (int j = 0; j < CA; ++j) ra[j] = __builtin_amdgcn_raw_buffer_load_b128(rsa, (int)(ao + j * a_rstep), 0, 0);
#pragma unroll
    for (int j = 0; j < CB; ++j) rb[j] = __builtin_amdgcn_raw_buffer_load_b128(rsb, (int)(bo + j * b_rstep), 0, 0);
    ld_kt += 1;
    const bool wrap = ld_kt >= kt_per_sample && ld_s + 1 < n_samples;
    ld_s = wrap ? ld_s + 1 : ld_s;
    ld_kt = wrap ? 0 : ld_kt;
  };
  auto store_lds = [&](int stage) {
    unsigned short* pa = As + stage * Cfg::A_STAGE + a_lds_w;
    unsigned short* pb = Bs + stage * Cfg::B_STAGE + b_lds_w;
#pragma unroll
    for (int j = 0; j < CA; ++j) *(u32x4_t*)(pa + j * A_RSTEP * LDA) = ra[j];
#pragma unroll
    for (int j = 0; j < CB; ++j) *(u32x4_t*)(pb + j * B_RSTEP * LDB) = rb[j];
  };

  // ---- fragment read plan (see header): lane -> (row in the 16-row k-step, column in the 32-wide block)
  const int f_row = 8 * (lane >> 5) + ((lane & 15) >> 2);
  const int f_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  const int a_lds_r = f_row * LDA + wave_m * Cfg::TM + f_col;
  const int b_lds_r = f_row * LDB + wave_n * Cfg::TN + f_col;

  f32x16_t acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  // Fragments are double-buffered: the transposed LDS reads of k-step ks+1 are issued before the
  // matrix-core work of k-step ks, and the first reads of the next k-tile right after the barrier,
  // ahead of the last k-step of this tile.
  constexpr int KS = BK / 16;
  static_assert(KS % 2 == 0, "fragment double buffering assumes an even number of k-steps per tile");
  s16x8_t fa[2][FM], fb[2][FN];
  auto load_frags = [&](int stage, int ks, s16x8_t* pfa, s16x8_t* pfb) {
    const unsigned short* pa = As + stage * Cfg::A_STAGE + a_lds_r + ks * 16 * LDA;
    const unsigned short* pb = Bs + stage * Cfg::B_STAGE + b_lds_r + ks * 16 * LDB;
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      const s16x4_t lo = lds_read_tr(pa + i * 32);
      const s16x4_t hi = lds_read_tr(pa + 4 * LDA + i * 32);
      pfa[i] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
#pragma unroll
    for (int j = 0; j < FN; ++j) {
      const s16x4_t lo = lds_read_tr(pb + j * 32);
      const s16x4_t hi = lds_read_tr(pb + 4 * LDB + j * 32);
      pfb[j] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
  };

  load_global();
  store_lds(0);
  load_global();
  __syncthreads();
  load_frags(0, 0, fa[0], fb[0]);

  constexpr int N_MMA = FM * FN, N_RD = 2 * (FM + FN);
  // One k-tile; `cur` is the LDS stage it computes from.
  auto k_tile = [&](int k, int cur) {
    static_for<KS>([&](auto ks_c) {
      constexpr int ks = decltype(ks_c)::value;
      constexpr int cb = ks & 1, nb = cb ^ 1;
      constexpr bool do_store = ks == (KS >= 4 ? KS / 2 - 1 : 0);
      constexpr bool do_fetch = ks == KS - 2;
      if constexpr (ks + 1 < KS) {
        load_frags(cur, ks + 1, fa[nb], fb[nb]);
      } else {
        __syncthreads();   // tile k+1 is in LDS, and every wave has read the last fragments of tile k
        load_frags(cur ^ 1, 0, fa[nb], fb[nb]);
      }
      if constexpr (do_store) store_lds(cur ^ 1);      // hand the prefetched tile to the other stage
      if constexpr (do_fetch) load_global();           // and start the next fetch into the freed registers
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) acc[i][j] = mfma32<DT>(fb[cb][j], fa[cb][i], acc[i][j]);
      sched_interleave<0, N_MMA, N_RD, do_store ? CA + CB : 0, do_fetch ? CA + CB : 0>();
    });
    if constexpr (MODE == MODE_ACCUM) {
      // sample boundary: rescale so that acc always holds sum_{j<=i} (c_j / c_i) G_j; exact up to one
      // fp32 rounding per boundary, and needs no second set of accumulators
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
  if constexpr (KS >= 4) {
    // 64-deep k-tiles: two k-tiles per loop trip with the LDS stage a compile-time constant (measured 3 %
    // faster); an odd tile count runs one extra k-tile on the zeros the parked fetch cursor delivers.
    for (int k = 0; k < nk; k += 2) {
      k_tile(k, 0);
      k_tile(k + 1, 1);
    }
  } else {
    // 32-deep k-tiles: the same unrolling measured 2 % slower, so one k-tile per trip
    for (int k = 0; k < nk; ++k) k_tile(k, k & 1);
  }
  __syncthreads();   // the reduction below reuses the LDS tiles

  tile_epilogue<Cfg, MODE, DT>(a, acc, lds, m0, n0, sample0, tile, tiles);
}

}  // namespace flashdp
