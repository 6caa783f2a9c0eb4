// Algorithm 1 in ONE launch, with its block-wise synchronisation as a barrier across the grid: the form the paper
// calls the ideal single-kernel solution (Section 4.2) and gave up for lack of a grid-wide barrier.  It applies when
// every output tile of the layer has a workgroup of its own on the chip at the same time (tiles of 256 x 256 <= CUs),
// e.g. a 4096 x 4096 layer on 256 CUs.
//
// One workgroup owns one output tile for ALL samples.  Its ring of direct-to-LDS loads runs on from one sample into
// the next (reduction index = all tokens of sample 0, then of sample 1, ...), so a workgroup starts and drains its
// pipeline once per layer instead of once per sample.  At every sample boundary the workgroup takes the squared norm
// of its tile (one partial per wave), parks the tile as bfloat16 - except the last sample's, which stays in the
// accumulators - and clears the accumulators.  After the last sample: the partials go to memory, all workgroups meet
// at the barrier, every workgroup sums the partials of every sample in the same fixed order (so all see the same clip
// factors), and forms sum_i c_i G_i + sigma C z for its own tile from its own parked tiles and the accumulators it
// still holds, and stores it.  Against the scratch schedule this saves two launches, the pipeline start-up per sample
// tile, one sample's round trip through memory, and the parked tiles are re-read by the workgroup that wrote them.
//
// The barrier is a counter in memory (release/acquire at device scope: the XCDs' L2s are written back / invalidated
// by those operations) with a BOUNDED wait: the workgroups are co-resident whenever the chip is otherwise idle, but
// nothing in an ordinary launch guarantees it, so a workgroup that has waited spin_limit rounds gives up, raises the
// error flag in the workspace and poisons its output with NaN instead of hanging the GPU.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_mfma_dma.hip.h"
#include "philox_gauss.h"

namespace flashdp {

struct FusedArgs {
  const void* X;        // [B][T][P]
  const void* dY;       // [B][T][D]
  int B, T, P, D;
  int tiles_m, tiles_n;
  float C;
  float noise_scale;    // sigma * C, or 0
  uint64_t seed;
  uint32_t layer;
  int accumulate;       // add to what out holds
  float* partials;      // [B][tiles][8] squared-norm partial sums, one per wave
  void* scratch;        // [B - 1][D][P] bfloat16 parked tiles
  unsigned int* sync;   // [0] arrival counter (zero at launch), [1] error flag (set when a wait gave up)
  float* out;           // [D][P]
  float* out_norms;     // [B] or null
  unsigned int spin_limit;
};

struct FusedCfg : DmaCfg<4> {
  // The ring; the parking of a tile borrows a consumed ring stage; after the last sample the whole allocation is
  // reused, first for the reduction of the partials, then for handing the accumulators over half a tile at a time
  // (per wave 64 rows x 64 columns of fp32, row pitch 68 floats).
  static constexpr int OUT_PITCH = 68;
  static constexpr int OUT_STAGE_BYTES = 8 * 64 * OUT_PITCH * 4;
  static constexpr int LDS_BYTES = OUT_STAGE_BYTES > DmaCfg<4>::OPERAND_BYTES ? OUT_STAGE_BYTES : DmaCfg<4>::OPERAND_BYTES;
  static constexpr int MAX_B = 16;
};

__global__ void fused_sync_reset_kernel(unsigned int* sync) {
  if (threadIdx.x < 2) sync[threadIdx.x] = 0u;
}

template <int DT>
__global__ __launch_bounds__(FusedCfg::NT, FusedCfg::WAVES_PER_EU) void fused_dp_kernel(const FusedArgs a) {
  using Cfg = FusedCfg;
  constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, FM = Cfg::FM, FN = Cfg::FN, STAGES = Cfg::STAGES;
  constexpr int ROW = 256;
  extern __shared__ __attribute__((aligned(16))) unsigned short lds[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wave_m = wave % Cfg::WAVES_M, wave_n = wave / Cfg::WAVES_M;
  const int tiles = a.tiles_m * a.tiles_n;
  const int tile = xcd_remap(blockIdx.x, tiles);
  int tm, tn;
  tile_coords<8>(tile, a.tiles_m, a.tiles_n, &tm, &tn);
  const int m0 = tm * BM, n0 = tn * BN;

  const int d_row = lds_plan::load_row(wave, lane);
  const int d_chunk = lds_plan::load_chunk(wave, lane);
  const bool a_ok = m0 + d_chunk * 8 < a.D;
  const bool b_ok = n0 + d_chunk * 8 < a.P;
  const uint32_t a_off0 = a_ok ? (uint32_t)(d_row * a.D + m0 + d_chunk * 8) * 2u : 0x80000000u;
  const uint32_t b_off0 = b_ok ? (uint32_t)(d_row * a.P + n0 + d_chunk * 8) * 2u : 0x80000000u;
  const uint32_t a_half = (uint32_t)(16 * a.D) * 2u, b_half = (uint32_t)(16 * a.P) * 2u;
  const uint32_t a_kstep = (uint32_t)(BK * a.D) * 2u, b_kstep = (uint32_t)(BK * a.P) * 2u;
  const uint32_t a_bytes = (uint32_t)a.T * (uint32_t)a.D * 2u, b_bytes = (uint32_t)a.T * (uint32_t)a.P * 2u;
  const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned short*)lds;

  // Every sample takes kt_pad k-tiles, a multiple of the ring depth, so that a sample boundary always falls after
  // stage STAGES - 1; k-tiles kt_per_sample .. kt_pad - 1 of a sample address rows >= T and read zeros.
  const int kt_per_sample = (a.T + BK - 1) / BK;
  const int kt_pad = (kt_per_sample + STAGES - 1) / STAGES * STAGES;

  int ld_s = 0, ld_kt = 0;   // fetch cursor; past the last sample it parks on rows >= T of that sample
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
    const bool wrap = ld_kt >= kt_pad && ld_s + 1 < a.B;
    ld_s = wrap ? ld_s + 1 : ld_s;
    ld_kt = wrap ? 0 : ld_kt;
  };

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
  wait_loads_outstanding<4 * (STAGES - 2)>();
  __syncthreads();
  load_frags(0, 0, fa[0], fb[0]);

  constexpr int N_MMA = FM * FN, N_RD = 2 * (FM + FN);
  auto k_tile = [&](auto cur_c, auto wait_c) {
    constexpr int cur = decltype(cur_c)::value;
    constexpr int nxt = (cur + 1) % STAGES, refill = (cur + STAGES - 1) % STAGES;
    load_frags(cur, 1, fa[1], fb[1]);
    issue_loads(refill);
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j) acc[i][j] = mfma32<DT>(fb[0][j], fa[0][i], acc[i][j]);
    sched_interleave<0, N_MMA, N_RD, 0, 0>();
    wait_loads_outstanding<decltype(wait_c)::value>();
    __syncthreads();
    load_frags(nxt, 0, fa[0], fb[0]);
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j) acc[i][j] = mfma32<DT>(fb[1][j], fa[1][i], acc[i][j]);
    sched_interleave<0, N_MMA, N_RD, 0, 0>();
  };

  __shared__ float ss_keep[Cfg::MAX_B][8];   // squared-norm partials of this workgroup, [sample][wave]
  // This wave's 128 x 64 part of the tile.  acc[i][j][4q + r] = G[row0 + 32i + lane%32][col0 + 32j + 8q + 4(lane/32) + r].
  const int row0 = m0 + wave_m * Cfg::TM, col0 = n0 + wave_n * Cfg::TN;
  // Staging of 32 rows x 64 columns of bfloat16 (4 KB) in the part of ring stage STAGES - 1 that only this wave's own
  // direct loads write (four 1 KB pieces: rows 8p .. 8p+7 of the staged block in piece p), so that no other wave and
  // no load in flight touches it: at a sample boundary that stage has been consumed by every wave (they all passed
  // the barrier after reading it) and is refilled by this wave's next issue_loads only.  The 16-byte chunk c of staged
  // row r is kept at chunk c ^ (r & 7).
  auto piece = [&](int p) { return lds_plan::load_dst_bytes(STAGES - 1, p >> 1, wave, p & 1); };

  // Stores count in the same in-order memory counter as the direct loads.  Right after a tile has been parked the
  // counter holds, oldest first: the loads of the next two k-tiles (issued before the parking), the 16 stores of the
  // parking, then the loads issued since.  "The next k-tile has landed" is then "at most 4 + 16 + 4 outstanding"
  // instead of "at most 8", which would wait for the stores to be acknowledged by memory (microseconds, with every
  // workgroup parking at about the same time).  Only a workgroup whose tile lies wholly inside the matrix issues
  // exactly 16 stores per lane and may count like this.
  const bool whole_tile = m0 + BM <= a.D && n0 + BN <= a.P;
  using W8 = std::integral_constant<int, 4 * (STAGES - 2)>;
  using W24 = std::integral_constant<int, 24>;
  for (int s = 0; s < a.B; ++s) {
    int k = 0;
    if (s > 0 && whole_tile) {
      k_tile(std::integral_constant<int, 0>{}, W24{});
      k_tile(std::integral_constant<int, 1>{}, W24{});
      k_tile(std::integral_constant<int, 2>{}, W8{});
      k_tile(std::integral_constant<int, 3>{}, W8{});
      k = STAGES;
    }
    for (; k < kt_pad; k += STAGES) {
      static_for<STAGES>([&](auto s_c) { k_tile(s_c, W8{}); });
    }
    // ---- sample boundary: squared norm of this wave's part, park it (all but the last sample), clear
    const bool park = s + 1 < a.B;
    float ss = 0.0f;
    if (park) {
      unsigned short* sc = (unsigned short*)a.scratch + (size_t)s * a.D * a.P;
      // The main loop needs every register: the addresses of this phase hang on a value the compiler cannot see
      // through, so that they are formed here, when needed, and not ahead of the loop and kept (spilled) across it.
      uint32_t hide = 0;
      asm volatile("" : "+v"(hide));
      const int ln = lane + (int)hide, r_p = ln & 31, h_p = ln >> 5;
#pragma unroll
      for (int i = 0; i < FM; ++i) {
        char* wr = (char*)lds + piece(r_p >> 3) + (r_p & 7) * 128 + 8 * h_p;
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            uint2 v;
            v.x = pack2_16bit<DT_BF16>(acc[i][j][4 * q], acc[i][j][4 * q + 1]);
            v.y = pack2_16bit<DT_BF16>(acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
            // the norm of the tile as parked: the clip factor then bounds what is summed (see tile_epilogue)
            const float r0 = __builtin_bit_cast(float, v.x << 16), r1 = __builtin_bit_cast(float, v.x & 0xFFFF0000u);
            const float r2 = __builtin_bit_cast(float, v.y << 16), r3 = __builtin_bit_cast(float, v.y & 0xFFFF0000u);
            ss = fmaf(r0, r0, ss); ss = fmaf(r1, r1, ss); ss = fmaf(r2, r2, ss); ss = fmaf(r3, r3, ss);
            *(uint2*)(wr + (((4 * j + q) ^ (r_p & 7)) << 4)) = v;
          }
        __builtin_amdgcn_wave_barrier();   // same wave, other lanes: LDS keeps a wave's accesses in order
        const int rr = ln >> 3, cc = ln & 7;
        const int col = col0 + 8 * cc;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          const u32x4_t v = *(const u32x4_t*)((const char*)lds + piece(p) + rr * 128 + ((cc ^ rr) << 4));
          const int row = row0 + 32 * i + 8 * p + rr;
          if (row < a.D && col < a.P) __builtin_nontemporal_store(v, (u32x4_t*)(sc + (size_t)row * a.P + col));
        }
        __builtin_amdgcn_wave_barrier();
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
    if (lane == 0) ss_keep[s][wave] = ss;   // to memory after the last sample: a store here would sit between the loads
    if (park) {
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
          for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
      // the first fragments of the next sample are read again here rather than kept across the parking, which needs
      // their registers (the ring stage they come from is untouched)
      load_frags(0, 0, fa[0], fb[0]);
    }
  }
  __builtin_amdgcn_wave_barrier();
  if (lane < a.B) a.partials[((size_t)lane * tiles + tile) * 8 + wave] = ss_keep[lane][wave];
  wait_loads_outstanding<0>();   // parked loads (zeros) still land in the ring; stores of tiles and partials are done
  __syncthreads();

  // ---- block-wise synchronisation: every tile of every sample has its partials in memory
  __shared__ unsigned int gave_up;
  if (tid == 0) {
    __hip_atomic_fetch_add(a.sync, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    unsigned int spins = 0, bad = 0;
    while (__hip_atomic_load(a.sync, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) < (unsigned int)tiles) {
      __builtin_amdgcn_s_sleep(32);
      if (++spins > a.spin_limit) { bad = 1; break; }
    }
    if (bad) __hip_atomic_store(a.sync + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    gave_up = bad;
  }
  __syncthreads();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");   // the other threads read the partials too

  // ---- inter-block reduce and clip factors: partials of sample i summed in a fixed order (fp64), by every workgroup
  __shared__ float factors[Cfg::MAX_B];
  double* red = (double*)lds;                     // [B][512]: the ring is dead
  const int n_part = tiles * 8;
  for (int i = 0; i < a.B; ++i) {
    double t = 0.0;
    for (int k = tid; k < n_part; k += Cfg::NT) t += (double)a.partials[(size_t)i * n_part + k];
    red[i * Cfg::NT + tid] = t;
  }
  __syncthreads();
  for (int wdt = Cfg::NT / 2; wdt > 0; wdt >>= 1) {
    if (tid < wdt)
      for (int i = 0; i < a.B; ++i) red[i * Cfg::NT + tid] += red[i * Cfg::NT + tid + wdt];
    __syncthreads();
  }
  if (tid < a.B) {
    const double n = sqrt(red[tid * Cfg::NT]);
    const double ratio = n / (double)a.C;
    // a NaN norm gives a NaN factor (never let through unclipped); a wait that gave up poisons the output
    float c = (float)(1.0 / (ratio <= 1.0 ? 1.0 : ratio));
    if (gave_up) c = __builtin_nanf("");
    factors[tid] = c;
    if (blockIdx.x == 0 && a.out_norms) a.out_norms[tid] = (float)n;
  }
  __syncthreads();   // factors are known, and nobody reads `red` any more: the allocation is free again

  // ---- clip, batch sum, noise, store: own tile, parked samples from memory, the last sample from the accumulators.
  // The accumulators are handed over through LDS half a tile at a time (rows 0..63, then 64..127 of this wave's part,
  // already scaled by the last sample's factor), so that the rest runs as an ordinary loop with whole-row accesses:
  // a lane takes four consecutive columns, sixteen lanes a 64-column row of the wave's part (256 bytes of out,
  // 128 bytes of a parked tile), one instruction four rows.  Summation order per element as in the streaming
  // aggregation kernel: samples 0 .. B-1 in turn, then the noise.
  const float c_last = factors[a.B - 1];
  const size_t S = (size_t)a.D * a.P;
  float* stage = (float*)lds + (size_t)wave * 64 * Cfg::OUT_PITCH;
  uint32_t hide2 = 0;
  asm volatile("" : "+v"(hide2));   // as at the sample boundaries: nothing of this phase is to be kept across the main loop
  const int lf = lane + (int)hide2, r_f = lf & 31, h_f = lf >> 5;
#pragma unroll
  for (int half = 0; half < 2; ++half) {
#pragma unroll
    for (int ii = 0; ii < 2; ++ii)
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int i = 2 * half + ii;
          *(float4*)(stage + (32 * ii + r_f) * Cfg::OUT_PITCH + 32 * j + 8 * q + 4 * h_f) =
              make_float4(c_last * acc[i][j][4 * q], c_last * acc[i][j][4 * q + 1], c_last * acc[i][j][4 * q + 2], c_last * acc[i][j][4 * q + 3]);
        }
    __builtin_amdgcn_wave_barrier();   // this wave's own region: LDS keeps a wave's accesses in order
    // (1) add the parked samples: all sixteen row groups of the half at once, so that sixteen loads per lane are in
    //     flight per sample (two waves per SIMD hide no latency by themselves); back to LDS
    {
      float4 v[16];
      size_t e[16];
      bool ok[16];
#pragma unroll
      for (int it = 0; it < 16; ++it) {
        const int rr = 4 * it + (lf >> 4), cc = 4 * (lf & 15);
        const int row = row0 + 64 * half + rr, col = col0 + cc;
        ok[it] = row < a.D && col < a.P;   // P is a multiple of 8 on this path: a group of 4 is all in or all out
        e[it] = (size_t)row * a.P + col;
        v[it] = make_float4(0.f, 0.f, 0.f, 0.f);
      }
      if (a.accumulate) {
#pragma unroll
        for (int it = 0; it < 16; ++it)
          if (ok[it]) v[it] = *(const float4*)(a.out + e[it]);
      }
      for (int s = 0; s + 1 < a.B; ++s) {
        const unsigned short* sp = (const unsigned short*)a.scratch + (size_t)s * S;
        const float c = factors[s];
        uint2 pk[16];
#pragma unroll
        for (int it = 0; it < 16; ++it) pk[it] = ok[it] ? *(const uint2*)(sp + e[it]) : make_uint2(0u, 0u);
#pragma unroll
        for (int it = 0; it < 16; ++it) {
          v[it].x = fmaf(c, __builtin_bit_cast(float, pk[it].x << 16), v[it].x);
          v[it].y = fmaf(c, __builtin_bit_cast(float, pk[it].x & 0xFFFF0000u), v[it].y);
          v[it].z = fmaf(c, __builtin_bit_cast(float, pk[it].y << 16), v[it].z);
          v[it].w = fmaf(c, __builtin_bit_cast(float, pk[it].y & 0xFFFF0000u), v[it].w);
        }
      }
#pragma unroll
      for (int it = 0; it < 16; ++it) {
        const int rr = 4 * it + (lf >> 4), cc = 4 * (lf & 15);
        float4* p = (float4*)(stage + rr * Cfg::OUT_PITCH + cc);
        const float4 last = *p;   // c_last * G: rounded once on its way through LDS, as fmaf(c, g, v) rounds once, later
        *p = make_float4(v[it].x + last.x, v[it].y + last.y, v[it].z + last.z, v[it].w + last.w);
      }
    }
    __builtin_amdgcn_wave_barrier();
    // (2) noise and store, an ordinary loop (the generator's code exists once)
    for (int it = 0; it < 16; ++it) {
      const int rr = 4 * it + (lf >> 4), cc = 4 * (lf & 15);
      const int row = row0 + 64 * half + rr, col = col0 + cc;
      float4 v = *(const float4*)(stage + rr * Cfg::OUT_PITCH + cc);
      if (row < a.D && col < a.P) {
        const size_t e = (size_t)row * a.P + col;
        if (a.noise_scale != 0.0f) {
          const Normals4 z = noise_group(a.seed, a.layer, e >> 2);
          v.x = fmaf(a.noise_scale, z.z[0], v.x);
          v.y = fmaf(a.noise_scale, z.z[1], v.y);
          v.z = fmaf(a.noise_scale, z.z[2], v.z);
          v.w = fmaf(a.noise_scale, z.z[3], v.w);
        }
        *(float4*)(a.out + e) = v;
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
}

}  // namespace flashdp
