// The memory-bound steps of Algorithm 1 after the grid-wide synchronisation: inter-block reduction of the
// squared norms and clip factor (B_G' = B_G / max(1, sqrt(||B_G||^2') / C)), and the batch aggregation with
// noise (B_dW = sum_b B_G' + N(0, sigma^2 C^2 I)) read back from the per-layer scratch.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_mfma.hip.h"
#include "philox_gauss.h"

namespace flashdp {

// Inter-block reduction of one sample's squared norm by one wave, in a fixed order so that the result does not
// depend on scheduling or on which kernel does it: lane l adds partials l, l + 64, ... (fp64), then a butterfly
// over the lanes (a + b == b + a, so every lane ends with the same bits).  Replaces the per-block atomic add of the
// paper's inter-block reduce; the kernel boundary before it is the block-wise synchronisation.
__device__ __forceinline__ double sample_norm_sq(const float* __restrict__ partials_i, int n, int lane) {
  double s = 0.0;
  for (int k = lane; k < n; k += 64) s += (double)partials_i[k];
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
  return s;
}

// c_i = 1 / max(1, n_i / C), written so that a NaN norm gives a NaN factor: a sample whose norm is unknown must not
// pass unclipped.
__device__ __forceinline__ float clip_factor_of(double norm, float C) {
  const double ratio = norm / (double)C;
  return (float)(1.0 / (ratio <= 1.0 ? 1.0 : ratio));
}

// n_i = sqrt(sum of partials), c_i: one wave per sample, four samples per workgroup.  (The streaming kernels of the
// scratch schedule do this themselves, see below; this kernel serves the schedules whose second pass is a contraction.)
__global__ __launch_bounds__(256) void clip_factors_kernel(const float* __restrict__ partials, int tiles, float C, int B,
                                                           float* __restrict__ factors, float* __restrict__ out_norms) {
  const int lane = threadIdx.x & 63;
  const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (i >= B) return;
  const double n = sqrt(sample_norm_sq(partials + (size_t)i * tiles, tiles, lane));
  if (lane == 0) {
    factors[i] = clip_factor_of(n, C);
    if (out_norms) out_norms[i] = (float)n;
  }
}

// The same inside a streaming kernel: every workgroup (4 waves) works out all clip factors into LDS for itself, wave w
// taking samples w, w + 4, ...; workgroup 0 also reports the norms.  Costs a workgroup about a microsecond and
// B * tiles * 4 bytes of (cached) reads, and saves a kernel launch per layer; B <= MAX_FUSED_CLIP_B.
constexpr int MAX_FUSED_CLIP_B = 64;
__device__ __forceinline__ void clip_factors_to_lds(const float* __restrict__ partials, int tiles, float C, int B,
                                                    float* lds_factors, float* __restrict__ out_norms) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int i = wave; i < B; i += 4) {
    const double n = sqrt(sample_norm_sq(partials + (size_t)i * tiles, tiles, lane));
    if (lane == 0) {
      lds_factors[i] = clip_factor_of(n, C);
      if (blockIdx.x == 0 && out_norms) out_norms[i] = (float)n;
    }
  }
  __syncthreads();
}

template <int DT>
__device__ __forceinline__ void widen8(const u32x4_t v, float* f) {
  if constexpr (DT == DT_BF16) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      f[2 * q] = __builtin_bit_cast(float, v[q] << 16);
      f[2 * q + 1] = __builtin_bit_cast(float, v[q] & 0xFFFF0000u);
    }
  } else {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      f[2 * q] = (float)__builtin_bit_cast(_Float16, (unsigned short)(v[q] & 0xFFFFu));
      f[2 * q + 1] = (float)__builtin_bit_cast(_Float16, (unsigned short)(v[q] >> 16));
    }
  }
}

// out[e] = sum_i c_i * scratch[i][e] + noise_scale * z[e], 8 consecutive elements per thread
// (16-byte loads from the 16-bit scratch, two Philox groups, two 16-byte stores).  n8 = S / 8.
// DEEP: four samples' loads in flight per thread (the kernels that have the chip to themselves); otherwise one, which
// keeps the kernel within the registers left over beside a resident contraction workgroup (the overlapped schedule).
template <int DT, bool DEEP>
__device__ __forceinline__ void aggregate16_one(const void* __restrict__ scratch, const float* __restrict__ factors, int B,
                                                size_t S, size_t v, float noise_scale, uint64_t seed, uint32_t layer,
                                                float* __restrict__ out, int accumulate);

template <int DT>
__global__ __launch_bounds__(256) void aggregate16_kernel(const void* __restrict__ scratch, const float* __restrict__ factors,
                                                          int B, size_t S, size_t n8, float noise_scale, uint64_t seed,
                                                          uint32_t layer, float* __restrict__ out, int accumulate) {
  const size_t v = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (v >= n8) return;
  aggregate16_one<DT, true>(scratch, factors, B, S, v, noise_scale, seed, layer, out, accumulate);
}

// The same work with a fixed, small number of workgroups striding over the elements: the form that runs on
// a second stream beside the next layer's contraction kernel.  The ordinary grid would take every slot a
// finishing contraction workgroup frees and starve the contraction (its workgroups need a whole CU's LDS)
// until the aggregation is done; a bounded grid becomes resident once and leaves the rest of the chip alone.
template <int DT>
__global__ __launch_bounds__(256) void aggregate16_persistent_kernel(const void* __restrict__ scratch,
                                                                     const float* __restrict__ factors, int B, size_t S,
                                                                     size_t n8, float noise_scale, uint64_t seed,
                                                                     uint32_t layer, float* __restrict__ out, int accumulate) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t v = (size_t)blockIdx.x * 256 + threadIdx.x; v < n8; v += stride)
    aggregate16_one<DT, false>(scratch, factors, B, S, v, noise_scale, seed, layer, out, accumulate);
}

// The whole tail of Algorithm 1 after the block-wise synchronisation in one kernel: inter-block reduce and clip
// factors (every workgroup for itself, into LDS), then the clipped batch sum with noise as above.  DEEP as in
// aggregate16_one: on for the ordinary grid, off for the bounded grid that runs beside a contraction kernel.
template <int DT, bool DEEP>
__global__ __launch_bounds__(256) void clip_aggregate16_kernel(const void* __restrict__ scratch, const float* __restrict__ partials,
                                                               int tiles, float C, float* __restrict__ out_norms, int B, size_t S,
                                                               size_t n8, float noise_scale, uint64_t seed, uint32_t layer,
                                                               float* __restrict__ out, int accumulate) {
  __shared__ float fac[MAX_FUSED_CLIP_B];
  clip_factors_to_lds(partials, tiles, C, B, fac, out_norms);
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t v = (size_t)blockIdx.x * 256 + threadIdx.x; v < n8; v += stride)
    aggregate16_one<DT, DEEP>(scratch, fac, B, S, v, noise_scale, seed, layer, out, accumulate);
}

template <int DT, bool DEEP>
__device__ __forceinline__ void aggregate16_one(const void* __restrict__ scratch, const float* __restrict__ factors, int B,
                                                size_t S, size_t v, float noise_scale, uint64_t seed, uint32_t layer,
                                                float* __restrict__ out, int accumulate) {
  float acc[8];
#pragma unroll
  for (int q = 0; q < 8; ++q) acc[q] = 0.0f;
  if (accumulate) {   // gradient accumulation: continue from the sum of the earlier micro-batches
    const float4 o0 = ((const float4*)out)[2 * v], o1 = ((const float4*)out)[2 * v + 1];
    acc[0] = o0.x; acc[1] = o0.y; acc[2] = o0.z; acc[3] = o0.w;
    acc[4] = o1.x; acc[5] = o1.y; acc[6] = o1.z; acc[7] = o1.w;
  }
  const u32x4_t* src = (const u32x4_t*)scratch + v;
  const size_t stride = S / 8;
  Normals4 z0 = {}, z1 = {};
  if constexpr (DEEP) {
    // Four samples' loads are issued before the first is used (64 bytes in flight per thread), and the noise, which
    // depends on nothing that is loaded, is generated while they are on their way; the sums keep the sample order.
    u32x4_t raw[4] = {};
    const int first = B < 4 ? B : 4;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if (q < first) raw[q] = __builtin_nontemporal_load(src + (size_t)q * stride);
    if (noise_scale != 0.0f) {
      z0 = noise_group(seed, layer, 2 * v);
      z1 = noise_group(seed, layer, 2 * v + 1);
    }
    int i = 0;
    while (i < B) {
      const int n = B - i < 4 ? B - i : 4;
      u32x4_t cur[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) cur[q] = raw[q];
      const int nn = B - i - n < 4 ? B - i - n : 4;
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (q < nn) raw[q] = __builtin_nontemporal_load(src + (size_t)(i + n + q) * stride);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (q < n) {
          const float c = factors[i + q];
          float f[8];
          widen8<DT>(cur[q], f);
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[e] = fmaf(c, f[e], acc[e]);
        }
      }
      i += n;
    }
  } else {
    for (int i = 0; i < B; ++i) {
      const u32x4_t raw = __builtin_nontemporal_load(src + (size_t)i * stride);
      const float c = factors[i];
      float f[8];
      widen8<DT>(raw, f);
#pragma unroll
      for (int q = 0; q < 8; ++q) acc[q] = fmaf(c, f[q], acc[q]);
    }
    if (noise_scale != 0.0f) {
      z0 = noise_group(seed, layer, 2 * v);
      z1 = noise_group(seed, layer, 2 * v + 1);
    }
  }
  if (noise_scale != 0.0f) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      acc[q] = fmaf(noise_scale, z0.z[q], acc[q]);
      acc[4 + q] = fmaf(noise_scale, z1.z[q], acc[4 + q]);
    }
  }
  typedef float f32x4_t __attribute__((ext_vector_type(4)));
  f32x4_t* dst = (f32x4_t*)out + 2 * v;
  const f32x4_t lo = {acc[0], acc[1], acc[2], acc[3]}, hi = {acc[4], acc[5], acc[6], acc[7]};
  __builtin_nontemporal_store(lo, dst);
  __builtin_nontemporal_store(hi, dst + 1);
}

// Generic version: any scratch type, any S; one Philox group (4 elements) per thread.
template <int DT>
__global__ __launch_bounds__(256) void aggregate_generic_kernel(const void* __restrict__ scratch, const float* __restrict__ factors,
                                                                int B, size_t S, float noise_scale, uint64_t seed,
                                                                uint32_t layer, float* __restrict__ out, int accumulate) {
  const size_t g = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (4 * g >= S) return;
  float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  if (accumulate) {
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if (4 * g + q < S) acc[q] = out[4 * g + q];
  }
  for (int i = 0; i < B; ++i) {
    const float c = factors[i];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const size_t e = 4 * g + q;
      if (e < S) {
        float val;
        if constexpr (DT == DT_F32) {
          val = ((const float*)scratch)[(size_t)i * S + e];
        } else if constexpr (DT == DT_BF16) {
          val = __builtin_bit_cast(float, (uint32_t)((const unsigned short*)scratch)[(size_t)i * S + e] << 16);
        } else {
          val = (float)((const _Float16*)scratch)[(size_t)i * S + e];
        }
        acc[q] = fmaf(c, val, acc[q]);
      }
    }
  }
  if (noise_scale != 0.0f) {
    const Normals4 z = noise_group(seed, layer, g);
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[q] = fmaf(noise_scale, z.z[q], acc[q]);
  }
#pragma unroll
  for (int q = 0; q < 4; ++q)
    if (4 * g + q < S) out[4 * g + q] = acc[q];
}

// ---- the explicit four-stage flow of Appendix B.2 on a materialised fp32 G[B][S] (measured comparison) ----

// Stage 2: per-sample squared norm of G_i read back from HBM.  grid = (chunks, B); every workgroup sums a
// contiguous chunk of 256 * 4 * ITER elements and writes one partial; clip_factors_kernel finishes.
__global__ __launch_bounds__(256) void explicit_norm_kernel(const float* __restrict__ G, size_t S, int chunks,
                                                            float* __restrict__ partials) {
  __shared__ float red[4];
  const int i = blockIdx.y, tid = threadIdx.x;
  const size_t per = (S + chunks - 1) / chunks;
  const size_t lo = (size_t)blockIdx.x * per, hi = lo + per < S ? lo + per : S;
  const float* g = G + (size_t)i * S;
  float ss = 0.0f;
  for (size_t e = lo + (size_t)tid * 4; e < hi; e += 1024) {
    if (e + 3 < hi && (((uintptr_t)(g + e)) & 15) == 0) {
      const float4 v = *(const float4*)(g + e);
      ss = fmaf(v.x, v.x, ss); ss = fmaf(v.y, v.y, ss); ss = fmaf(v.z, v.z, ss); ss = fmaf(v.w, v.w, ss);
    } else {
      for (size_t q = e; q < hi && q < e + 4; ++q) ss = fmaf(g[q], g[q], ss);
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
  if ((tid & 63) == 0) red[tid >> 6] = ss;
  __syncthreads();
  if (tid == 0) partials[(size_t)i * chunks + blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

// Stage 3: G'_i = c_i * G_i, in place (load G and the factor, store the clipped gradient back to HBM).
__global__ __launch_bounds__(256) void explicit_clip_kernel(float* __restrict__ G, size_t S, const float* __restrict__ factors) {
  const int i = blockIdx.y;
  const float c = factors[i];
  float* g = G + (size_t)i * S;
  const size_t e = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (e + 3 < S && (((uintptr_t)(g + e)) & 15) == 0) {
    float4 v = *(float4*)(g + e);
    v.x *= c; v.y *= c; v.z *= c; v.w *= c;
    *(float4*)(g + e) = v;
  } else {
    for (size_t q = e; q < S && q < e + 4; ++q) g[q] *= c;
  }
}

// Stage 4: out = sum_i G'_i + noise (one Philox group of 4 elements per thread).  With `factors` the clip
// factor is applied here instead (out = sum_i c_i G_i + noise): the aggregation of the scratch schedule
// for fp32 inputs, whose scratch is fp32 as well.
__global__ __launch_bounds__(256) void aggregate32_kernel(const float* __restrict__ G, const float* __restrict__ factors, int B,
                                                          size_t S, float noise_scale, uint64_t seed, uint32_t layer,
                                                          float* __restrict__ out, int accumulate) {
  const size_t g4 = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t e = g4 * 4;
  if (e >= S) return;
  float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  const bool vec = e + 3 < S && (S & 3) == 0;
  if (accumulate) {
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if (e + q < S) acc[q] = out[e + q];
  }
  for (int i = 0; i < B; ++i) {
    const float* g = G + (size_t)i * S + e;
    const float c = factors ? factors[i] : 1.0f;
    if (vec) {
      typedef float f32x4_t __attribute__((ext_vector_type(4)));
      const f32x4_t v = __builtin_nontemporal_load((const f32x4_t*)g);
      acc[0] = fmaf(c, v.x, acc[0]); acc[1] = fmaf(c, v.y, acc[1]); acc[2] = fmaf(c, v.z, acc[2]); acc[3] = fmaf(c, v.w, acc[3]);
    } else {
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (e + q < S) acc[q] = fmaf(c, g[q], acc[q]);
    }
  }
  if (noise_scale != 0.0f) {
    const Normals4 z = noise_group(seed, layer, g4);
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[q] = fmaf(noise_scale, z.z[q], acc[q]);
  }
  if (vec) {
    *(float4*)(out + e) = make_float4(acc[0], acc[1], acc[2], acc[3]);
  } else {
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if (e + q < S) out[e + q] = acc[q];
  }
}

// out[e] = (ADD ? out[e] : 0) + scale * z[e]: the noise step alone (second pass of the two-pass schedule,
// and the stand-alone field for checks).
template <bool ADD>
__global__ __launch_bounds__(256) void noise_kernel(float* __restrict__ out, size_t S, float scale, uint64_t seed, uint32_t layer) {
  const size_t g = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (4 * g >= S) return;
  const Normals4 z = noise_group(seed, layer, g);
  if (4 * g + 3 < S && (((uintptr_t)out) & 15) == 0) {
    float4* p = (float4*)out + g;
    float4 v = ADD ? *p : make_float4(0.f, 0.f, 0.f, 0.f);
    v.x = fmaf(scale, z.z[0], v.x);
    v.y = fmaf(scale, z.z[1], v.y);
    v.z = fmaf(scale, z.z[2], v.z);
    v.w = fmaf(scale, z.z[3], v.w);
    *p = v;
  } else {
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if (4 * g + q < S) out[4 * g + q] = fmaf(scale, z.z[q], ADD ? out[4 * g + q] : 0.0f);
  }
}

// z = BoxMuller(words): the uniform -> normal map on caller-supplied words, for checking edge cases
// (extreme uniforms, quadrant boundaries) that a keyed field reaches only by chance.
__global__ __launch_bounds__(256) void box_muller_kernel(const uint32_t* __restrict__ words, size_t n_groups, float* __restrict__ z) {
  const size_t g = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (g >= n_groups) return;
  Words4 w;
#pragma unroll
  for (int q = 0; q < 4; ++q) w.w[q] = words[4 * g + q];
  const Normals4 o = box_muller4(w);
#pragma unroll
  for (int q = 0; q < 4; ++q) z[4 * g + q] = o.z[q];
}

}  // namespace flashdp
