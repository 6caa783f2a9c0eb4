// Counter-based Gaussian noise for the aggregation step of Algorithm 1
// (B_dW = sum_b B_G' + N(0, sigma^2 C^2 I)).  The paper names no generator; this is
// Philox4x32-10 (Salmon et al., SC'11) followed by Box-Muller on 24-bit uniforms,
// written so that fp32 device arithmetic lands within a few 1e-7 of the exact map.
//
// Plain inline functions, usable from device code and (for CPU-side checks of the
// arithmetic) from a host compiler: FLASHDP_HD expands to __host__ __device__ under hipcc.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define FLASHDP_HD __host__ __device__ __forceinline__
#else
#include <math.h>
#define FLASHDP_HD static inline
#endif

namespace flashdp {

struct Words4 { uint32_t w[4]; };
struct Normals4 { float z[4]; };

// Ten rounds of Philox4x32: two 32x32->64 multiplies per round, the high halves are
// xored with the neighbouring counter words and the round key; keys advance by the
// Weyl constants between rounds.
FLASHDP_HD Words4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1) {
  const uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#if defined(__HIPCC__)
#pragma unroll
#endif
  for (int r = 0; r < 10; ++r) {
    if (r > 0) { k0 += W0; k1 += W1; }
    const uint64_t p0 = (uint64_t)M0 * c0;
    const uint64_t p1 = (uint64_t)M1 * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = n0;
    c2 = n2;
  }
  Words4 o; o.w[0] = c0; o.w[1] = c1; o.w[2] = c2; o.w[3] = c3;
  return o;
}

// -2 ln u for u = (2k+1) / 2^25, k = r >> 8 (the 24-bit uniform with the half-step offset).
// u is written as 2^(e-25) * (1+f) with 1+f in [0.75, 1.5): f = (n - 2^e) / 2^e is an exact
// fp32 number because |n - 2^e| < 2^24, so there is no rounding before the logarithm and no
// cancellation as u -> 1 (there e = 25 and the result is -2 log1p(f) alone).
// log1p(f) = 2 atanh(s), s = f / (2 + f), |s| <= 0.2, odd series to s^11.
FLASHDP_HD float neg2_log_uniform24(uint32_t r) {
  const uint32_t n = ((r >> 8) << 1) | 1u;                    // odd, 1 <= n < 2^25
#if defined(__HIPCC__) && defined(__HIP_DEVICE_COMPILE__)
  int lead = 31 - __clz((int)n);
#else
  int lead = 31 - __builtin_clz(n);
#endif
  // 2^lead <= n < 2^(lead+1).  Use e = lead+1 when n >= 1.5 * 2^lead so that 1+f stays in [0.75, 1.5).
  const uint32_t three_half = 3u << (lead > 0 ? lead - 1 : 0);
  int e = lead + ((lead > 0 && n >= three_half) ? 1 : 0);
  const int32_t diff = (int32_t)n - (int32_t)(1u << e);       // |diff| < 2^24: exact in fp32
  // 2^-e as a float, built from its exponent field (e in 0..25)
  union { uint32_t u; float f; } sc; sc.u = (uint32_t)(127 - e) << 23;
  const float f = (float)diff * sc.f;
  const float s = f / (2.0f + f);
  const float s2 = s * s;
  float p = 1.0f / 11.0f;
  p = p * s2 + 1.0f / 9.0f;
  p = p * s2 + 1.0f / 7.0f;
  p = p * s2 + 1.0f / 5.0f;
  p = p * s2 + 1.0f / 3.0f;
  p = p * s2;                                                  // atanh(s)/s - 1
  const float log1pf_f = 2.0f * (s + s * p);
  const float ln2_hi = 0.693145751953125f;                     // 0x3f317200: 16 significant bits, (e-25)*ln2_hi exact
  const float ln2_lo = 1.42860676533018e-06f;
  const float ke = (float)(e - 25);
  const float lnu = (ke * ln2_hi) + (ke * ln2_lo + log1pf_f);
  return -2.0f * lnu;
}

// (cos, sin)(2 pi u) for the same u = n / 2^25.  The quadrant and the position inside it are
// split off in integers, folded to [0, pi/4], and evaluated by Taylor polynomials.
FLASHDP_HD void cos_sin_2pi_uniform24(uint32_t r, float* c_out, float* s_out) {
  const uint32_t n = ((r >> 8) << 1) | 1u;                    // angle = 2 pi n / 2^25
  const uint32_t q = n >> 23;                                  // quadrant 0..3
  uint32_t m = n & 0x7FFFFFu;                                  // position in the quadrant, /2^23, odd so never 0
  const bool fold = m > 0x400000u;                             // beyond pi/4: use the complementary angle
  if (fold) m = 0x800000u - m;
  const float x = (float)m * (1.5707963267948966f / 8388608.0f);   // in (0, pi/4]
  const float x2 = x * x;
  float sp = -1.0f / 39916800.0f;                              // -x^11/11!
  sp = sp * x2 + 1.0f / 362880.0f;
  sp = sp * x2 - 1.0f / 5040.0f;
  sp = sp * x2 + 1.0f / 120.0f;
  sp = sp * x2 - 1.0f / 6.0f;
  const float sn = x + x * (sp * x2);
  float cp = 1.0f / 3628800.0f * -1.0f;                        // -x^10/10!
  cp = cp * x2 + 1.0f / 40320.0f;
  cp = cp * x2 - 1.0f / 720.0f;
  cp = cp * x2 + 1.0f / 24.0f;
  cp = cp * x2 - 0.5f;
  const float cs = 1.0f + cp * x2;
  const float a = fold ? sn : cs;                              // cos of the in-quadrant angle
  const float b = fold ? cs : sn;                              // sin of the in-quadrant angle
  // rotate by q quarter turns
  float c, s;
  switch (q) {
    case 0: c = a; s = b; break;
    case 1: c = -b; s = a; break;
    case 2: c = -a; s = -b; break;
    default: c = b; s = -a; break;
  }
  *c_out = c;
  *s_out = s;
}

FLASHDP_HD float sqrt_f32(float x) {
#if defined(__HIPCC__) && defined(__HIP_DEVICE_COMPILE__)
  return __fsqrt_rn(x);
#else
  return sqrtf(x);
#endif
}

// Four standard normals from the four Philox words: (r0, r1) and (r2, r3) are (radius, angle) pairs.
FLASHDP_HD Normals4 box_muller4(const Words4& r) {
  Normals4 o;
  float c, s;
  float rho = sqrt_f32(neg2_log_uniform24(r.w[0]));
  cos_sin_2pi_uniform24(r.w[1], &c, &s);
  o.z[0] = rho * c;
  o.z[1] = rho * s;
  rho = sqrt_f32(neg2_log_uniform24(r.w[2]));
  cos_sin_2pi_uniform24(r.w[3], &c, &s);
  o.z[2] = rho * c;
  o.z[3] = rho * s;
  return o;
}

// The four normals of group g (elements 4g .. 4g+3) of the field keyed by (seed, layer).
FLASHDP_HD Normals4 noise_group(uint64_t seed, uint32_t layer, uint64_t g) {
  return box_muller4(philox4x32_10((uint32_t)g, (uint32_t)(g >> 32), layer, 0u,
                                   (uint32_t)seed, (uint32_t)(seed >> 32)));
}

}  // namespace flashdp
