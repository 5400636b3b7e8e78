// ae_philox.h — the counter-based generator and the u32 -> normal map, shared by the kernels that draw
// channel noise or message bits (device code only).
//
// Counter layout: key = (seed_lo, seed_hi); counter = (sample_lo, sample_hi, quad, stream) with `sample` the
// global sample index, `quad` = element index / 4 in (c,h,w) order, stream 0 = channel noise, 1 = message
// bits.  The u32 -> normal map is a fixed sequence of correctly rounded binary32 operations (explicit
// round-to-nearest intrinsics, never contracted; sqrtf correctly rounded by the build flags), so the noise
// tensor is reproducible bit for bit.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ae {

struct U4 { uint32_t x, y, z, w; };

__device__ __forceinline__ U4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                            uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return U4{c0, c1, c2, c3};
}

// ln(u) for u in [2^-33, 1]: u = m 2^e, m in [sqrt(1/2), sqrt(2)); ln(1+f) = f + f^2 Q(f)
__device__ __forceinline__ float ln_unit(float u) {
  const uint32_t bits = __float_as_uint(u);
  int e = (int)(bits >> 23) - 127;
  const uint32_t mant = bits & 0x007FFFFFu;
  float m = __uint_as_float(mant | 0x3F800000u);
  if (mant > 0x003504F3u) { m = __fmul_rn(m, 0.5f); e += 1; }
  const float f = __fadd_rn(m, -1.0f);
  float q = -0x1.383e66p-4f;
  q = __fmaf_rn(q, f, 0x1.084e9p-3f);
  q = __fmaf_rn(q, f, -0x1.0f3778p-3f);
  q = __fmaf_rn(q, f, 0x1.227084p-3f);
  q = __fmaf_rn(q, f, -0x1.542744p-3f);
  q = __fmaf_rn(q, f, 0x1.99a402p-3f);
  q = __fmaf_rn(q, f, -0x1.000428p-2f);
  q = __fmaf_rn(q, f, 0x1.55555p-2f);
  q = __fmaf_rn(q, f, -0x1.fffff8p-2f);
  const float f2 = __fmul_rn(f, f);
  const float l1 = __fmaf_rn(f2, q, f);
  return __fmaf_rn((float)e, 0x1.62e43p-1f, l1);
}

// Box-Muller on two words; see the header's description of model_noise.
__device__ __forceinline__ void gauss_pair(uint32_t w0, uint32_t w1, float& g0, float& g1) {
  const float u = __fmaf_rn(__uint2float_rn(w0), 0x1p-32f, 0x1p-33f);
  const float rho = sqrtf(__fmul_rn(-2.0f, ln_unit(u)));  // sqrtf is correctly rounded (-fhip-fp32-correctly-rounded-divide-sqrt); __fsqrt_rn is not
  const uint32_t quadrant = w1 >> 30;
  const float t = __fmul_rn(__uint2float_rn((w1 >> 6) & 0x00FFFFFFu), 0x1p-24f);
  const bool swap = t > 0.5f;
  const float r = swap ? __fadd_rn(1.0f, -t) : t;
  const float z = __fmul_rn(r, r);
  float sp = -0x1.2d9302p-8f;
  sp = __fmaf_rn(sp, z, 0x1.465e92p-4f);
  sp = __fmaf_rn(sp, z, -0x1.4abbbap-1f);
  sp = __fmaf_rn(sp, z, 0x1.921fb6p+0f);
  float s = __fmul_rn(r, sp);
  float c = 0x1.d99f54p-11f;
  c = __fmaf_rn(c, z, -0x1.55c4eap-6f);
  c = __fmaf_rn(c, z, 0x1.03c1dap-2f);
  c = __fmaf_rn(c, z, -0x1.3bd3ccp+0f);
  c = __fmaf_rn(c, z, 1.0f);
  if (swap) { const float tmp = s; s = c; c = tmp; }
  // rotate by quadrant * 90 degrees
  const float cq = (quadrant & 1u) ? s : c;
  const float sq = (quadrant & 1u) ? c : s;
  const float cs = (quadrant == 1u || quadrant == 2u) ? -cq : cq;
  const float ss = (quadrant >= 2u) ? -sq : sq;
  g0 = __fmul_rn(rho, cs);
  g1 = __fmul_rn(rho, ss);
}

__device__ __forceinline__ void normal_quad(uint64_t seed, uint64_t sample, uint32_t quad, float (&g)[4]) {
  const U4 w = philox4x32_10((uint32_t)sample, (uint32_t)(sample >> 32), quad, 0u, (uint32_t)seed,
                             (uint32_t)(seed >> 32));
  gauss_pair(w.x, w.y, g[0], g[1]);
  gauss_pair(w.z, w.w, g[2], g[3]);
}

}  // namespace ae
