// ae_device.h — small device-side helpers: bfloat16 conversion, 16-byte vector
// access in either storage type, wavefront (64 lanes) and block reductions.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ae {

typedef uint16_t bf16_t;  // raw bfloat16 bit pattern

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float((uint32_t)b << 16); }

// round to nearest, ties to even: gfx950 has a hardware conversion (v_cvt_pk_bf16_f32),
// which the compiler selects for a float -> __bf16 cast
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  const __bf16 h = (__bf16)f;
  return __builtin_bit_cast(bf16_t, h);
}

template <typename T> struct Store;
template <> struct Store<float> {
  static constexpr int VEC = 4;  // elements per 16 bytes
  static __device__ __forceinline__ float ld(const float* p) { return *p; }
  static __device__ __forceinline__ void st(float* p, float v) { *p = v; }
  static __device__ __forceinline__ void ldv(const float* p, float (&v)[4]) {
    float4 t = *reinterpret_cast<const float4*>(p);
    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
  }
  static __device__ __forceinline__ void stv(float* p, const float (&v)[4]) {
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  }
};
template <> struct Store<bf16_t> {
  static constexpr int VEC = 8;
  static __device__ __forceinline__ float ld(const bf16_t* p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void st(bf16_t* p, float v) { *p = f32_to_bf16(v); }
  static __device__ __forceinline__ void ldv(const bf16_t* p, float (&v)[8]) {
    uint4 t = *reinterpret_cast<const uint4*>(p);
    uint32_t w[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = __uint_as_float(w[i] << 16);
      v[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
    }
  }
  static __device__ __forceinline__ void stv(bf16_t* p, const float (&v)[8]) {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = (uint32_t)f32_to_bf16(v[2 * i]) | ((uint32_t)f32_to_bf16(v[2 * i + 1]) << 16);
    *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[2], w[3]);
  }
};

// value as it reads back after being stored in T
template <typename T> __device__ __forceinline__ float round_to_storage(float v);
template <> __device__ __forceinline__ float round_to_storage<float>(float v) { return v; }
template <> __device__ __forceinline__ float round_to_storage<bf16_t>(float v) { return bf16_to_f32(f32_to_bf16(v)); }

// Sum over the 64 lanes of a wavefront; every lane receives the total.
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// Sum over a block of NT threads (NT a multiple of 64, at most 1024); result valid in every thread.
template <int NT, typename F>
__device__ __forceinline__ F block_sum(F v, F* smem /* NT/64 + 1 entries */) {
  v = wave_sum(v);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  __syncthreads();
  if (lane == 0) smem[wave] = v;
  __syncthreads();
  if (threadIdx.x == 0) {
    F t = smem[0];
    for (int i = 1; i < NT / 64; ++i) t += smem[i];
    smem[NT / 64] = t;
  }
  __syncthreads();
  return smem[NT / 64];
}

__device__ __forceinline__ float apply_act(float v, int act) {
  if (act == 1) return v > 0.0f ? v : 0.0f;
  if (act == 2) return 1.0f / (1.0f + __expf(-v));
  return v;
}

// ---- MX block quantisation (the paper's Eq. 1) with FP4 E2M1 elements, shared by the stand-alone kernel
// and the GEMM epilogue that quantises its output ----
// scale exponent of a block from its largest magnitude (> 0): floor(log2 amax) - r_max (r_max = 2 for FP4 E2M1),
// clamped to the E8M0 range
__device__ __forceinline__ int mx_scale_exp(float amax, int r_max = 2) {
  int k = ilogbf(amax) - r_max;                  // subnormal maxima included
  k = k < -127 ? -127 : k;
  return k > 127 ? 127 : k;
}
// s * Q_e(v / s) for s = 2^k: nearest E2M1 magnitude, ties to even, saturating at 6
__device__ __forceinline__ float mx_quant_e2m1(float v, float inv_s, float s) {
  const float y = v * inv_s;                     // exact (power of two), |y| < 8
  const float a = fabsf(y);
  float r = a < 2.0f ? rintf(a * 2.0f) * 0.5f : (a < 4.0f ? rintf(a) : rintf(a * 0.5f) * 2.0f);
  r = fminf(r, 6.0f);
  return copysignf(r, y) * s;                    // at most two significant bits times a power of two: exact
}

// Other element formats under the same block scale.  MX_FP8: FP8 E4M3 of the OCP 8-bit floating point specification
// (subnormal spacing 2^-9 below 2^-6, three mantissa bits above, largest value 448, r_max = 8).  MX_INT4: the integer
// element the paper evaluates is not a standard format; reading: magnitudes k/4, k = 0..7, r_max = 0, saturating at 1.75.
enum { MX_FP4 = 0, MX_INT4 = 1, MX_FP8 = 2 };
template <int FMT> struct MxFormat;
template <> struct MxFormat<MX_FP4> {
  static constexpr int r_max = 2;
  static __device__ __forceinline__ float quant(float v, float inv_s, float s) { return mx_quant_e2m1(v, inv_s, s); }
};
template <> struct MxFormat<MX_INT4> {
  static constexpr int r_max = 0;
  static __device__ __forceinline__ float quant(float v, float inv_s, float s) {
    const float y = v * inv_s;                   // exact, |y| < 2
    return copysignf(fminf(rintf(fabsf(y) * 4.0f), 7.0f) * 0.25f, y) * s;
  }
};
template <> struct MxFormat<MX_FP8> {
  static constexpr int r_max = 8;
  static __device__ __forceinline__ float quant(float v, float inv_s, float s) {
    const float y = v * inv_s;                   // exact, |y| < 512
    const float a = fabsf(y);
    // normal range: round the binary32 mantissa to its three leading bits, to nearest, ties to even (a carry runs
    // into the exponent, as it should); below 2^-6 the format's subnormals have the fixed spacing 2^-9
    const uint32_t b = __float_as_uint(a);
    const float rn = __uint_as_float((b + 0x7FFFFu + ((b >> 20) & 1u)) & 0xFFF00000u);
    const float rs = rintf(a * 512.0f) * 0.001953125f;
    const float r = a < 0.015625f ? rs : rn;
    return copysignf(fminf(r, 448.0f), y) * s;
  }
};

}  // namespace ae
