// ae_mx.hip — the MX block quantiser Q(x) of the paper's Section "MX quantization", Eq. (1):
//   per block of B consecutive elements of a row:  s = 2^(floor(log2(max_j |x_j|)) - r_max),
//   Q(x)_j = s * Q_e(x_j / s),
// with Q_e the FP4 E2M1 element quantiser (magnitudes 0, 0.5, 1, 1.5, 2, 3, 4, 6; r_max = 2).
// Readings where the paper is silent: Q_e rounds to nearest, ties to the even code, saturating at
// +-6; an all-zero block gives zeros; the scale exponent is clamped to the E8M0 range [-127, 127].
//
// The operation is one read and one write of the tensor (HBM-bound).  Every step is exact in
// binary32 (scaling by powers of two; rounding to a grid of at most two significant bits), so
// the result does not depend on the order of anything and is compared bit for bit.
#include <hip/hip_runtime.h>

#include "ae_device.h"
#include "ae_internal.h"

namespace ae {
namespace {

constexpr int NT = 256;

// scale exponent of a block from its largest magnitude (> 0)
__device__ __forceinline__ int mx_scale_exp(float amax) {
  int k = ilogbf(amax) - 2;                      // floor(log2 amax) - r_max, subnormal maxima included
  k = k < -127 ? -127 : k;
  return k > 127 ? 127 : k;
}

// s * Q_e(v / s) for s = 2^k: nearest E2M1 magnitude, ties to even, saturating
__device__ __forceinline__ float mx_quant_e2m1(float v, float inv_s, float s) {
  const float y = v * inv_s;                     // exact (power of two), |y| < 8
  const float a = fabsf(y);
  float r = a < 2.0f ? rintf(a * 2.0f) * 0.5f : (a < 4.0f ? rintf(a) : rintf(a * 0.5f) * 2.0f);
  r = fminf(r, 6.0f);
  return copysignf(r, y) * s;                    // at most two significant bits times a power of two: exact
}

// Vector path: a lane owns 16 bytes (V elements); the LPB = B / V lanes of a block are neighbours
// in a wavefront and find the block maximum with xor-shuffles.
template <typename T>
__global__ __launch_bounds__(NT) void k_mx_quantize(const T* x, T* q, int64_t nchunks, int lpb) {   // q may be x
  constexpr int V = Store<T>::VEC;
  const int64_t span = (int64_t)gridDim.x * NT;
  const int64_t rounds = (nchunks + span - 1) / span;       // every lane of every wave runs every round: the shuffles need them
  for (int64_t it = 0; it < rounds; ++it) {
    const int64_t c = it * span + (int64_t)blockIdx.x * NT + threadIdx.x;
    const bool valid = c < nchunks;
    float v[V];
    if (valid) Store<T>::ldv(x + c * V, v);
    else {
#pragma unroll
      for (int j = 0; j < V; ++j) v[j] = 0.0f;
    }
    float amax = 0.0f;
#pragma unroll
    for (int j = 0; j < V; ++j) amax = fmaxf(amax, fabsf(v[j]));
    for (int off = 1; off < lpb; off <<= 1) amax = fmaxf(amax, __shfl_xor(amax, off, 64));
    float o[V];
    if (amax > 0.0f) {
      const int k = mx_scale_exp(amax);
      const float s = ldexpf(1.0f, k), inv_s = ldexpf(1.0f, -k);
#pragma unroll
      for (int j = 0; j < V; ++j) o[j] = mx_quant_e2m1(v[j], inv_s, s);
    } else {
#pragma unroll
      for (int j = 0; j < V; ++j) o[j] = 0.0f;
    }
    if (valid) Store<T>::stv(q + c * V, o);
  }
}

// Any other block size or alignment: one thread per block, two passes over its elements.
template <typename T>
__global__ void k_mx_quantize_generic(const T* x, T* q, int64_t nblocks, int block) {
  for (int64_t b = (int64_t)blockIdx.x * NT + threadIdx.x; b < nblocks; b += (int64_t)gridDim.x * NT) {
    const T* xb = x + b * block;
    T* qb = q + b * block;
    float amax = 0.0f;
    for (int j = 0; j < block; ++j) amax = fmaxf(amax, fabsf(Store<T>::ld(xb + j)));
    if (amax > 0.0f) {
      const int k = mx_scale_exp(amax);
      const float s = ldexpf(1.0f, k), inv_s = ldexpf(1.0f, -k);
      for (int j = 0; j < block; ++j) Store<T>::st(qb + j, mx_quant_e2m1(Store<T>::ld(xb + j), inv_s, s));
    } else {
      for (int j = 0; j < block; ++j) Store<T>::st(qb + j, 0.0f);
    }
  }
}

template <typename T>
int launch_mx(const void* x, void* q, int64_t total, int block, hipStream_t s) {
  constexpr int V = Store<T>::VEC;
  const int lpb = block / V;
  const bool vec = block % V == 0 && lpb >= 1 && lpb <= 64 && (lpb & (lpb - 1)) == 0 &&
                   (((uintptr_t)x | (uintptr_t)q) & 15) == 0;
  if (vec) {
    const int64_t nchunks = total / V;
    int64_t g = (nchunks + NT - 1) / NT;
    if (g > 256 * 32) g = 256 * 32;                       // 32 workgroups per compute unit, then rounds
    hipLaunchKernelGGL((k_mx_quantize<T>), dim3((unsigned)g), dim3(NT), 0, s, (const T*)x, (T*)q, nchunks, lpb);
  } else {
    const int64_t nblocks = total / block;
    int64_t g = (nblocks + NT - 1) / NT;
    if (g > 65535) g = 65535;
    hipLaunchKernelGGL((k_mx_quantize_generic<T>), dim3((unsigned)g), dim3(NT), 0, s, (const T*)x, (T*)q, nblocks, block);
  }
  return launch_status("mx_quantize");
}

}  // namespace
}  // namespace ae

extern "C" int model_mx_quantize(const void* x, void* q, int64_t rows, int64_t d, int block, int dtype, void* stream) {
  using namespace ae;
  if (!x || !q) return fail(AE_EINVAL, "model_mx_quantize: null argument");
  if (rows < 0 || d <= 0 || block < 1 || d % block != 0) return fail(AE_EINVAL, "model_mx_quantize: d must be a positive multiple of block");
  if (dtype != AE_F32 && dtype != AE_BF16) return fail(AE_EINVAL, "model_mx_quantize: bad dtype");
  if (rows > ((int64_t)1 << 40) / d) return fail(AE_EINVAL, "model_mx_quantize: tensor too large");
  if (rows == 0) return AE_OK;
  hipStream_t s = (hipStream_t)stream;
  return dtype == AE_BF16 ? launch_mx<bf16_t>(x, q, rows * d, block, s) : launch_mx<float>(x, q, rows * d, block, s);
}
