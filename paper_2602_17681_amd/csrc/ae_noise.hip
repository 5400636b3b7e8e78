// ae_noise.hip — the channel: per-sample power normalisation fused with additive
// white Gaussian noise drawn from Philox4x32-10, its backward, and the
// Monte-Carlo bookkeeping kernels (message bits, error counts).
//
// Counter layout: key = (seed_lo, seed_hi); counter = (sample_lo, sample_hi,
// quad, stream) with `sample` the global sample index, `quad` = element index / 4
// in (c,h,w) order, stream 0 = channel noise, 1 = message bits.  The u32 -> normal
// map is a fixed sequence of correctly rounded binary32 operations (explicit
// round-to-nearest intrinsics, never contracted), so the noise tensor is
// reproducible bit for bit.
#include "ae_device.h"
#include "ae_internal.h"
#include "ae_philox.h"

namespace ae {
namespace {

constexpr int NT = 256;

template <typename T> __device__ __forceinline__ void ld4(const T* p, float (&v)[4]);
template <> __device__ __forceinline__ void ld4<float>(const float* p, float (&v)[4]) {
  const float4 t = *reinterpret_cast<const float4*>(p);
  v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
}
template <> __device__ __forceinline__ void ld4<bf16_t>(const bf16_t* p, float (&v)[4]) {
  const uint2 t = *reinterpret_cast<const uint2*>(p);
  v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xFFFF0000u);
  v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xFFFF0000u);
}
template <typename T> __device__ __forceinline__ void st4(T* p, const float (&v)[4]);
template <> __device__ __forceinline__ void st4<float>(float* p, const float (&v)[4]) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
}
template <> __device__ __forceinline__ void st4<bf16_t>(bf16_t* p, const float (&v)[4]) {
  uint2 t;
  t.x = (uint32_t)f32_to_bf16(v[0]) | ((uint32_t)f32_to_bf16(v[1]) << 16);
  t.y = (uint32_t)f32_to_bf16(v[2]) | ((uint32_t)f32_to_bf16(v[3]) << 16);
  *reinterpret_cast<uint2*>(p) = t;
}

// One wavefront per sample (TPS = 64) or, for small batches, one workgroup per sample (TPS = 256).  FLAT: the sample is a contiguous vector of n = C
// elements with n % 4 == 0 (16-byte / 8-byte vector access).  Otherwise the sample
// is stored [HW][C] and element i = c*HW + hw of the (c,h,w) order is gathered.
template <int TPS>
__device__ __forceinline__ float sample_sum(float v, float* sm) {
  if (TPS == 64) return wave_sum(v);
  return block_sum<NT>(v, sm);
}

// (z and y may be the same buffer: no __restrict__; every lane reads the elements it writes before it writes them)
template <typename T, bool FLAT, int TPS>
__global__ void k_pnorm_awgn(const T* z, T* y, int64_t batch, int C, int HW, int do_pnorm,
                             int do_awgn, float sigma, uint64_t seed, uint64_t first_sample) {
  __shared__ float sm[NT / 64 + 1];
  const int lane = threadIdx.x % TPS;
  const int64_t b = (int64_t)blockIdx.x * (NT / TPS) + (threadIdx.x / TPS);
  if (b >= batch) return;                        // whole wavefronts (TPS = 64) or never (TPS = 256: grid = batch)
  const int64_t n = (int64_t)C * HW;
  const T* zb = z + b * n;
  T* yb = y + b * n;
  const int64_t nquads = (n + 3) >> 2;
  float scale = 1.0f;
  if (do_pnorm) {
    float ss = 0.0f;
    if (FLAT) {
#pragma unroll 4
      for (int64_t q = lane; q < nquads; q += TPS) {
        float v[4];
        ld4<T>(zb + 4 * q, v);
        ss = fmaf(v[0], v[0], ss); ss = fmaf(v[1], v[1], ss); ss = fmaf(v[2], v[2], ss); ss = fmaf(v[3], v[3], ss);
      }
    } else {
#pragma unroll 8
      for (int64_t i = lane; i < n; i += TPS) { float v = Store<T>::ld(zb + i); ss = fmaf(v, v, ss); }
    }
    ss = sample_sum<TPS>(ss, sm);
    const float ms = ss / (float)n;
    scale = ms > 0.0f ? 1.0f / sqrtf(ms) : 0.0f;
  }
  const uint64_t sample = first_sample + (uint64_t)b;
  for (int64_t q = lane; q < nquads; q += TPS) {
    float g[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (do_awgn) {
      normal_quad(seed, sample, (uint32_t)q, g);
#pragma unroll
      for (int j = 0; j < 4; ++j) g[j] = __fmul_rn(sigma, g[j]);
    }
    if (FLAT) {
      float v[4];
      ld4<T>(zb + 4 * q, v);
#pragma unroll
      for (int j = 0; j < 4; ++j) v[j] = __fadd_rn(__fmul_rn(v[j], scale), g[j]);
      st4<T>(yb + 4 * q, v);
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int64_t i = 4 * q + j;
        if (i < n) {
          const int c = (int)(i / HW), hw = (int)(i % HW);
          const int64_t pos = (int64_t)hw * C + c;
          Store<T>::st(yb + pos, __fadd_rn(__fmul_rn(Store<T>::ld(zb + pos), scale), g[j]));
        }
      }
    }
  }
}

// Short flat latents (n = 4 L elements, L a power of two up to 32): L neighbouring lanes own one sample, one
// quad each, so a wavefront holds 64 / L samples and every lane of it loads, generates and stores; the sum
// of squares is reduced inside each group of L lanes with xor-shuffles (the same order for every sample,
// wherever it sits in the batch).  z and y may be the same buffer.
template <typename T, int L>
__global__ __launch_bounds__(NT) void k_pnorm_awgn_short(const T* z, T* y, int64_t batch, int do_pnorm, int do_awgn,
                                                         float sigma, uint64_t seed, uint64_t first_sample) {
  const int lane = threadIdx.x % L;
  const int64_t b = (int64_t)blockIdx.x * (NT / L) + (threadIdx.x / L);
  const bool valid = b < batch;                  // every lane stays for the shuffles
  float v[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  if (valid) ld4<T>(z + b * (4 * L) + 4 * lane, v);
  float scale = 1.0f;
  if (do_pnorm) {
    float ss = 0.0f;
    ss = fmaf(v[0], v[0], ss); ss = fmaf(v[1], v[1], ss); ss = fmaf(v[2], v[2], ss); ss = fmaf(v[3], v[3], ss);
#pragma unroll
    for (int off = L / 2; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
    const float ms = ss / (float)(4 * L);
    scale = ms > 0.0f ? 1.0f / sqrtf(ms) : 0.0f;
  }
  float g[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  if (do_awgn) {
    normal_quad(seed, first_sample + (uint64_t)b, (uint32_t)lane, g);
#pragma unroll
    for (int j = 0; j < 4; ++j) g[j] = __fmul_rn(sigma, g[j]);
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) v[j] = __fadd_rn(__fmul_rn(v[j], scale), g[j]);
  if (valid) st4<T>(y + b * (4 * L) + 4 * lane, v);
}

// x = z/r: dz = g/r - z * sum(g z) / (n r^3); elementwise in storage order
template <typename T, int TPS>
__global__ void k_pnorm_bwd(const T* __restrict__ z, const T* __restrict__ g, T* __restrict__ dz, int64_t batch,
                            int64_t n) {
  __shared__ float sm[NT / 64 + 1];
  const int lane = threadIdx.x % TPS;
  const int64_t b = (int64_t)blockIdx.x * (NT / TPS) + (threadIdx.x / TPS);
  if (b >= batch) return;
  const T* zb = z + b * n;
  const T* gb = g + b * n;
  float szz = 0.0f, sgz = 0.0f;
#pragma unroll 8
  for (int64_t i = lane; i < n; i += TPS) {
    const float zv = Store<T>::ld(zb + i), gv = Store<T>::ld(gb + i);
    szz = fmaf(zv, zv, szz);
    sgz = fmaf(gv, zv, sgz);
  }
  szz = sample_sum<TPS>(szz, sm);
  sgz = sample_sum<TPS>(sgz, sm);
  const float ms = szz / (float)n;
  float inv_r = 0.0f, coef = 0.0f;
  if (ms > 0.0f) {
    inv_r = 1.0f / sqrtf(ms);
    coef = sgz / (float)n * inv_r * inv_r * inv_r;
  }
#pragma unroll 8
  for (int64_t i = lane; i < n; i += TPS) {
    const float zv = Store<T>::ld(zb + i), gv = Store<T>::ld(gb + i);
    Store<T>::st(dz + b * n + i, gv * inv_r - zv * coef);
  }
}

__global__ void k_noise(uint64_t seed, uint64_t first_sample, int64_t batch, int64_t n, float* __restrict__ out) {
  const int64_t nquads = (n + 3) >> 2;
  const int64_t total = batch * nquads;
  for (int64_t it = (int64_t)blockIdx.x * NT + threadIdx.x; it < total; it += (int64_t)gridDim.x * NT) {
    const int64_t b = it / nquads, q = it % nquads;
    float g[4];
    normal_quad(seed, first_sample + (uint64_t)b, (uint32_t)q, g);
    for (int j = 0; j < 4; ++j)
      if (4 * q + j < n) out[b * n + 4 * q + j] = g[j];
  }
}

__global__ void k_gen_bits(uint64_t seed, uint64_t first_sample, int64_t batch, int k, float* __restrict__ x) {
  const int64_t total = batch * k;
  for (int64_t it = (int64_t)blockIdx.x * NT + threadIdx.x; it < total; it += (int64_t)gridDim.x * NT) {
    const int64_t b = it / k;
    const int j = (int)(it % k);
    const uint64_t sample = first_sample + (uint64_t)b;
    const U4 w = philox4x32_10((uint32_t)sample, (uint32_t)(sample >> 32), (uint32_t)(j >> 7), 1u, (uint32_t)seed,
                               (uint32_t)(seed >> 32));
    const int wi = (j >> 5) & 3;
    const uint32_t word = wi == 0 ? w.x : (wi == 1 ? w.y : (wi == 2 ? w.z : w.w));
    x[it] = ((word >> (j & 31)) & 1u) ? 1.0f : -1.0f;
  }
}

__global__ void k_count_errors(const float* __restrict__ y, const float* __restrict__ x, int64_t batch, int k,
                               unsigned long long* bit_err, unsigned long long* blk_err) {
  __shared__ float sm[NT / 64 + 1];
  float be = 0.0f, ke = 0.0f;  // counts per thread are small integers: exact in binary32
  const int64_t b = (int64_t)blockIdx.x * NT + threadIdx.x;
  if (b < batch) {
    int wrong = 0;
    for (int j = 0; j < k; ++j) wrong += ((y[b * k + j] > 0.5f) != (x[b * k + j] > 0.0f)) ? 1 : 0;
    be = (float)wrong;
    ke = wrong ? 1.0f : 0.0f;
  }
  be = block_sum<NT>(be, sm);  // at most 256*k < 2^24 when k < 65536
  ke = block_sum<NT>(ke, sm);
  if (threadIdx.x == 0) {
    if (be > 0.0f) atomicAdd(bit_err, (unsigned long long)be);
    if (ke > 0.0f) atomicAdd(blk_err, (unsigned long long)ke);
  }
}

inline int grid_for(int64_t items, int cap) {
  int64_t g = (items + NT - 1) / NT;
  if (g < 1) g = 1;
  if (g > cap) g = cap;
  return (int)g;
}

}  // namespace

// small batches of long vectors get a whole workgroup per sample
static bool block_per_sample(int64_t batch, int64_t n) { return batch < 1024 && n >= 1024; }

int launch_pnorm_awgn(const void* z, void* y, int64_t batch, int c, int hw, int dtype, int do_pnorm, int do_awgn,
                      float sigma, uint64_t seed, uint64_t first_sample, hipStream_t s) {
  // a flat vector is a tensor with hw == 1 (or c == 1: then (c,h,w) order is storage order too)
  int C = c, HW = hw;
  if (C == 1) { C = HW; HW = 1; }
  const bool flat = HW == 1 && (C % 4 == 0);
  if (flat && C <= 128 && (C & (C - 1)) == 0) {
    // short latents: several samples per wavefront
    const int L = C / 4;
    const int64_t blocks = (batch + NT / L - 1) / (NT / L);
    if (blocks > 0x7FFFFFFF) return fail(AE_EINVAL, "pnorm_awgn: batch too large");
#define LAUNCH_S(T, LV)                                                                                              \
  hipLaunchKernelGGL((k_pnorm_awgn_short<T, LV>), dim3((unsigned)blocks), dim3(NT), 0, s, (const T*)z, (T*)y, batch, \
                     do_pnorm, do_awgn, sigma, seed, first_sample)
#define LAUNCH_SL(T)                                                                                 \
  switch (L) {                                                                                       \
    case 1: LAUNCH_S(T, 1); break;   case 2: LAUNCH_S(T, 2); break;   case 4: LAUNCH_S(T, 4); break;  \
    case 8: LAUNCH_S(T, 8); break;   case 16: LAUNCH_S(T, 16); break; default: LAUNCH_S(T, 32); break; \
  }
    if (dtype == AE_BF16) { LAUNCH_SL(bf16_t) } else { LAUNCH_SL(float) }
#undef LAUNCH_SL
#undef LAUNCH_S
    return launch_status("pnorm_awgn_short");
  }
  const bool wide = block_per_sample(batch, (int64_t)C * HW);
  const int64_t blocks = wide ? batch : (batch + NT / 64 - 1) / (NT / 64);
  if (blocks > 0x7FFFFFFF) return fail(AE_EINVAL, "pnorm_awgn: batch too large");
#define LAUNCH(T, F, TPSV)                                                                                          \
  hipLaunchKernelGGL((k_pnorm_awgn<T, F, TPSV>), dim3((unsigned)blocks), dim3(NT), 0, s, (const T*)z, (T*)y, batch, C, \
                     HW, do_pnorm, do_awgn, sigma, seed, first_sample)
#define LAUNCH_F(T, F) do { if (wide) LAUNCH(T, F, 256); else LAUNCH(T, F, 64); } while (0)
  if (dtype == AE_BF16) { if (flat) LAUNCH_F(bf16_t, true); else LAUNCH_F(bf16_t, false); }
  else { if (flat) LAUNCH_F(float, true); else LAUNCH_F(float, false); }
#undef LAUNCH_F
#undef LAUNCH
  return launch_status("pnorm_awgn");
}

int launch_pnorm_bwd(const void* z, const void* g, void* dz, int64_t batch, int64_t n, int dtype, hipStream_t s) {
  const bool wide = block_per_sample(batch, n);
  const int64_t blocks = wide ? batch : (batch + NT / 64 - 1) / (NT / 64);
#define LAUNCH(T, TPSV)                                                                                             \
  hipLaunchKernelGGL((k_pnorm_bwd<T, TPSV>), dim3((unsigned)blocks), dim3(NT), 0, s, (const T*)z, (const T*)g, (T*)dz, \
                     batch, n)
  if (dtype == AE_BF16) { if (wide) LAUNCH(bf16_t, 256); else LAUNCH(bf16_t, 64); }
  else { if (wide) LAUNCH(float, 256); else LAUNCH(float, 64); }
#undef LAUNCH
  return launch_status("pnorm_bwd");
}

int launch_noise(uint64_t seed, uint64_t first_sample, int64_t batch, int64_t n, float* out, hipStream_t s) {
  hipLaunchKernelGGL(k_noise, dim3(grid_for(batch * ((n + 3) / 4), 1 << 20)), dim3(NT), 0, s, seed, first_sample, batch,
                     n, out);
  return launch_status("noise");
}

int launch_gen_bits(uint64_t seed, uint64_t first_sample, int64_t batch, int k, float* x, hipStream_t s) {
  hipLaunchKernelGGL(k_gen_bits, dim3(grid_for(batch * k, 1 << 20)), dim3(NT), 0, s, seed, first_sample, batch, k, x);
  return launch_status("gen_bits");
}

int launch_count_errors(const float* y, const float* x, int64_t batch, int k, uint64_t* bit_err, uint64_t* blk_err,
                        hipStream_t s) {
  if (k >= 65536) return fail(AE_EINVAL, "count_errors: k must be below 65536");
  hipLaunchKernelGGL(k_count_errors, dim3((unsigned)((batch + NT - 1) / NT)), dim3(NT), 0, s, y, x, batch, k,
                     (unsigned long long*)bit_err, (unsigned long long*)blk_err);
  return launch_status("count_errors");
}

}  // namespace ae
