// ae_calib.hip — measurement aid: what a loop of nothing but matrix-core instructions reaches on
// this device (the practical ceiling the convolution kernels are compared with, beside the
// nominal peak), optionally with the LDS fragment reads of a 128x64 wave tile in the loop, on
// operands of all ones or of random values (the shader clock under matrix-core load depends on
// how many operand bits toggle; the kernel reports the clock it ran at).
#include <hip/hip_runtime.h>

#include "ae_internal.h"

namespace ae {
namespace {

typedef __attribute__((ext_vector_type(4))) unsigned calib_uint4;
typedef __attribute__((ext_vector_type(8))) __bf16 calib_bf16x8;
typedef __attribute__((ext_vector_type(16))) float calib_floatx16;
typedef __attribute__((address_space(3))) char calib_lds_char;

// two bf16 values with random signs and mantissas and exponents of 0.5 .. 4 (a linear congruential step per call)
__device__ __forceinline__ unsigned calib_random_pair(unsigned& h) {
  h = h * 1664525u + 1013904223u;
  const unsigned lo = (h & 0x807fu) | ((126u + ((h >> 8) % 3u)) << 7);
  const unsigned hi = ((h >> 16) & 0x807fu) | ((126u + ((h >> 24) % 3u)) << 7);
  return lo | (hi << 16);
}

// READS: 16-byte LDS reads per lane and iteration (conflict-free: lane l reads 16 bytes at 16*l),
// issued before the eight independent 32x32x16 bf16 MFMAs and waited for after them.  Two
// wavefronts share each SIMD (the register budget is held to that), as in the convolution kernels.
// clk[0..1]: shader-clock and 100 MHz wall-clock ticks wavefront 0 of workgroup 0 spent in the kernel.
template <int READS>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void k_calib_mfma(float* __restrict__ out, int iters,
                                                                                           int random_data, long long* __restrict__ clk) {
  __shared__ __attribute__((aligned(16))) char smem[65536];
  const int tid = threadIdx.x, lane = tid & 63;
  const long long c0 = clock64(), w0 = wall_clock64();
  unsigned h = (unsigned)tid * 2654435761u + blockIdx.x * 40503u + 12345u;
  for (int i = tid; i < 65536 / 4; i += 256)
    reinterpret_cast<unsigned*>(smem)[i] = random_data ? calib_random_pair(h) : 0x3f803f80u;   // else bf16 1.0 pairs
  __syncthreads();
  calib_floatx16 acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[j][e] = 0.0f;
  calib_uint4 f[8];
#pragma unroll
  for (int r = 0; r < 8; ++r)
#pragma unroll
    for (int c = 0; c < 4; ++c) f[r][c] = random_data ? calib_random_pair(h) : 0x3f803f80u;
  [[maybe_unused]] unsigned base = (unsigned)(size_t)(calib_lds_char*)smem + (unsigned)((tid >> 6) * 8192 + lane * 16);
  for (int it = 0; it < iters; ++it) {
#if defined(__HIP_DEVICE_COMPILE__)
#pragma unroll
    for (int r = 0; r < READS; ++r) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(f[r]) : "v"(base), "n"(r * 1024));
#endif
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      const calib_bf16x8 a = __builtin_bit_cast(calib_bf16x8, f[(m + 4) & 7]);
      const calib_bf16x8 b = __builtin_bit_cast(calib_bf16x8, f[(m + 7) & 7]);
      acc[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[m], 0, 0, 0);
    }
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int r = 0; r < 8; ++r) asm volatile("" : "+v"(f[r]));
#endif
    base ^= 4096u;
  }
  float s = 0.0f;
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += acc[j][e];
  if (s == 12345.678f) out[tid] = s;   // keeps the accumulators alive; never true
  if (blockIdx.x == 0 && tid == 0) { clk[0] = clock64() - c0; clk[1] = wall_clock64() - w0; }
}

}  // namespace
}  // namespace ae

extern "C" int model_calibrate_mfma(int lds_reads, int random_data, int iters, float* scratch_dev, double* tflops,
                                    double* shader_mhz, void* stream) {
  using namespace ae;
  if (!scratch_dev || !tflops) return fail(AE_EINVAL, "model_calibrate_mfma: null argument");
  if ((reinterpret_cast<uintptr_t>(scratch_dev) & 7) != 0) return fail(AE_EINVAL, "model_calibrate_mfma: scratch_dev must be 8-byte aligned");
  if ((lds_reads != 0 && lds_reads != 6) || iters < 1 || iters > (1 << 20))
    return fail(AE_EINVAL, "model_calibrate_mfma: lds_reads is 0 or 6, iters 1..2^20");
  hipStream_t s = (hipStream_t)stream;
  hipDeviceProp_t prop;
  int dev = 0;
  AE_HIP(hipGetDevice(&dev));
  AE_HIP(hipGetDeviceProperties(&prop, dev));
  const int grid = prop.multiProcessorCount * 2;             // two workgroups (eight wavefronts) per compute unit
  hipEvent_t e0, e1;
  AE_HIP(hipEventCreate(&e0));
  AE_HIP(hipEventCreate(&e1));
  for (int pass = 0; pass < 2; ++pass) {                      // pass 0: warm-up
    if (pass == 1) AE_HIP(hipEventRecord(e0, s));
    long long* clk = reinterpret_cast<long long*>(scratch_dev);   // the first 16 bytes; the rest is the (never taken) result sink
    if (lds_reads == 0) hipLaunchKernelGGL((k_calib_mfma<0>), dim3(grid), dim3(256), 0, s, scratch_dev + 4, pass ? iters : 16, random_data != 0, clk);
    else hipLaunchKernelGGL((k_calib_mfma<6>), dim3(grid), dim3(256), 0, s, scratch_dev + 4, pass ? iters : 16, random_data != 0, clk);
  }
  AE_HIP(hipEventRecord(e1, s));
  AE_HIP(hipEventSynchronize(e1));
  float ms = 0.0f;
  AE_HIP(hipEventElapsedTime(&ms, e0, e1));
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  AE_TRY(launch_status("calibrate_mfma"));
  if (shader_mhz) {
    long long ticks[2] = {0, 0};
    AE_HIP(hipMemcpy(ticks, scratch_dev, sizeof(ticks), hipMemcpyDeviceToHost));
    *shader_mhz = ticks[1] > 0 ? 100.0 * (double)ticks[0] / (double)ticks[1] : 0.0;
  }
  // 8 MFMAs of 2*32*32*16 FLOP per wavefront and iteration, 4 wavefronts per workgroup
  *tflops = (double)grid * 4.0 * 8.0 * 32768.0 * (double)iters / ((double)ms * 1e9);
  return AE_OK;
}
