// ae_fold.hip — folding affine transformations T(x) = A x + v into linear layers f(x) = W x + b and into an
// embedding table (the paper's appendix "Folding & Transformation Structure"):
//   x -> T_l(f(T_r^-1(x)))  has weights  W~ = A_l W A_r^-1  and bias  b~ = A_l b - W~ v_r + v_l,
// either side optional; a matrix smaller than the side it acts on is applied block-wise (the same p x p matrix on
// every group of p features: one transformation shared by the attention heads), its shift replicated.
//
// The products run on the matrix cores through the dense case of the implicit-GEMM kernel
// (y[m][n] = sum_k x[m][k] w[n][k]).  A right factor multiplies the contiguous K axis of W directly (W viewed as
// [out*in/q][q]); a left factor multiplies the contiguous axis of the transposed intermediate, so the left side costs
// two transposes (HBM-bound, 64 x 64 tiles through LDS).  The bias is one wavefront per output row.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include "ae_device.h"
#include "ae_internal.h"

namespace ae {
namespace {

// dst[c][r] = src[r][c]; 32 x 32 tiles, any sizes
template <typename T>
__global__ __launch_bounds__(256) void k_transpose(const T* __restrict__ src, int64_t rows, int64_t cols, T* __restrict__ dst) {
  __shared__ float tile[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  const int64_t r0 = (int64_t)blockIdx.y * 32, c0 = (int64_t)blockIdx.x * 32;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int64_t r = r0 + ty + 8 * j, c = c0 + tx;
    if (r < rows && c < cols) tile[ty + 8 * j][tx] = Store<T>::ld(src + r * cols + c);
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int64_t c = c0 + ty + 8 * j, r = r0 + tx;
    if (r < rows && c < cols) Store<T>::st(dst + c * rows + r, tile[tx][ty + 8 * j]);
  }
}

// 64 x 64 tiles, 16 bytes (8 bf16) or 32 bytes (8 fp32) per lane on both sides; rows % 64 == 0, cols % 64 == 0
template <typename T>
__global__ __launch_bounds__(256) void k_transpose64(const T* __restrict__ src, int64_t rows, int64_t cols, T* __restrict__ dst) {
  __shared__ float tile[64][65];
  const int64_t r0 = (int64_t)blockIdx.y * 64, c0 = (int64_t)blockIdx.x * 64;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int chunk = threadIdx.x + 256 * j, lr = chunk >> 3, lc = (chunk & 7) << 3;
    float v[8];
    if (sizeof(T) == 2) {
      Store<bf16_t>::ldv(reinterpret_cast<const bf16_t*>(src) + (r0 + lr) * cols + c0 + lc, v);
    } else {
      const float* p = reinterpret_cast<const float*>(src) + (r0 + lr) * cols + c0 + lc;
      const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
      v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    }
#pragma unroll
    for (int t = 0; t < 8; ++t) tile[lr][lc + t] = v[t];
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int chunk = threadIdx.x + 256 * j, lr = chunk >> 3, lc = (chunk & 7) << 3;   // output row c0 + lr, columns r0 + lc ..
    float v[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) v[t] = tile[lc + t][lr];
    if (sizeof(T) == 2) {
      Store<bf16_t>::stv(reinterpret_cast<bf16_t*>(dst) + (c0 + lr) * rows + r0 + lc, v);
    } else {
      float* p = reinterpret_cast<float*>(dst) + (c0 + lr) * rows + r0 + lc;
      *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
      *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
    }
  }
}

// b~[o] = (A_l b)[o] - sum_j W~[o][j] v_r[j mod q] + v_l[o mod p]; one wavefront per output row, four rows per workgroup
template <typename T>
__global__ __launch_bounds__(256) void k_fold_bias(const T* __restrict__ wt, const float* __restrict__ b, int64_t out, int64_t in,
                                                   const T* __restrict__ a_left, int p, const float* __restrict__ v_left,
                                                   const float* __restrict__ v_right, int q, float* __restrict__ b_out) {
  const int lane = threadIdx.x & 63;
  const int64_t o = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (o >= out) return;                                   // (whole wavefronts: no shuffle partner is lost)
  double acc = 0.0;
  if (a_left) {
    const int64_t g = o / p;
    const int r = (int)(o - g * p);
    if (b) {                                               // p is a multiple of 16: eight entries per lane and pass
      for (int k = lane * 8; k < p; k += 512) {
        float av[8];
        if (sizeof(T) == 2) {
          Store<bf16_t>::ldv(reinterpret_cast<const bf16_t*>(a_left) + (int64_t)r * p + k, av);
        } else {
          const float* pa = reinterpret_cast<const float*>(a_left) + (int64_t)r * p + k;
          const float4 a = *reinterpret_cast<const float4*>(pa), c = *reinterpret_cast<const float4*>(pa + 4);
          av[0] = a.x; av[1] = a.y; av[2] = a.z; av[3] = a.w; av[4] = c.x; av[5] = c.y; av[6] = c.z; av[7] = c.w;
        }
        const float* pb = b + g * p + k;
        float part = 0.0f;
#pragma unroll
        for (int t = 0; t < 8; ++t) part = fmaf(av[t], pb[t], part);
        acc += (double)part;
      }
    }
  } else if (b && lane == 0) {
    acc = (double)b[o];
  }
  if (v_right) {
    if ((in & 7) == 0 && (q & 7) == 0) {                   // eight entries (16 or 32 bytes) per lane and pass
      for (int64_t j = (int64_t)lane * 8; j < in; j += 512) {
        float wv[8];
        if (sizeof(T) == 2) {
          Store<bf16_t>::ldv(reinterpret_cast<const bf16_t*>(wt) + o * in + j, wv);
        } else {
          const float* pw = reinterpret_cast<const float*>(wt) + o * in + j;
          const float4 a = *reinterpret_cast<const float4*>(pw), c = *reinterpret_cast<const float4*>(pw + 4);
          wv[0] = a.x; wv[1] = a.y; wv[2] = a.z; wv[3] = a.w; wv[4] = c.x; wv[5] = c.y; wv[6] = c.z; wv[7] = c.w;
        }
        const float* pv = v_right + j % q;                 // a chunk of eight never straddles a group of q
        float part = 0.0f;
#pragma unroll
        for (int t = 0; t < 8; ++t) part = fmaf(wv[t], pv[t], part);
        acc -= (double)part;
      }
    } else {
      for (int64_t j = lane; j < in; j += 64) acc -= (double)Store<T>::ld(wt + o * in + j) * (double)v_right[j % q];
    }
  }
  acc = wave_sum(acc);
  if (lane == 0) b_out[o] = (float)(acc + (v_left ? (double)v_left[o % p] : 0.0));
}

template <typename T>
void launch_transpose(const void* src, int64_t rows, int64_t cols, void* dst, hipStream_t s) {
  if (rows % 64 == 0 && cols % 64 == 0)
    hipLaunchKernelGGL((k_transpose64<T>), dim3((unsigned)(cols / 64), (unsigned)(rows / 64)), dim3(256), 0, s, (const T*)src, rows, cols, (T*)dst);
  else
    hipLaunchKernelGGL((k_transpose<T>), dim3((unsigned)((cols + 31) / 32), (unsigned)((rows + 31) / 32)), dim3(256), 0, s, (const T*)src, rows, cols, (T*)dst);
}
void transpose(const void* src, int64_t rows, int64_t cols, void* dst, int dtype, hipStream_t s) {
  if (dtype == AE_BF16) launch_transpose<bf16_t>(src, rows, cols, dst, s);
  else launch_transpose<float>(src, rows, cols, dst, s);
}

// y[m][n] = sum_k x[m][k] w[n][k] (+ bias[n]): x [rows][k], w [n][k], y [rows][n]
ConvArgs product_args(const void* x, const void* w, const float* bias, void* y, int64_t rows, int64_t k, int64_t n, int dtype) {
  ConvArgs a;
  memset(&a, 0, sizeof(a));
  a.x = x; a.w = w; a.bias = bias; a.y = y;
  a.n = (int)rows; a.hc = a.wc = 1; a.cin = (int)k; a.cout = (int)n; a.k = 1; a.up = 0; a.act = ACT_NONE; a.dtype = dtype;
  return a;
}

int check_side(const char* who, const char* side, int64_t full, int64_t blk, int dtype) {
  const int64_t step = 64 / (int64_t)dtype_size(dtype);
  if (blk < 32 || blk % step != 0 || full % blk != 0)
    return fail(AE_EINVAL, "%s: the %s matrix size must be a multiple of %d, at least 32, and divide the layer's side", who, side, (int)step);
  return AE_OK;
}

}  // namespace
}  // namespace ae

extern "C" int model_fold_workspace(int64_t out, int64_t in, int64_t p, int64_t q, int dtype, int64_t* bytes) {
  using namespace ae;
  if (!bytes || out <= 0 || in <= 0 || p < 0 || q < 0 || (dtype != AE_F32 && dtype != AE_BF16))
    return fail(AE_EINVAL, "model_fold_workspace: bad argument");
  if (out > (1 << 24) || in > (1 << 24) || out * in >= ((int64_t)1 << 30)) return fail(AE_EINVAL, "model_fold_workspace: layer too large");
  const int64_t es = (int64_t)dtype_size(dtype);
  *bytes = (q * q + 3 * out * in) * es + 1024;
  return AE_OK;
}

extern "C" int model_fold_linear(const void* w, const float* b, int64_t out, int64_t in, const void* a_left, int64_t p,
                                 const float* v_left, const void* a_right_inv, int64_t q, const float* v_right, int dtype,
                                 void* w_out, float* b_out, void* workspace, void* stream) {
  using namespace ae;
  if (!w || !w_out || !b_out || !workspace) return fail(AE_EINVAL, "model_fold_linear: null argument");
  if (dtype != AE_F32 && dtype != AE_BF16) return fail(AE_EINVAL, "model_fold_linear: bad dtype");
  if (out <= 0 || in <= 0 || out > (1 << 24) || in > (1 << 24) || out * in >= ((int64_t)1 << 30))
    return fail(AE_EINVAL, "model_fold_linear: bad layer size");
  if ((v_left && !a_left) || (v_right && !a_right_inv)) return fail(AE_EINVAL, "model_fold_linear: a shift needs its matrix");
  if (a_left) AE_TRY(check_side("model_fold_linear", "left", out, p, dtype));
  if (a_right_inv) AE_TRY(check_side("model_fold_linear", "right", in, q, dtype));
  if (in % (16 / (int64_t)dtype_size(dtype)) != 0) return fail(AE_EINVAL, "model_fold_linear: rows of w must be a multiple of 16 bytes");
  if (((reinterpret_cast<uintptr_t>(w) | reinterpret_cast<uintptr_t>(w_out) | reinterpret_cast<uintptr_t>(workspace) |
        reinterpret_cast<uintptr_t>(a_left) | reinterpret_cast<uintptr_t>(a_right_inv)) & 15) != 0)
    return fail(AE_EINVAL, "model_fold_linear: the matrices and the workspace must be 16-byte aligned");
  if (w == w_out) return fail(AE_EINVAL, "model_fold_linear: w_out must not be w");
  hipStream_t s = (hipStream_t)stream;
  const int64_t es = (int64_t)dtype_size(dtype);
  char* ws = reinterpret_cast<char*>(workspace);
  void* art = ws;                                      // (A_r^-1)^T         [q][q]
  void* z = ws + ((q * q * es + 255) / 256) * 256;     // W A_r^-1           [out][in]
  void* zt = (char*)z + out * in * es;                 // its transpose      [in][out]
  void* wtt = (char*)zt + out * in * es;               // (A_l W A_r^-1)^T   [in][out]
  const void* cur = w;                                 // [out][in]
  if (a_right_inv) {
    transpose(a_right_inv, q, q, art, dtype, s);
    AE_TRY(launch_status("fold_transpose"));
    void* dst = a_left ? z : w_out;
    const ConvArgs a = product_args(cur, art, nullptr, dst, out * (in / q), q, q, dtype);
    if (!conv_mfma_supported(a)) return fail(AE_EINVAL, "model_fold_linear: shape not supported by the matrix-core kernel");
    AE_TRY(launch_conv_mfma(a, s));
    cur = dst;
  }
  if (a_left) {
    transpose(cur, out, in, zt, dtype, s);
    AE_TRY(launch_status("fold_transpose"));
    const ConvArgs a = product_args(zt, a_left, nullptr, wtt, in * (out / p), p, p, dtype);
    if (!conv_mfma_supported(a)) return fail(AE_EINVAL, "model_fold_linear: shape not supported by the matrix-core kernel");
    AE_TRY(launch_conv_mfma(a, s));
    transpose(wtt, in, out, w_out, dtype, s);
    AE_TRY(launch_status("fold_transpose"));
  } else if (!a_right_inv) {
    AE_HIP(hipMemcpyAsync(w_out, w, out * in * es, hipMemcpyDeviceToDevice, s));
  }
  const unsigned grid = (unsigned)((out + 3) / 4);
  if (dtype == AE_BF16)
    hipLaunchKernelGGL((k_fold_bias<bf16_t>), dim3(grid), dim3(256), 0, s, (const bf16_t*)w_out, b, out, in, (const bf16_t*)a_left,
                       (int)p, v_left, v_right, (int)(q > 0 ? q : 1), b_out);
  else
    hipLaunchKernelGGL((k_fold_bias<float>), dim3(grid), dim3(256), 0, s, (const float*)w_out, b, out, in, (const float*)a_left,
                       (int)p, v_left, v_right, (int)(q > 0 ? q : 1), b_out);
  return launch_status("fold_bias");
}

extern "C" int model_fold_embedding(const void* e, int64_t vocab, int64_t d, const void* a, const float* v, int dtype,
                                    void* e_out, void* stream) {
  using namespace ae;
  if (!e || !a || !e_out) return fail(AE_EINVAL, "model_fold_embedding: null argument");
  if (dtype != AE_F32 && dtype != AE_BF16) return fail(AE_EINVAL, "model_fold_embedding: bad dtype");
  if (vocab <= 0 || d <= 0 || vocab >= 0x7FFFFFFF || d > (1 << 24)) return fail(AE_EINVAL, "model_fold_embedding: bad size");
  if (e == e_out) return fail(AE_EINVAL, "model_fold_embedding: e_out must not be e");
  const ConvArgs g = product_args(e, a, v, e_out, vocab, d, d, dtype);       // row j: A w_j + v
  if (!conv_mfma_supported(g)) return fail(AE_EINVAL, "model_fold_embedding: d must be a multiple of 32 (bf16) or 16 (fp32), at least 32, the table below 2 GiB");
  return launch_conv_mfma(g, (hipStream_t)stream);
}
