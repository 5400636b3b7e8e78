// ae_affine.hip — the LU parametrisation of a learnable invertible matrix (the paper's Section on learning
// affine transformations, Eq. 4):  A = P L (U + diag(s)),  L unit lower triangular, U strictly upper triangular,
// s = sign * exp(log_s) (the paper learns log|s| and keeps the signs), P a fixed permutation given as an index
// vector ((P M)[i] = M[perm[i]]); the gradients of the free parameters given dLoss/dA; and the volume regulariser
// in its practical form (sum_i log|s_i|)^2 (Eq. 6 and the paragraph after it).
//
// The three d x d x d products run on the matrix cores through the dense case of the implicit-GEMM kernel
// (y[m][n] = sum_k x[m][k] w[n][k], operands in the storage type, binary32 accumulation); small element-wise
// kernels materialise the triangular operands from the binary32 master parameters (transposed where the product
// needs it) and cut the products back to the triangles the parameters live on.
#include <hip/hip_runtime.h>
#include <string.h>

#include "ae_device.h"
#include "ae_internal.h"

namespace ae {
namespace {

struct LuSrc {
  const float* lp; const float* up; const float* log_s; const float* sign; const int* perm; const void* g;
  int d;
};
enum { LU_PL = 0, LU_UD = 1, LU_G = 2 };

// entry (r, c) of P L, of U + diag(s), or of G
template <typename T, int SRC>
__device__ __forceinline__ float lu_elem(const LuSrc& q, int r, int c) {
  if (SRC == LU_PL) {
    int row = q.perm[r];
    if ((unsigned)row >= (unsigned)q.d) row = r;                       // not a permutation: stay inside the arrays
    return c < row ? q.lp[(int64_t)row * q.d + c] : (c == row ? 1.0f : 0.0f);
  }
  if (SRC == LU_UD) return r < c ? q.up[(int64_t)r * q.d + c] : (r == c ? q.sign[c] * expf(q.log_s[c]) : 0.0f);
  return Store<T>::ld(reinterpret_cast<const T*>(q.g) + (int64_t)r * q.d + c);
}

// out = the matrix SRC (TR = false) or its transpose (TR = true), in the storage type; 32 x 32 tiles, d % 32 == 0
template <typename T, int SRC, bool TR>
__global__ __launch_bounds__(256) void k_lu_build(LuSrc q, T* __restrict__ out) {
  __shared__ float tile[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
  if (!TR) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int r = r0 + ty + 8 * j;
      Store<T>::st(out + (int64_t)r * q.d + c0 + tx, lu_elem<T, SRC>(q, r, c0 + tx));
    }
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j) tile[ty + 8 * j][tx] = lu_elem<T, SRC>(q, c0 + ty + 8 * j, r0 + tx);   // source row c, column r
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 4; ++j) Store<T>::st(out + (int64_t)(r0 + ty + 8 * j) * q.d + c0 + tx, tile[tx][ty + 8 * j]);
  }
}

// d/dU = strictly upper part of L^T P^T G, d/dlog_s = its diagonal times s
template <typename T>
__global__ __launch_bounds__(256) void k_lu_grad_upper(const T* __restrict__ dud, const float* __restrict__ log_s,
                                                       const float* __restrict__ sign, int d, float* __restrict__ dup,
                                                       float* __restrict__ dlog_s) {
  const int64_t n = (int64_t)d * d;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int k = (int)(i / d), c = (int)(i - (int64_t)k * d);
    const float v = Store<T>::ld(dud + i);
    dup[i] = c > k ? v : 0.0f;
    if (c == k) dlog_s[k] = v * (sign[k] * expf(log_s[k]));
  }
}

// d/dL: row i of G (U + diag s)^T belongs to row perm[i] of L; strictly lower part only
template <typename T>
__global__ __launch_bounds__(256) void k_lu_grad_lower(const T* __restrict__ dpl, const int* __restrict__ perm, int d,
                                                       float* __restrict__ dlp) {
  const int64_t n = (int64_t)d * d;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int r = (int)(i / d), c = (int)(i - (int64_t)r * d);
    int row = perm[r];
    if ((unsigned)row >= (unsigned)d) row = r;
    dlp[(int64_t)row * d + c] = c < row ? Store<T>::ld(dpl + i) : 0.0f;
  }
}

// (sum_i log|s_i|)^2 and its gradient 2 sum, one workgroup, fixed order
__global__ __launch_bounds__(256) void k_vol_penalty(const float* __restrict__ log_s, int d, float* __restrict__ value,
                                                     float* __restrict__ grad) {
  __shared__ double sm[256 / 64 + 1];
  __shared__ float total;
  double acc = 0.0;
  for (int i = threadIdx.x; i < d; i += 256) acc += (double)log_s[i];
  acc = block_sum<256>(acc, sm);
  if (threadIdx.x == 0) { total = (float)acc; *value = (float)(acc * acc); }
  __syncthreads();
  if (grad) for (int i = threadIdx.x; i < d; i += 256) grad[i] = 2.0f * total;
}

template <typename T, int SRC, bool TR>
void launch_build(const LuSrc& q, void* out, hipStream_t s) {
  hipLaunchKernelGGL((k_lu_build<T, SRC, TR>), dim3(q.d / 32, q.d / 32), dim3(256), 0, s, q, reinterpret_cast<T*>(out));
}

// y[m][n] = sum_k x[m][k] w[n][k], all d x d in the storage type
int dense_product(const void* x, const void* w, void* y, int d, int dtype, hipStream_t s) {
  ConvArgs a;
  memset(&a, 0, sizeof(a));
  a.x = x; a.w = w; a.bias = nullptr; a.y = y;
  a.n = d; a.hc = a.wc = 1; a.cin = a.cout = d; a.k = 1; a.up = 0; a.act = ACT_NONE; a.dtype = dtype;
  return launch_conv_mfma(a, s);
}

int check_lu_size(const char* who, int64_t d, int dtype) {
  if (dtype != AE_F32 && dtype != AE_BF16) return fail(AE_EINVAL, "%s: bad dtype", who);
  if (d < 32 || d % 32 != 0 || d > 16384) return fail(AE_EINVAL, "%s: d must be a multiple of 32 between 32 and 16384", who);
  return AE_OK;
}

}  // namespace
}  // namespace ae

extern "C" int model_lu_workspace(int64_t d, int dtype, int64_t* bytes) {
  using namespace ae;
  if (!bytes) return fail(AE_EINVAL, "model_lu_workspace: null argument");
  AE_TRY(check_lu_size("model_lu_workspace", d, dtype));
  *bytes = 5 * d * d * (int64_t)dtype_size(dtype);
  return AE_OK;
}

extern "C" int model_lu_compose(const float* lp, const float* up, const float* log_s, const float* sign_s, const int* perm,
                                int64_t d, int dtype, void* a_out, void* workspace, void* stream) {
  using namespace ae;
  if (!lp || !up || !log_s || !sign_s || !perm || !a_out || !workspace) return fail(AE_EINVAL, "model_lu_compose: null argument");
  AE_TRY(check_lu_size("model_lu_compose", d, dtype));
  hipStream_t s = (hipStream_t)stream;
  const int64_t mat = d * d * (int64_t)dtype_size(dtype);
  char* ws = reinterpret_cast<char*>(workspace);
  void* pl = ws;                // P L               [i][k]
  void* udt = ws + mat;         // (U + diag s)^T    [n][k]
  LuSrc q{lp, up, log_s, sign_s, perm, nullptr, (int)d};
  if (dtype == AE_BF16) { launch_build<bf16_t, LU_PL, false>(q, pl, s); launch_build<bf16_t, LU_UD, true>(q, udt, s); }
  else { launch_build<float, LU_PL, false>(q, pl, s); launch_build<float, LU_UD, true>(q, udt, s); }
  AE_TRY(launch_status("lu_build"));
  return dense_product(pl, udt, a_out, (int)d, dtype, s);
}

extern "C" int model_lu_backward(const void* g, const float* lp, const float* up, const float* log_s, const float* sign_s,
                                 const int* perm, int64_t d, int dtype, float* d_lp, float* d_up, float* d_log_s,
                                 void* workspace, void* stream) {
  using namespace ae;
  if (!g || !lp || !up || !log_s || !sign_s || !perm || !d_lp || !d_up || !d_log_s || !workspace)
    return fail(AE_EINVAL, "model_lu_backward: null argument");
  AE_TRY(check_lu_size("model_lu_backward", d, dtype));
  hipStream_t s = (hipStream_t)stream;
  const int64_t mat = d * d * (int64_t)dtype_size(dtype);
  char* ws = reinterpret_cast<char*>(workspace);
  void* plt = ws;               // (P L)^T           [k][i]
  void* gt = ws + mat;          // G^T               [n][i]
  void* ud = ws + 2 * mat;      // U + diag s        [k][n]
  void* dud = ws + 3 * mat;     // (P L)^T G         [k][n]
  void* dpl = ws + 4 * mat;     // G (U + diag s)^T  [i][k]
  LuSrc q{lp, up, log_s, sign_s, perm, g, (int)d};
  if (dtype == AE_BF16) {
    launch_build<bf16_t, LU_PL, true>(q, plt, s); launch_build<bf16_t, LU_G, true>(q, gt, s); launch_build<bf16_t, LU_UD, false>(q, ud, s);
  } else {
    launch_build<float, LU_PL, true>(q, plt, s); launch_build<float, LU_G, true>(q, gt, s); launch_build<float, LU_UD, false>(q, ud, s);
  }
  AE_TRY(launch_status("lu_build"));
  AE_TRY(dense_product(plt, gt, dud, (int)d, dtype, s));
  AE_TRY(dense_product(g, ud, dpl, (int)d, dtype, s));
  const int64_t n = d * d;
  const unsigned grid = (unsigned)((n + 256 * 8 - 1) / (256 * 8) < 4096 ? (n + 256 * 8 - 1) / (256 * 8) : 4096);
  if (dtype == AE_BF16) {
    hipLaunchKernelGGL((k_lu_grad_upper<bf16_t>), dim3(grid), dim3(256), 0, s, (const bf16_t*)dud, log_s, sign_s, (int)d, d_up, d_log_s);
    hipLaunchKernelGGL((k_lu_grad_lower<bf16_t>), dim3(grid), dim3(256), 0, s, (const bf16_t*)dpl, perm, (int)d, d_lp);
  } else {
    hipLaunchKernelGGL((k_lu_grad_upper<float>), dim3(grid), dim3(256), 0, s, (const float*)dud, log_s, sign_s, (int)d, d_up, d_log_s);
    hipLaunchKernelGGL((k_lu_grad_lower<float>), dim3(grid), dim3(256), 0, s, (const float*)dpl, perm, (int)d, d_lp);
  }
  return launch_status("lu_backward");
}

extern "C" int model_vol_penalty(const float* log_s, int64_t d, float* value, float* d_log_s, void* stream) {
  using namespace ae;
  if (!log_s || !value) return fail(AE_EINVAL, "model_vol_penalty: null argument");
  if (d < 1 || d > (1 << 24)) return fail(AE_EINVAL, "model_vol_penalty: bad size");
  hipLaunchKernelGGL(k_vol_penalty, dim3(1), dim3(256), 0, (hipStream_t)stream, log_s, (int)d, value, d_log_s);
  return launch_status("vol_penalty");
}
