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
#include <string.h>

#include <mutex>

#include "ae_device.h"
#include "ae_internal.h"

namespace ae {
namespace {

constexpr int NT = 256;

// Vector path: a lane owns 16 bytes (V elements); the LPB = B / V lanes of a block are neighbours
// in a wavefront and find the block maximum with xor-shuffles.
template <typename T, int FMT>
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
      const int k = mx_scale_exp(amax, MxFormat<FMT>::r_max);
      const float s = ldexpf(1.0f, k), inv_s = ldexpf(1.0f, -k);
#pragma unroll
      for (int j = 0; j < V; ++j) o[j] = MxFormat<FMT>::quant(v[j], inv_s, s);
    } else {
#pragma unroll
      for (int j = 0; j < V; ++j) o[j] = 0.0f;
    }
    if (valid) Store<T>::stv(q + c * V, o);
  }
}

// Any other block size or alignment: one thread per block, two passes over its elements.
template <typename T, int FMT>
__global__ void k_mx_quantize_generic(const T* x, T* q, int64_t nblocks, int block) {
  for (int64_t b = (int64_t)blockIdx.x * NT + threadIdx.x; b < nblocks; b += (int64_t)gridDim.x * NT) {
    const T* xb = x + b * block;
    T* qb = q + b * block;
    float amax = 0.0f;
    for (int j = 0; j < block; ++j) amax = fmaxf(amax, fabsf(Store<T>::ld(xb + j)));
    if (amax > 0.0f) {
      const int k = mx_scale_exp(amax, MxFormat<FMT>::r_max);
      const float s = ldexpf(1.0f, k), inv_s = ldexpf(1.0f, -k);
      for (int j = 0; j < block; ++j) Store<T>::st(qb + j, MxFormat<FMT>::quant(Store<T>::ld(xb + j), inv_s, s));
    } else {
      for (int j = 0; j < block; ++j) Store<T>::st(qb + j, 0.0f);
    }
  }
}

template <typename T, int FMT>
int launch_mx(const void* x, void* q, int64_t total, int block, hipStream_t s) {
  constexpr int V = Store<T>::VEC;
  const int lpb = block / V;
  const bool vec = block % V == 0 && lpb >= 1 && lpb <= 64 && (lpb & (lpb - 1)) == 0 &&
                   (((uintptr_t)x | (uintptr_t)q) & 15) == 0;
  if (vec) {
    const int64_t nchunks = total / V;
    int64_t g = (nchunks + NT - 1) / NT;
    if (g > 256 * 32) g = 256 * 32;                       // 32 workgroups per compute unit, then rounds
    hipLaunchKernelGGL((k_mx_quantize<T, FMT>), dim3((unsigned)g), dim3(NT), 0, s, (const T*)x, (T*)q, nchunks, lpb);
  } else {
    const int64_t nblocks = total / block;
    int64_t g = (nblocks + NT - 1) / NT;
    if (g > 65535) g = 65535;
    hipLaunchKernelGGL((k_mx_quantize_generic<T, FMT>), dim3((unsigned)g), dim3(NT), 0, s, (const T*)x, (T*)q, nblocks, block);
  }
  return launch_status("mx_quantize");
}

// Block errors from the per-tile column sums of squares: eb[i] = 1/(rows*block) * sum over tiles and over the
// block's columns of partial[tile][1][column], added in a fixed order in double; one workgroup per block.
__global__ void k_mse_blocks(const float* __restrict__ partial, int tiles, int N, int block, double inv, float* __restrict__ eb) {
  __shared__ double sm[NT / 64 + 1];
  const int i = blockIdx.x;
  double acc = 0.0;
  const int64_t items = (int64_t)tiles * block;
  for (int64_t it = threadIdx.x; it < items; it += NT) {
    const int64_t t = it / block;
    const int j = (int)(it - t * block);
    acc += (double)partial[(t * 2 + 1) * N + (int64_t)i * block + j];
  }
  acc = block_sum<NT>(acc, sm);
  if (threadIdx.x == 0) eb[i] = (float)(acc * inv);
}
// E = mean of the block errors (one workgroup, fixed order)
__global__ void k_mse_total(const float* __restrict__ eb, int nb, float* __restrict__ e) {
  __shared__ double sm[NT / 64 + 1];
  double acc = 0.0;
  for (int i = threadIdx.x; i < nb; i += NT) acc += (double)eb[i];
  acc = block_sum<NT>(acc, sm);
  if (threadIdx.x == 0) *e = (float)(acc / (double)nb);
}

// Scratch of model_transform_mse_static: the per-tile column sums the residual epilogue hands to k_mse_blocks,
// in device memory the code object itself carries (no allocation at run time).  Every device the library
// runs on holds its own copy at its own address; the address is looked up once per device.
constexpr int64_t kStaticScratchBytes = 4 << 20;
static __device__ __align__(256) float g_static_scratch[kStaticScratchBytes / 4];
constexpr int kMaxDevices = 64;
float* g_static_scratch_ptr[kMaxDevices];      // per device, filled on that device's first call
std::mutex g_static_scratch_mutex;

int static_scratch(float** out) {
  int dev = -1;
  AE_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(AE_EHIP, "model_transform_mse_static: device index %d not supported", dev);
  std::lock_guard<std::mutex> lock(g_static_scratch_mutex);
  if (!g_static_scratch_ptr[dev]) {
    float* ptr = nullptr;
    AE_HIP(hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(g_static_scratch)));
    if (!ptr) return fail(AE_EHIP, "model_transform_mse_static: the scratch array has no device address");
    g_static_scratch_ptr[dev] = ptr;
  }
  *out = g_static_scratch_ptr[dev];
  return AE_OK;
}

// The constant term of the inverse map of Definition 3.1, T^-1(y) = A^-1 y - A^-1 v:  out[i] = -sum_j ainv[i][j] v[j].
// One wavefront per row; products and sums in double (d of them per row: nothing to gain from less).
template <typename T>
__global__ __launch_bounds__(NT) void k_inverse_shift(const T* __restrict__ ainv, const float* __restrict__ v, int d,
                                                      float* __restrict__ out) {
  const int row = blockIdx.x * (NT / 64) + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= d) return;
  const T* r = ainv + (int64_t)row * d;
  double acc = 0.0;
  for (int j = lane; j < d; j += 64) acc += (double)Store<T>::ld(r + j) * (double)v[j];
  acc = wave_sum(acc);
  if (lane == 0) out[row] = (float)(-acc);
}

int transform_tile_rows(int64_t rows, int64_t d, int dtype) {
  ConvArgs a;
  memset(&a, 0, sizeof(a));
  a.n = (int)rows; a.hc = a.wc = 1; a.cin = a.cout = (int)d; a.k = 1; a.dtype = dtype;
  return conv_partial_rows(a, true);
}

}  // namespace
}  // namespace ae

extern "C" int model_transform_mse_workspace(int64_t rows, int64_t d, int dtype, int64_t* bytes) {
  using namespace ae;
  if (!bytes || rows <= 0 || d <= 0 || (dtype != AE_F32 && dtype != AE_BF16)) return fail(AE_EINVAL, "model_transform_mse_workspace: bad argument");
  if (rows >= 0x7FFFFFFF || d >= 0x7FFFFFFF) return fail(AE_EINVAL, "model_transform_mse_workspace: tensor too large");
  const int64_t tiles = (rows + transform_tile_rows(rows, d, dtype) - 1) / transform_tile_rows(rows, d, dtype);
  *bytes = tiles * 2 * d * 4;
  return AE_OK;
}

extern "C" int model_transform_mse_elem(const void* x, const void* a_mat, const float* v, const void* a_inv, const float* inv_shift,
                                        int64_t rows, int64_t d, int block, int elem, int dtype, void* yq, void* workspace,
                                        float* e_blocks, float* e_total, void* stream);

extern "C" int model_transform_mse(const void* x, const void* a_mat, const float* v, const void* a_inv, const float* inv_shift,
                                   int64_t rows, int64_t d, int block, int dtype, void* yq, void* workspace,
                                   float* e_blocks, float* e_total, void* stream) {
  return model_transform_mse_elem(x, a_mat, v, a_inv, inv_shift, rows, d, block, 0, dtype, yq, workspace, e_blocks, e_total, stream);
}

extern "C" int model_transform_mse_elem(const void* x, const void* a_mat, const float* v, const void* a_inv, const float* inv_shift,
                                        int64_t rows, int64_t d, int block, int elem, int dtype, void* yq, void* workspace,
                                        float* e_blocks, float* e_total, void* stream) {
  using namespace ae;
  if (elem != MX_FP4 && elem != MX_INT4 && elem != MX_FP8) return fail(AE_EINVAL, "model_transform_mse: bad element format");
  if (!x || !a_mat || !v || !a_inv || !inv_shift || !yq || !workspace || !e_blocks || !e_total)
    return fail(AE_EINVAL, "model_transform_mse: null argument");
  if (dtype != AE_F32 && dtype != AE_BF16) return fail(AE_EINVAL, "model_transform_mse: bad dtype");
  if (rows <= 0 || d <= 0 || rows >= 0x7FFFFFFF || d >= 0x7FFFFFFF) return fail(AE_EINVAL, "model_transform_mse: bad size");
  const int epc = 16 / (int)dtype_size(dtype);
  if (block < epc || block > 64 || (block & (block - 1)) != 0)
    return fail(AE_EINVAL, "model_transform_mse: the fused epilogue quantises blocks of 8 (bf16) / 4 (fp32) to 64 columns, a power of two");
  hipStream_t s = (hipStream_t)stream;
  ConvArgs g1;
  memset(&g1, 0, sizeof(g1));
  g1.x = x; g1.w = a_mat; g1.bias = v; g1.y = yq;
  g1.n = (int)rows; g1.hc = g1.wc = 1; g1.cin = g1.cout = (int)d; g1.k = 1; g1.up = 0; g1.act = ACT_NONE; g1.dtype = dtype;
  g1.epi = CONV_EPI_MXQ;
  g1.mx_block = block;
  g1.mx_elem = elem;
  if (!conv_epi_usable(g1))
    return fail(AE_EINVAL, "model_transform_mse: d must be a multiple of 128 and rows a multiple of the row tile (256 bf16 / 128 fp32), tensors below 2 GiB");
  // T(x) = x A^T + v, rounded to the storage type and MX-quantised in the GEMM's epilogue
  AE_TRY(launch_conv_mfma(g1, s));
  // T^-1(Q(T x)) = yq A^-T - A^-1 v is never stored: the second GEMM's epilogue forms x - T^-1(...) and its column sums of squares
  ConvArgs g2 = g1;
  g2.x = yq; g2.w = a_inv; g2.bias = inv_shift; g2.y = nullptr;
  g2.epi = CONV_EPI_RESID; g2.resid = x; g2.partial = (float*)workspace;
  if (!conv_epi_usable(g2)) return fail(AE_EINVAL, "model_transform_mse: shape not supported");
  AE_TRY(launch_conv_mfma(g2, s));
  const int tile_rows = transform_tile_rows(rows, d, dtype);
  const int tiles = (int)(rows / tile_rows);
  const int nb = (int)(d / block);
  hipLaunchKernelGGL(k_mse_blocks, dim3(nb), dim3(NT), 0, s, (const float*)workspace, tiles, (int)d, block,
                     1.0 / ((double)rows * (double)block), e_blocks);
  hipLaunchKernelGGL(k_mse_total, dim3(1), dim3(NT), 0, s, e_blocks, nb, e_total);
  return launch_status("transform_mse");
}

extern "C" int model_inverse_shift(const void* a_inv, const float* v, int64_t d, int dtype, float* inv_shift, void* stream) {
  using namespace ae;
  if (!a_inv || !v || !inv_shift) return fail(AE_EINVAL, "model_inverse_shift: null argument");
  if (dtype != AE_F32 && dtype != AE_BF16) return fail(AE_EINVAL, "model_inverse_shift: bad dtype");
  if (d <= 0 || d > 46340) return fail(AE_EINVAL, "model_inverse_shift: d must be 1 .. 46340");
  const unsigned blocks = (unsigned)((d + NT / 64 - 1) / (NT / 64));
  if (dtype == AE_BF16)
    hipLaunchKernelGGL(k_inverse_shift<bf16_t>, dim3(blocks), dim3(NT), 0, (hipStream_t)stream, (const bf16_t*)a_inv, v, (int)d, inv_shift);
  else
    hipLaunchKernelGGL(k_inverse_shift<float>, dim3(blocks), dim3(NT), 0, (hipStream_t)stream, (const float*)a_inv, v, (int)d, inv_shift);
  return launch_status("inverse_shift");
}

extern "C" int model_transform_mse_static(const void* x, const void* a_mat, const float* v, const void* a_inv,
                                          const float* inv_shift, int64_t rows, int64_t d, int block, int elem, int dtype,
                                          void* yq, float* e_blocks, float* e_total, void* stream) {
  using namespace ae;
  int64_t need = 0;
  AE_TRY(model_transform_mse_workspace(rows, d, dtype, &need));
  if (need > kStaticScratchBytes)
    return fail(AE_EINVAL, "model_transform_mse_static: this shape needs %lld bytes of scratch, the built-in buffer holds %lld "
                "(use model_transform_mse with a workspace of your own)", (long long)need, (long long)kStaticScratchBytes);
  float* scratch = nullptr;
  AE_TRY(static_scratch(&scratch));
  // every float of the scratch that k_mse_blocks reads is written by the second product's epilogue first: nothing to clear
  return model_transform_mse_elem(x, a_mat, v, a_inv, inv_shift, rows, d, block, elem, dtype, yq, scratch, e_blocks, e_total, stream);
}

extern "C" int model_mx_quantize_elem(const void* x, void* q, int64_t rows, int64_t d, int block, int elem, int dtype, void* stream) {
  using namespace ae;
  if (!x || !q) return fail(AE_EINVAL, "model_mx_quantize: null argument");
  if (rows < 0 || d <= 0 || block < 1 || d % block != 0) return fail(AE_EINVAL, "model_mx_quantize: d must be a positive multiple of block");
  if (dtype != AE_F32 && dtype != AE_BF16) return fail(AE_EINVAL, "model_mx_quantize: bad dtype");
  if (elem != MX_FP4 && elem != MX_INT4 && elem != MX_FP8) return fail(AE_EINVAL, "model_mx_quantize: bad element format");
  if (rows > ((int64_t)1 << 40) / d) return fail(AE_EINVAL, "model_mx_quantize: tensor too large");
  if (rows == 0) return AE_OK;
  hipStream_t s = (hipStream_t)stream;
  const int64_t n = rows * d;
  if (dtype == AE_BF16) {
    if (elem == MX_FP4) return launch_mx<bf16_t, MX_FP4>(x, q, n, block, s);
    if (elem == MX_INT4) return launch_mx<bf16_t, MX_INT4>(x, q, n, block, s);
    return launch_mx<bf16_t, MX_FP8>(x, q, n, block, s);
  }
  if (elem == MX_FP4) return launch_mx<float, MX_FP4>(x, q, n, block, s);
  if (elem == MX_INT4) return launch_mx<float, MX_INT4>(x, q, n, block, s);
  return launch_mx<float, MX_FP8>(x, q, n, block, s);
}

extern "C" int model_mx_quantize(const void* x, void* q, int64_t rows, int64_t d, int block, int dtype, void* stream) {
  return model_mx_quantize_elem(x, q, rows, d, block, 0, dtype, stream);
}
