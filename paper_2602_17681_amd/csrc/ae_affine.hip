// ae_affine.hip — the LU parametrisation of a learnable invertible matrix (the paper's Section on learning
// affine transformations, Eq. 4):  A = P L (U + diag(s)),  L unit lower triangular, U strictly upper triangular,
// s = sign * exp(log_s) (the paper learns log|s| and keeps the signs), P a fixed permutation given as an index
// vector ((P M)[i] = M[perm[i]]); the gradients of the free parameters given dLoss/dA; and the volume regulariser
// in its practical form (sum_i log|s_i|)^2 (Eq. 6 and the paragraph after it).
//
// The three d x d x d products run on the matrix cores through the dense case of the implicit-GEMM kernel
// (y[m][n] = sum_k x[m][k] w[n][k], operands in the storage type, binary32 accumulation); small element-wise
// kernels materialise the triangular operands from the binary32 master parameters (transposed where the product
// needs it), apply the permutation to rows (of L (U + diag s) forward, of G backward), and cut the products back
// to the triangles the parameters live on.  Every product has a triangular operand and, backward, only a triangle
// of the result is wanted: the GEMM kernel walks only the K range of each tile that can hold non-zeros and skips
// the tiles nobody reads — a third of the multiply-adds of three dense products.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include <mutex>
#include "ae_device.h"
#include "ae_internal.h"

namespace ae {
namespace {

struct LuSrc {
  const float* lp; const float* up; const float* log_s; const float* sign; const int* inv_perm; const void* g;
  int d;
};
enum { LU_L = 0, LU_UD = 1, LU_B = 2 };

// entry (r, c) of L, of U + diag(s), or of B = P^T G (row r of B is row inv_perm[r] of G)
template <typename T, int SRC>
__device__ __forceinline__ float lu_elem(const LuSrc& q, int r, int c) {
  if (SRC == LU_L) return c < r ? q.lp[(int64_t)r * q.d + c] : (c == r ? 1.0f : 0.0f);
  if (SRC == LU_UD) return r < c ? q.up[(int64_t)r * q.d + c] : (r == c ? q.sign[c] * expf(q.log_s[c]) : 0.0f);
  return Store<T>::ld(reinterpret_cast<const T*>(q.g) + (int64_t)q.inv_perm[r] * q.d + c);
}

// eight consecutive entries of one row, to and from the storage type
template <typename T> __device__ __forceinline__ void load8(const T* p, float (&v)[8]);
template <> __device__ __forceinline__ void load8<bf16_t>(const bf16_t* p, float (&v)[8]) { Store<bf16_t>::ldv(p, v); }
template <> __device__ __forceinline__ void load8<float>(const float* p, float (&v)[8]) {
  const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
template <typename T> __device__ __forceinline__ void store8(T* p, const float (&v)[8]);
template <> __device__ __forceinline__ void store8<bf16_t>(bf16_t* p, const float (&v)[8]) { Store<bf16_t>::stv(p, v); }
template <> __device__ __forceinline__ void store8<float>(float* p, const float (&v)[8]) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}

// out = the transpose of the matrix SRC in the storage type: 64 x 64 tiles through LDS, eight entries per lane on both
// sides; source chunks that lie wholly in the zero triangle read nothing.  d % 64 == 0.
template <typename T, int SRC>
__global__ __launch_bounds__(256) void k_lu_build_transposed(LuSrc q, T* __restrict__ out) {
  __shared__ float tile[64][65];
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;           // output tile: rows r0.., columns c0..
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int chunk = threadIdx.x + 256 * j;
    const int sr = c0 + (chunk >> 3), sc0 = r0 + ((chunk & 7) << 3);   // source row (an output column), first source column
    float v[8];
    if (SRC == LU_B) {
      load8<T>(reinterpret_cast<const T*>(q.g) + (int64_t)q.inv_perm[sr] * q.d + sc0, v);
    } else if (SRC == LU_L ? sc0 + 7 < sr : sc0 > sr) {
      load8<float>((SRC == LU_L ? q.lp : q.up) + (int64_t)sr * q.d + sc0, v);
    } else if (SRC == LU_L ? sc0 > sr : sc0 + 7 < sr) {
#pragma unroll
      for (int t = 0; t < 8; ++t) v[t] = 0.0f;
    } else {
#pragma unroll
      for (int t = 0; t < 8; ++t) v[t] = lu_elem<T, SRC>(q, sr, sc0 + t);
    }
#pragma unroll
    for (int t = 0; t < 8; ++t) tile[chunk >> 3][((chunk & 7) << 3) + t] = v[t];
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int chunk = threadIdx.x + 256 * j;
    const int orow = chunk >> 3, oc0 = (chunk & 7) << 3;           // output row r0 + orow, columns c0 + oc0 ..
    float v[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) v[t] = tile[oc0 + t][orow];
    store8<T>(out + (int64_t)(r0 + orow) * q.d + c0 + oc0, v);
  }
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

// out = the matrix SRC, row by row, eight entries per lane; chunks that lie wholly in the zero triangle read nothing
template <typename T, int SRC>
__global__ __launch_bounds__(256) void k_lu_build_rows(LuSrc q, T* __restrict__ out) {
  const int cpr = q.d >> 3;
  const int64_t n = (int64_t)q.d * cpr;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int r = (int)(i / cpr), c0 = (int)(i - (int64_t)r * cpr) << 3;
    float v[8];
    if (SRC == LU_B) {
      load8<T>(reinterpret_cast<const T*>(q.g) + (int64_t)q.inv_perm[r] * q.d + c0, v);
    } else if (SRC == LU_L ? c0 + 7 < r : c0 > r) {
      load8<float>((SRC == LU_L ? q.lp : q.up) + (int64_t)r * q.d + c0, v);       // wholly inside the used triangle
    } else if (SRC == LU_L ? c0 > r : c0 + 7 < r) {
#pragma unroll
      for (int t = 0; t < 8; ++t) v[t] = 0.0f;
    } else {
#pragma unroll
      for (int t = 0; t < 8; ++t) v[t] = lu_elem<T, SRC>(q, r, c0 + t);           // the chunk that holds the diagonal
    }
    store8<T>(out + (int64_t)r * q.d + c0, v);
  }
}

// inv[i] = i, then inv[perm[i]] = i (two launches): entries of perm outside 0..d-1 are ignored, so every inv[r]
// stays inside 0..d-1 whatever perm holds
__global__ void k_lu_iota(int* __restrict__ inv, int d) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < d) inv[i] = i;
}
__global__ void k_lu_invert_perm(const int* __restrict__ perm, int* __restrict__ inv, int d) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < d && (unsigned)perm[i] < (unsigned)d) inv[perm[i]] = i;
}

// A[i][:] = Y[perm[i]][:], 16 bytes per lane (row bytes are a multiple of 64)
__global__ __launch_bounds__(256) void k_lu_permute_rows(const uint4* __restrict__ y, const int* __restrict__ perm, int d,
                                                         int chunks_per_row, uint4* __restrict__ a) {
  const int64_t n = (int64_t)d * chunks_per_row;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int r = (int)(i / chunks_per_row), c = (int)(i - (int64_t)r * chunks_per_row);
    int src = perm[r];
    if ((unsigned)src >= (unsigned)d) src = r;                        // not a permutation: stay inside the arrays
    a[i] = y[(int64_t)src * chunks_per_row + c];
  }
}

// d/dU = strictly upper part of L^T B, d/dlog_s = its diagonal times s  (tiles below the diagonal were never written:
// chunks wholly below it are not read)
template <typename T>
__global__ __launch_bounds__(256) void k_lu_grad_upper(const T* __restrict__ dud, const float* __restrict__ log_s,
                                                       const float* __restrict__ sign, int d, float* __restrict__ dup,
                                                       float* __restrict__ dlog_s) {
  const int cpr = d >> 3;
  const int64_t n = (int64_t)d * cpr;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int k = (int)(i / cpr), c0 = (int)(i - (int64_t)k * cpr) << 3;
    float v[8];
    if (c0 + 7 >= k) {
      load8<T>(dud + (int64_t)k * d + c0, v);
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        if (c0 + t == k) dlog_s[k] = v[t] * (sign[k] * expf(log_s[k]));
        if (c0 + t <= k) v[t] = 0.0f;
      }
    } else {
#pragma unroll
      for (int t = 0; t < 8; ++t) v[t] = 0.0f;
    }
    store8<float>(dup + (int64_t)k * d + c0, v);
  }
}

// d/dL = strictly lower part of B (U + diag s)^T  (tiles above the diagonal were never written: not read)
template <typename T>
__global__ __launch_bounds__(256) void k_lu_grad_lower(const T* __restrict__ dl, int d, float* __restrict__ dlp) {
  const int cpr = d >> 3;
  const int64_t n = (int64_t)d * cpr;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int r = (int)(i / cpr), c0 = (int)(i - (int64_t)r * cpr) << 3;
    float v[8];
    if (c0 < r) {
      load8<T>(dl + (int64_t)r * d + c0, v);
#pragma unroll
      for (int t = 0; t < 8; ++t) if (c0 + t >= r) v[t] = 0.0f;
    } else {
#pragma unroll
      for (int t = 0; t < 8; ++t) v[t] = 0.0f;
    }
    store8<float>(dlp + (int64_t)r * d + c0, v);
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

// ---- inverse of the parametrised matrix ---------------------------------------------------------------------
// A^-1 = (U + diag s)^-1 L^-1 P^T.  Both triangular inverses use the same blocked recursion on a LOWER triangular
// matrix M (L itself; (U + diag s)^T for the upper factor): 128 x 128 diagonal blocks are inverted by substitution,
// then neighbouring inverses X11, X22 of blocks of size b merge into the inverse of the 2b x 2b block,
//     [[X11, 0], [-X22 M21 X11, X22]].
// X and X^T live as full d x d binary32 matrices that start block diagonal and fill level by level; one level is
// two launches of the matrix-core kernel over ALL pairs at once (K-range modes CONV_TRI_PAIR_*) and a transposing copy:
//     T' = -(M21 X11)^T  into the upper blocks of a scratch matrix,   X21 = X22 T'^T  in place into X,
//     X21^T  into X^T.

// entry (r, c) of the lower triangular matrix: WHICH 0: L; 1: (U + diag s)^T.  Rows and columns past d belong to
// the identity block that pads the matrix to the working size of the recursion.
template <int WHICH>
__device__ __forceinline__ float tri_elem(const LuSrc& q, int r, int c) {
  if (c > r) return 0.0f;
  if (r >= q.d) return r == c ? 1.0f : 0.0f;
  if (WHICH == 0) return c < r ? q.lp[(int64_t)r * q.d + c] : 1.0f;
  return c < r ? q.up[(int64_t)c * q.d + r] : q.sign[c] * expf(q.log_s[c]);
}

// mneg = -M (full dp x dp), x = xt = 0: 32 x 32 tiles
template <int WHICH>
__global__ __launch_bounds__(256) void k_tri_prepare(LuSrc q, int dp, float* __restrict__ mneg, float* __restrict__ x, float* __restrict__ xt) {
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int r = r0 + ty + 8 * j, c = c0 + tx;
    const int64_t i = (int64_t)r * dp + c;
    // (U + diag s)^T is read along its columns: the tile is small enough for the cache to absorb the stride
    mneg[i] = -tri_elem<WHICH>(q, r, c);
    x[i] = 0.0f;
    xt[i] = 0.0f;
  }
}

// One merge level of the in-LDS recursion: for every pair p of neighbouring B x B diagonal blocks of the 128 x 128
// matrix, X21 = -X22 (M21 X11) into xb below the diagonal blocks.  64 / B pairs, 256 threads, each a TR x TC register
// tile of outputs (rows tr + (B/TR) i, columns tc + (B/TC) j: neighbouring threads read neighbouring LDS columns).
// X11 and X22 are lower triangular inside xb, whose other entries are zero, so the K ranges are cut per thread only:
// the first product starts at the thread's first column, the second ends at its last row.  Ends on a barrier.
template <int B, int TR, int TC>
__device__ __forceinline__ void tri128_merge(float (*mb)[129], float (*xb)[129], float* tb, int tid) {
  constexpr int PAIRS = 64 / B, TPP = 256 / PAIRS, TCN = B / TC, TRN = B / TR;
  static_assert(TRN * TCN == TPP, "one register tile per thread");
  const int p = tid / TPP, t = tid % TPP, tr = t / TCN, tc = t % TCN;
  const int o0 = 2 * p * B, o1 = o0 + B;             // first row / column of the pair's two diagonal blocks
  float* tp = tb + p * B * B;
  float acc[TR][TC];
#pragma unroll
  for (int i = 0; i < TR; ++i)
#pragma unroll
    for (int j = 0; j < TC; ++j) acc[i][j] = 0.0f;
#pragma unroll 4
  for (int k = tc; k < B; ++k) {                       // T = M21 X11:  X11[k][c] = 0 for k < c, and c >= tc
    float a[TR], x[TC];
#pragma unroll
    for (int i = 0; i < TR; ++i) a[i] = mb[o1 + tr + TRN * i][o0 + k];
#pragma unroll
    for (int j = 0; j < TC; ++j) x[j] = xb[o0 + k][o0 + tc + TCN * j];
#pragma unroll
    for (int i = 0; i < TR; ++i)
#pragma unroll
      for (int j = 0; j < TC; ++j) acc[i][j] = fmaf(a[i], x[j], acc[i][j]);
  }
#pragma unroll
  for (int i = 0; i < TR; ++i)
#pragma unroll
    for (int j = 0; j < TC; ++j) {
      tp[(tr + TRN * i) * B + tc + TCN * j] = acc[i][j];
      acc[i][j] = 0.0f;
    }
  __syncthreads();
  const int kend = tr + TRN * (TR - 1);                // X21 = -X22 T:  X22[r][k] = 0 for k > r, and r <= kend
#pragma unroll 4
  for (int k = 0; k <= kend; ++k) {
    float a[TR], x[TC];
#pragma unroll
    for (int i = 0; i < TR; ++i) a[i] = xb[o1 + tr + TRN * i][o1 + k];
#pragma unroll
    for (int j = 0; j < TC; ++j) x[j] = tp[k * B + tc + TCN * j];
#pragma unroll
    for (int i = 0; i < TR; ++i)
#pragma unroll
      for (int j = 0; j < TC; ++j) acc[i][j] = fmaf(a[i], x[j], acc[i][j]);
  }
#pragma unroll
  for (int i = 0; i < TR; ++i)
#pragma unroll
    for (int j = 0; j < TC; ++j) xb[o1 + tr + TRN * i][o0 + tc + TCN * j] = -acc[i][j];   // (below the diagonal blocks: nobody reads it in this pass)
  __syncthreads();
}

// xb = mb^-1 for a lower triangular 128 x 128 matrix in LDS (all 256 threads of the workgroup; xb must be zero on
// entry and both arrays visible to every thread; ends on a barrier): 16 x 16 diagonal blocks by forward substitution
// (thread j solves column j of its block), then three levels of merges [[X11, 0], [-X22 M21 X11, X22]] (tri128_merge).
// tb: 64 * 64 values of scratch.
__device__ __forceinline__ void tri128_inverse_lds(float (*mb)[129], float (*xb)[129], float* tb, int tid) {
  if (tid < 128) {                                     // column tid of its 16 x 16 diagonal block
    const int j = tid, b0 = j & ~15;
    for (int i = j; i < b0 + 16; ++i) {
      float acc = 0.0f;
      for (int k = j; k < i; ++k) acc = fmaf(mb[i][k], xb[k][j], acc);
      xb[i][j] = i == j ? 1.0f / mb[j][j] : -acc / mb[i][i];
    }
  }
  __syncthreads();
  tri128_merge<16, 2, 2>(mb, xb, tb, tid);
  tri128_merge<32, 2, 4>(mb, xb, tb, tid);
  tri128_merge<64, 4, 4>(mb, xb, tb, tid);
}

// X_bb = M_bb^-1 for every 128 x 128 diagonal block b (one workgroup of 256 threads each) by the recursion above;
// the block and its transpose are written into the full matrices x and xt.
template <int WHICH>
__global__ __launch_bounds__(256) void k_tri_diag_inverse(LuSrc q, int dp, float* __restrict__ x, float* __restrict__ xt) {
  __shared__ float mb[128][129];
  __shared__ float xb[128][129];
  __shared__ float tb[64 * 64];
  const int blk = blockIdx.x, tid = threadIdx.x, o = blk * 128;
  for (int e = tid; e < 128 * 128; e += 256) {
    const int i = e >> 7, j = e & 127;
    mb[i][j] = tri_elem<WHICH>(q, o + i, o + j);
    xb[i][j] = 0.0f;
  }
  __syncthreads();
  tri128_inverse_lds(mb, xb, tb, tid);
  for (int e = tid; e < 128 * 128; e += 256) {
    const int i = e >> 7, j = e & 127;
    x[(int64_t)(o + i) * dp + o + j] = xb[i][j];
    xt[(int64_t)(o + i) * dp + o + j] = xb[j][i];
  }
}

// ---- many small matrices at once (the per-block transformations: one d x d parameter set per transformer block, d the
// head dimension) --------------------------------------------------------------------------------------------------
// For d <= 128 a matrix fits into LDS, and the full-size path above would be a dozen launch-bound kernels per matrix.
// Here one workgroup of 256 threads owns one matrix and one launch covers `count` of them; the products are plain
// binary32 multiply-adds out of LDS (2 d^3 operations per product: microseconds).  Thread (ty, tx) = (tid / 16,
// tid % 16) owns the outputs (ty + 16 a, tx + 16 b), a, b = 0..7.
__device__ __forceinline__ LuSrc small_src(const float* lp, const float* up, const float* log_s, const float* sign_s, int d, int m) {
  const int64_t mo = (int64_t)m * d * d, vo = (int64_t)m * d;
  return LuSrc{lp + mo, up + mo, log_s + vo, sign_s + vo, nullptr, nullptr, d};
}
__device__ __forceinline__ int small_perm(const int* perm, int d, int i) {       // an entry out of range is treated as i
  const int p = perm[i];
  return (unsigned)p < (unsigned)d ? p : i;
}

// out[r][j] = sum_k L[perm[r]][k] (U + diag s)[k][j]
template <typename T>
__global__ __launch_bounds__(256) void k_lu_small_compose(const float* __restrict__ lp, const float* __restrict__ up, const float* __restrict__ log_s,
                                                          const float* __restrict__ sign_s, const int* __restrict__ perm, int d, T* __restrict__ out) {
  __shared__ float lm[128][129];
  __shared__ float um[128][129];
  const int m = blockIdx.x, tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
  const LuSrc q = small_src(lp, up, log_s, sign_s, d, m);
  for (int e = tid; e < d * d; e += 256) {
    const int i = e / d, j = e - i * d;
    lm[i][j] = tri_elem<0>(q, i, j);
    um[j][i] = tri_elem<1>(q, i, j);                   // tri_elem<1> is (U + diag s)^T
  }
  __syncthreads();
  int pr[8];
#pragma unroll
  for (int a = 0; a < 8; ++a) pr[a] = ty + 16 * a < d ? small_perm(perm + (int64_t)m * d, d, ty + 16 * a) : 0;
  float acc[8][8];
#pragma unroll
  for (int a = 0; a < 8; ++a)
#pragma unroll
    for (int b = 0; b < 8; ++b) acc[a][b] = 0.0f;
  for (int k = 0; k < d; ++k) {
    float av[8], bv[8];
#pragma unroll
    for (int a = 0; a < 8; ++a) av[a] = ty + 16 * a < d ? lm[pr[a]][k] : 0.0f;
#pragma unroll
    for (int b = 0; b < 8; ++b) bv[b] = tx + 16 * b < d ? um[k][tx + 16 * b] : 0.0f;
#pragma unroll
    for (int a = 0; a < 8; ++a)
#pragma unroll
      for (int b = 0; b < 8; ++b) acc[a][b] = fmaf(av[a], bv[b], acc[a][b]);
  }
  T* o = out + (int64_t)m * d * d;
#pragma unroll
  for (int a = 0; a < 8; ++a)
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      const int r = ty + 16 * a, j = tx + 16 * b;
      if (r < d && j < d) Store<T>::st(o + (int64_t)r * d + j, acc[a][b]);
    }
}

// B = P^T G (B[perm[i]] = G[i]);  d_up = strictly upper part of L^T B, d_log_s = its diagonal times s,
// d_lp = strictly lower part of B (U + diag s)^T
template <typename T>
__global__ __launch_bounds__(256) void k_lu_small_backward(const T* __restrict__ g, const float* __restrict__ lp, const float* __restrict__ up,
                                                           const float* __restrict__ log_s, const float* __restrict__ sign_s, const int* __restrict__ perm,
                                                           int d, float* __restrict__ d_lp, float* __restrict__ d_up, float* __restrict__ d_log_s) {
  __shared__ float bm[128][129];
  __shared__ float fm[128][129];
  const int m = blockIdx.x, tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
  const int64_t mo = (int64_t)m * d * d, vo = (int64_t)m * d;
  const LuSrc q = small_src(lp, up, log_s, sign_s, d, m);
  for (int e = tid; e < d * d; e += 256) {
    const int i = e / d, j = e - i * d;
    bm[i][j] = 0.0f;                                   // (rows that a perm with duplicates never names)
    fm[i][j] = tri_elem<0>(q, i, j);
  }
  __syncthreads();
  for (int e = tid; e < d * d; e += 256) {
    const int i = e / d, j = e - i * d;
    bm[small_perm(perm + vo, d, i)][j] = Store<T>::ld(g + mo + e);
  }
  __syncthreads();
  float acc[8][8];
#pragma unroll
  for (int a = 0; a < 8; ++a)
#pragma unroll
    for (int b = 0; b < 8; ++b) acc[a][b] = 0.0f;
  for (int i = 0; i < d; ++i) {                        // (L^T B)[k][n] = sum_i L[i][k] B[i][n]
    float av[8], bv[8];
#pragma unroll
    for (int a = 0; a < 8; ++a) av[a] = ty + 16 * a < d ? fm[i][ty + 16 * a] : 0.0f;
#pragma unroll
    for (int b = 0; b < 8; ++b) bv[b] = tx + 16 * b < d ? bm[i][tx + 16 * b] : 0.0f;
#pragma unroll
    for (int a = 0; a < 8; ++a)
#pragma unroll
      for (int b = 0; b < 8; ++b) acc[a][b] = fmaf(av[a], bv[b], acc[a][b]);
  }
#pragma unroll
  for (int a = 0; a < 8; ++a)
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      const int k = ty + 16 * a, n = tx + 16 * b;
      if (k < d && n < d) {
        d_up[mo + (int64_t)k * d + n] = n > k ? acc[a][b] : 0.0f;
        if (n == k) d_log_s[vo + k] = acc[a][b] * (q.sign[k] * expf(q.log_s[k]));
      }
      acc[a][b] = 0.0f;
    }
  __syncthreads();
  for (int e = tid; e < d * d; e += 256) {
    const int i = e / d, j = e - i * d;
    fm[j][i] = tri_elem<1>(q, i, j);                   // fm = U + diag s
  }
  __syncthreads();
  for (int n = 0; n < d; ++n) {                        // (B (U + diag s)^T)[r][k] = sum_n B[r][n] (U + diag s)[k][n]
    float av[8], bv[8];
#pragma unroll
    for (int a = 0; a < 8; ++a) av[a] = ty + 16 * a < d ? bm[ty + 16 * a][n] : 0.0f;
#pragma unroll
    for (int b = 0; b < 8; ++b) bv[b] = tx + 16 * b < d ? fm[tx + 16 * b][n] : 0.0f;
#pragma unroll
    for (int a = 0; a < 8; ++a)
#pragma unroll
      for (int b = 0; b < 8; ++b) acc[a][b] = fmaf(av[a], bv[b], acc[a][b]);
  }
#pragma unroll
  for (int a = 0; a < 8; ++a)
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      const int r = ty + 16 * a, k = tx + 16 * b;
      if (r < d && k < d) d_lp[mo + (int64_t)r * d + k] = k < r ? acc[a][b] : 0.0f;
    }
}

// out[i][c] = ((U + diag s)^-1 L^-1)[i][perm[c]]: both factors inverted by the in-LDS recursion (padded to 128 with an
// identity block), L^-1 parked in registers while (U + diag s)^T is inverted
template <typename T>
__global__ __launch_bounds__(256) void k_lu_small_inverse(const float* __restrict__ lp, const float* __restrict__ up, const float* __restrict__ log_s,
                                                          const float* __restrict__ sign_s, const int* __restrict__ perm, int d, T* __restrict__ out) {
  __shared__ float mb[128][129];
  __shared__ float xb[128][129];
  __shared__ float tb[64 * 64];
  const int m = blockIdx.x, tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
  const LuSrc q = small_src(lp, up, log_s, sign_s, d, m);
  for (int e = tid; e < 128 * 128; e += 256) {
    const int i = e >> 7, j = e & 127;
    mb[i][j] = tri_elem<0>(q, i, j);
    xb[i][j] = 0.0f;
  }
  __syncthreads();
  tri128_inverse_lds(mb, xb, tb, tid);
  float keep[64];                                      // L^-1, element tid + 256 e
#pragma unroll
  for (int e = 0; e < 64; ++e) keep[e] = xb[(tid + 256 * e) >> 7][(tid + 256 * e) & 127];
  __syncthreads();
  for (int e = tid; e < 128 * 128; e += 256) {
    const int i = e >> 7, j = e & 127;
    mb[i][j] = tri_elem<1>(q, i, j);
    xb[i][j] = 0.0f;
  }
  __syncthreads();
  tri128_inverse_lds(mb, xb, tb, tid);                 // xb = ((U + diag s)^T)^-1 = ((U + diag s)^-1)^T
#pragma unroll
  for (int e = 0; e < 64; ++e) mb[(tid + 256 * e) >> 7][(tid + 256 * e) & 127] = keep[e];
  __syncthreads();
  int pc[8];
#pragma unroll
  for (int b = 0; b < 8; ++b) pc[b] = tx + 16 * b < d ? small_perm(perm + (int64_t)m * d, d, tx + 16 * b) : 0;
  float acc[8][8];
#pragma unroll
  for (int a = 0; a < 8; ++a)
#pragma unroll
    for (int b = 0; b < 8; ++b) acc[a][b] = 0.0f;
  for (int k = 0; k < d; ++k) {                        // sum_k (U + diag s)^-1[i][k] L^-1[k][j]
    float av[8], bv[8];
#pragma unroll
    for (int a = 0; a < 8; ++a) av[a] = xb[k][ty + 16 * a];
#pragma unroll
    for (int b = 0; b < 8; ++b) bv[b] = mb[k][pc[b]];
#pragma unroll
    for (int a = 0; a < 8; ++a)
#pragma unroll
      for (int b = 0; b < 8; ++b) acc[a][b] = fmaf(av[a], bv[b], acc[a][b]);
  }
  T* o = out + (int64_t)m * d * d;
#pragma unroll
  for (int a = 0; a < 8; ++a)
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      const int i = ty + 16 * a, c = tx + 16 * b;
      if (i < d && c < d) Store<T>::st(o + (int64_t)i * d + c, acc[a][b]);
    }
}

// out[r][c] = z[r][perm[c]] in the storage type (z P^T); z has rows of dp entries, out is d x d
template <typename T>
__global__ __launch_bounds__(256) void k_lu_inverse_out(const float* __restrict__ z, const int* __restrict__ perm, int d, int dp, T* __restrict__ out) {
  const int64_t n = (int64_t)d * d;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int r = (int)(i / d), c = (int)(i - (int64_t)r * d);
    int src = perm[c];
    if ((unsigned)src >= (unsigned)d) src = c;                         // not a permutation: stay inside the arrays
    Store<T>::st(out + i, z[(int64_t)r * dp + src]);
  }
}

// dst [d][d] = the leading d x d part of src, whose rows hold dp entries (both multiples of 128: 16-byte vectors)
__global__ __launch_bounds__(256) void k_tri_compact(const float* __restrict__ src, int dp, int d, float* __restrict__ dst) {
  const int64_t n4 = (int64_t)d * (d / 4);
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (int64_t)gridDim.x * 256) {
    const int r = (int)(i / (d / 4)), c4 = (int)(i - (int64_t)r * (d / 4));
    reinterpret_cast<float4*>(dst)[i] = *reinterpret_cast<const float4*>(src + (int64_t)r * dp + 4 * c4);
  }
}

template <typename T, int SRC>
void launch_build_transposed(const LuSrc& q, void* out, hipStream_t s) {
  if (q.d % 64 == 0) hipLaunchKernelGGL((k_lu_build_transposed<T, SRC>), dim3(q.d / 64, q.d / 64), dim3(256), 0, s, q, reinterpret_cast<T*>(out));
  else launch_build<T, SRC, true>(q, out, s);
}

template <typename T, int SRC>
void launch_build_rows(const LuSrc& q, void* out, hipStream_t s) {
  const int64_t g = ((int64_t)q.d * (q.d / 8) + 255) / 256;
  hipLaunchKernelGGL((k_lu_build_rows<T, SRC>), dim3((unsigned)(g < 8192 ? g : 8192)), dim3(256), 0, s, q, reinterpret_cast<T*>(out));
}

// measurement aid (model_lu_timing): HIP events around every matrix-core product, waited for at once
bool g_timing = false;
double g_timing_ms = 0.0;
int64_t g_timing_launches = 0;
hipEvent_t g_ev0 = nullptr, g_ev1 = nullptr;

// one stream of the library's own (default priority, created on first use, kept until the process ends) for work that
// runs beside the caller's stream; null if it cannot be created (the callers then stay on one stream)
hipStream_t lu_side_stream() {
  static std::once_flag once;
  static hipStream_t side = nullptr;
  std::call_once(once, [] {
    if (hipStreamCreateWithFlags(&side, hipStreamNonBlocking) != hipSuccess) side = nullptr;
  });
  return side;
}

// A second branch of work beside the caller's stream: begin() forks the library's stream from `main`, end() joins it
// back — also after an error, so that `main` always covers both branches.  The two events are created once per host
// thread and reused by every call (a wait enqueued on a stream refers to the record that preceded it, so recording
// the event again for the next call does not disturb waits already enqueued); calls from several host threads only
// share the stream.  Disabled (or no stream / events to be had): side == main, everything stays in order.
struct SideBranch {
  hipStream_t main = nullptr, side = nullptr;
  hipEvent_t fork = nullptr, join = nullptr;
  static bool events(hipEvent_t* f, hipEvent_t* j) {
    static thread_local hipEvent_t ev[2] = {nullptr, nullptr};
    static thread_local bool tried = false;
    if (!tried) {
      tried = true;
      if (hipEventCreateWithFlags(&ev[0], hipEventDisableTiming) != hipSuccess) ev[0] = nullptr;
      if (ev[0] && hipEventCreateWithFlags(&ev[1], hipEventDisableTiming) != hipSuccess) {
        (void)hipEventDestroy(ev[0]);
        ev[0] = ev[1] = nullptr;
      }
    }
    *f = ev[0];
    *j = ev[1];
    return ev[0] != nullptr;
  }
  int begin(hipStream_t s, bool enable, const char* who) {
    main = side = s;
    hipStream_t s2 = enable ? lu_side_stream() : nullptr;
    hipEvent_t f = nullptr, j = nullptr;
    if (!s2 || !events(&f, &j)) return AE_OK;
    if (hipEventRecord(f, s) != hipSuccess || hipStreamWaitEvent(s2, f, 0) != hipSuccess)
      return fail(AE_EHIP, "%s: cannot fork the side stream", who);
    fork = f;
    join = j;
    side = s2;
    return AE_OK;
  }
  int end(int rc, const char* who) {
    if (!fork) return rc;
    const bool joined = hipEventRecord(join, side) == hipSuccess && hipStreamWaitEvent(main, join, 0) == hipSuccess;
    fork = join = nullptr;
    if (!joined && rc == AE_OK) rc = fail(AE_EHIP, "%s: cannot join the side stream", who);
    return rc;
  }
};

// y[m][n] = sum_k x[m][k] w[n][k], all d x d in the storage type; tri: which operand is triangular (CONV_TRI_*)
int dense_product(const void* x, const void* w, void* y, int d, int dtype, int tri, hipStream_t s) {
  ConvArgs a;
  memset(&a, 0, sizeof(a));
  a.x = x; a.w = w; a.bias = nullptr; a.y = y;
  a.n = d; a.hc = a.wc = 1; a.cin = a.cout = d; a.k = 1; a.up = 0; a.act = ACT_NONE; a.dtype = dtype;
  a.tri = tri;
  if (!g_timing) return launch_conv_mfma(a, s);
  AE_HIP(hipEventRecord(g_ev0, s));
  AE_TRY(launch_conv_mfma(a, s));
  AE_HIP(hipEventRecord(g_ev1, s));
  AE_HIP(hipEventSynchronize(g_ev1));
  float ms = 0.0f;
  AE_HIP(hipEventElapsedTime(&ms, g_ev0, g_ev1));
  g_timing_ms += ms;
  ++g_timing_launches;
  return AE_OK;
}

int64_t lu_mat_bytes(int64_t d, int dtype) { return d * d * (int64_t)dtype_size(dtype); }
unsigned lu_grid(int64_t items) {
  const int64_t g = (items + 256 * 8 - 1) / (256 * 8);
  return (unsigned)(g < 4096 ? (g < 1 ? 1 : g) : 4096);
}

// xt[c][r] = x[r][c] over the lower off-diagonal block (rows in block 2p+1, columns in block 2p, blocks of b) of every
// pair p = blockIdx.z: 32 x 32 tiles through LDS
__global__ __launch_bounds__(256) void k_tri_pair_transpose(const float* __restrict__ x, float* __restrict__ xt, int dp, int b) {
  __shared__ float tile[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  const int r0 = (2 * (int)blockIdx.z + 1) * b + (int)blockIdx.y * 32, c0 = 2 * (int)blockIdx.z * b + (int)blockIdx.x * 32;
#pragma unroll
  for (int j = 0; j < 4; ++j) tile[ty + 8 * j][tx] = x[(int64_t)(r0 + ty + 8 * j) * dp + c0 + tx];
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 4; ++j) xt[(int64_t)(c0 + ty + 8 * j) * dp + r0 + tx] = tile[tx][ty + 8 * j];
}

// 128 times the smallest power of two that reaches d: the working size of the recursion
int64_t tri_padded_size(int64_t d) {
  int64_t dp = 128;
  while (dp < d) dp *= 2;
  return dp;
}

// the blocked recursion above for one lower triangular matrix, padded with an identity block to the working size
// d = dp (128 times a power of two, at least q.d): x = M^-1 and xt = its transpose ([dp][dp] binary32 each);
// mneg and tt are scratch of the same size
template <int WHICH>
int tri_inverse(const LuSrc& q, int dp, float* mneg, float* tt, float* x, float* xt, hipStream_t s) {
  const int d = dp;
  hipLaunchKernelGGL((k_tri_prepare<WHICH>), dim3(d / 32, d / 32), dim3(256), 0, s, q, d, mneg, x, xt);
  hipLaunchKernelGGL((k_tri_diag_inverse<WHICH>), dim3(d / 128), dim3(256), 0, s, q, d, x, xt);
  AE_TRY(launch_status("tri_diag_inverse"));
  for (int b = 128; b < d; b *= 2) {
    ConvArgs a;
    memset(&a, 0, sizeof(a));
    a.n = d; a.hc = a.wc = 1; a.cin = a.cout = d; a.k = 1; a.up = 0; a.act = ACT_NONE; a.dtype = AE_F32;
    a.tri_b = b;
    a.tri_pairs = (q.d + 2 * b - 1) / (2 * b);                            // pairs wholly inside the identity padding stay as they are
    a.tri_d = q.d < d ? q.d : 0;                                          // ... and so do the zero parts of the last pair
    a.x = xt; a.w = mneg; a.y = tt; a.tri = CONV_TRI_PAIR_UPPER_K0;       // T' = X11^T (-M21)^T = -(M21 X11)^T
    AE_TRY(launch_conv_mfma(a, s));
    a.x = x; a.w = tt; a.y = x; a.tri = CONV_TRI_PAIR_LOWER_K1;           // X21 = X22 T'^T (reads the diagonal blocks of x, writes below them)
    AE_TRY(launch_conv_mfma(a, s));
    // X21^T into X^T: a transposing copy (a third product would give the same block at fifteen times the cost)
    hipLaunchKernelGGL(k_tri_pair_transpose, dim3(b / 32, b / 32, a.tri_pairs), dim3(256), 0, s, (const float*)x, xt, d, b);
    AE_TRY(launch_status("tri_pair_transpose"));
  }
  return AE_OK;
}

// ---- QR parametrisation (Eq. 5):  Q = exp((G - G^T) / 2),  A = Q (R + diag s) ------------------------------------
// The exponential is scaling and squaring: X = S / 2^J, the Taylor polynomial of order 8, then J squarings — all
// binary32 products on the matrix cores.  The polynomial is evaluated in powers of Y = X^3 (four products instead of
// the seven of Horner's rule in X):
//     X2 = X X,  Y = X2 X,   B0 = I + X + X2/2,  B1 = I/3! + X/4! + X2/5!,  B2 = I/6! + X/7! + X2/8!,
//     U = B1 + B2 Y,   Q_0 = B0 + U Y.
// The product kernel computes y = x w^T; X is exactly skew-symmetric, so X^T = -X, X2^T = X2, Y^T = -Y and none of
// these factors needs a transposed copy (x X = -(x X^T)).  The backward pass is the adjoint of this chain, step by
// step, with the stored X, X2, Y, U, U^T, B2, B2^T and Q_i, Q_i^T (eight products for the polynomial, two per
// squaring); one fused element-wise pass (k_qr_combine) forms sums, scalings and transposes.
constexpr int kQrOrder = 8;

// out = ident * I + alpha * y (+ beta * y2), out_t = out^T; 32 x 32 tiles.  y2, out, out_t may be null.
__global__ __launch_bounds__(256) void k_qr_combine(const float* __restrict__ y, const float* __restrict__ y2, float alpha, float beta,
                                                    float ident, int d, float* __restrict__ out, float* __restrict__ out_t) {
  __shared__ float tile[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int r = r0 + ty + 8 * j, c = c0 + tx;
    const int64_t i = (int64_t)r * d + c;
    float v = alpha * y[i] + (r == c ? ident : 0.0f);
    if (y2) v += beta * y2[i];
    if (out) out[i] = v;
    tile[ty + 8 * j][tx] = v;
  }
  __syncthreads();
  if (out_t) {
#pragma unroll
    for (int j = 0; j < 4; ++j) out_t[(int64_t)(c0 + ty + 8 * j) * d + r0 + tx] = tile[tx][ty + 8 * j];
  }
}

// out = scale * (g - g^T): the scaled skew part (scale = 1 / (2 * 2^J) forward; the same form gives dG from dX)
__global__ __launch_bounds__(256) void k_qr_skew(const float* __restrict__ g, float scale, int d, float* __restrict__ out) {
  __shared__ float tile[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
#pragma unroll
  for (int j = 0; j < 4; ++j) tile[ty + 8 * j][tx] = g[(int64_t)(c0 + ty + 8 * j) * d + r0 + tx];   // g[c][r]
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int r = r0 + ty + 8 * j, c = c0 + tx;
    out[(int64_t)r * d + c] = scale * (g[(int64_t)r * d + c] - tile[tx][ty + 8 * j]);
  }
}

// rowsum[i] = sum_j |m[i][j]|: one wavefront per row, fixed order
__global__ __launch_bounds__(256) void k_row_abs_sum(const float* __restrict__ m, int d, float* __restrict__ rowsum) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= d) return;
  float acc = 0.0f;
  for (int j = lane; j < d; j += 64) acc += fabsf(m[(int64_t)row * d + j]);
  acc = wave_sum(acc);
  if (lane == 0) rowsum[row] = acc;
}
// out[0] = max_i v[i] (one workgroup; NaN propagates as +inf so that the caller refuses it)
__global__ __launch_bounds__(256) void k_vec_max(const float* __restrict__ v, int d, float* __restrict__ out) {
  __shared__ float sm[256];
  float mx = 0.0f;
  for (int i = threadIdx.x; i < d; i += 256) { const float x = v[i]; mx = (x == x) ? fmaxf(mx, x) : INFINITY; }
  sm[threadIdx.x] = mx;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off) sm[threadIdx.x] = fmaxf(sm[threadIdx.x], sm[threadIdx.x + off]);
    __syncthreads();
  }
  if (threadIdx.x == 0) out[0] = sm[0];
}

// acc = (first ? 0 : acc) + alpha * y
__global__ __launch_bounds__(256) void k_qr_axpy(float* __restrict__ acc, const float* __restrict__ y, float alpha, int first, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256)
    acc[i] = (first ? 0.0f : acc[i]) + alpha * y[i];
}

// binary32 <-> storage type
template <typename T>
__global__ __launch_bounds__(256) void k_to_f32(const T* __restrict__ in, float* __restrict__ out, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) out[i] = Store<T>::ld(in + i);
}
template <typename T>
__global__ __launch_bounds__(256) void k_from_f32(const float* __restrict__ in, T* __restrict__ out, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) Store<T>::st(out + i, in[i]);
}

void qr_combine(const float* y, const float* y2, float alpha, float beta, float ident, int d, float* out, float* out_t, hipStream_t s) {
  hipLaunchKernelGGL(k_qr_combine, dim3(d / 32, d / 32), dim3(256), 0, s, y, y2, alpha, beta, ident, d, out, out_t);
}

// workspace of the QR calls: binary32 d x d matrices
struct QrSlots {
  float* base; int64_t dd; int J;
  float* x() const { return base; }                                  // S / 2^J
  float* h(int k) const { return base + (int64_t)(k - 1) * dd; }     // slots 1 .. kQrOrder-1 (k = 2 .. kQrOrder):
  float* x2() const { return h(2); }                                 //   X X (symmetric)
  float* y3() const { return h(3); }                                 //   X^3 (skew-symmetric)
  float* u() const { return h(4); }                                  //   U = B1 + B2 Y
  float* ut() const { return h(5); }
  float* b2() const { return h(6); }                                 //   B2 = I/6! + X/7! + X2/8!
  float* b2t() const { return h(7); }
  float* spare() const { return h(8); }                              //   a seventh temporary of the backward pass
  float* q(int i) const { return base + (int64_t)(kQrOrder + i) * dd; }              // Q_i, i = 0 .. J
  float* qt(int i) const { return base + (int64_t)(kQrOrder + J + 1 + i) * dd; }     // Q_i^T
  float* tmp(int t) const { return base + (int64_t)(kQrOrder + 2 * (J + 1) + t) * dd; }   // six temporaries
  static int64_t count(int J) { return kQrOrder + 2 * (J + 1) + 6; }
};

int check_qr_args(const char* who, int64_t d, int dtype, int squarings) {
  if (dtype != AE_F32 && dtype != AE_BF16) return fail(AE_EINVAL, "%s: bad dtype", who);
  if (d < 32 || d % 32 != 0 || d > 16384) return fail(AE_EINVAL, "%s: d must be a multiple of 32 between 32 and 16384", who);
  if (squarings < 0 || squarings > 16) return fail(AE_EINVAL, "%s: squarings must be 0 .. 16", who);
  return AE_OK;
}

int check_lu_size(const char* who, int64_t d, int dtype) {
  if (dtype != AE_F32 && dtype != AE_BF16) return fail(AE_EINVAL, "%s: bad dtype", who);
  if (d < 32 || d % 32 != 0 || d > 16384) return fail(AE_EINVAL, "%s: d must be a multiple of 32 between 32 and 16384", who);
  return AE_OK;
}

int check_small_batch(const char* who, int64_t count, int64_t d, int dtype) {
  if (dtype != AE_F32 && dtype != AE_BF16) return fail(AE_EINVAL, "%s: bad dtype", who);
  if (d < 1 || d > 128) return fail(AE_EINVAL, "%s: d must be 1 .. 128 (larger matrices take the full-size calls)", who);
  if (count < 1 || count > (1 << 20)) return fail(AE_EINVAL, "%s: count must be 1 .. 2^20", who);
  return AE_OK;
}

}  // namespace
}  // namespace ae

extern "C" int model_lu_compose_batch(const float* lp, const float* up, const float* log_s, const float* sign_s, const int* perm,
                                      int64_t count, int64_t d, int dtype, void* a_out, void* stream) {
  using namespace ae;
  if (!lp || !up || !log_s || !sign_s || !perm || !a_out) return fail(AE_EINVAL, "model_lu_compose_batch: null argument");
  AE_TRY(check_small_batch("model_lu_compose_batch", count, d, dtype));
  hipStream_t s = (hipStream_t)stream;
  if (dtype == AE_BF16) hipLaunchKernelGGL((k_lu_small_compose<bf16_t>), dim3((unsigned)count), dim3(256), 0, s, lp, up, log_s, sign_s, perm, (int)d, (bf16_t*)a_out);
  else hipLaunchKernelGGL((k_lu_small_compose<float>), dim3((unsigned)count), dim3(256), 0, s, lp, up, log_s, sign_s, perm, (int)d, (float*)a_out);
  return launch_status("lu_small_compose");
}

extern "C" int model_lu_backward_batch(const void* g, const float* lp, const float* up, const float* log_s, const float* sign_s,
                                       const int* perm, int64_t count, int64_t d, int dtype, float* d_lp, float* d_up,
                                       float* d_log_s, void* stream) {
  using namespace ae;
  if (!g || !lp || !up || !log_s || !sign_s || !perm || !d_lp || !d_up || !d_log_s) return fail(AE_EINVAL, "model_lu_backward_batch: null argument");
  AE_TRY(check_small_batch("model_lu_backward_batch", count, d, dtype));
  hipStream_t s = (hipStream_t)stream;
  if (dtype == AE_BF16) hipLaunchKernelGGL((k_lu_small_backward<bf16_t>), dim3((unsigned)count), dim3(256), 0, s, (const bf16_t*)g, lp, up, log_s, sign_s, perm, (int)d, d_lp, d_up, d_log_s);
  else hipLaunchKernelGGL((k_lu_small_backward<float>), dim3((unsigned)count), dim3(256), 0, s, (const float*)g, lp, up, log_s, sign_s, perm, (int)d, d_lp, d_up, d_log_s);
  return launch_status("lu_small_backward");
}

extern "C" int model_lu_inverse_batch(const float* lp, const float* up, const float* log_s, const float* sign_s, const int* perm,
                                      int64_t count, int64_t d, int dtype, void* a_inv_out, void* stream) {
  using namespace ae;
  if (!lp || !up || !log_s || !sign_s || !perm || !a_inv_out) return fail(AE_EINVAL, "model_lu_inverse_batch: null argument");
  AE_TRY(check_small_batch("model_lu_inverse_batch", count, d, dtype));
  hipStream_t s = (hipStream_t)stream;
  if (dtype == AE_BF16) hipLaunchKernelGGL((k_lu_small_inverse<bf16_t>), dim3((unsigned)count), dim3(256), 0, s, lp, up, log_s, sign_s, perm, (int)d, (bf16_t*)a_inv_out);
  else hipLaunchKernelGGL((k_lu_small_inverse<float>), dim3((unsigned)count), dim3(256), 0, s, lp, up, log_s, sign_s, perm, (int)d, (float*)a_inv_out);
  return launch_status("lu_small_inverse");
}

extern "C" int model_lu_workspace(int64_t d, int dtype, int64_t* bytes) {
  using namespace ae;
  if (!bytes) return fail(AE_EINVAL, "model_lu_workspace: null argument");
  AE_TRY(check_lu_size("model_lu_workspace", d, dtype));
  *bytes = 6 * lu_mat_bytes(d, dtype) + ((d * 4 + 255) / 256) * 256;
  return AE_OK;
}

extern "C" int model_lu_compose(const float* lp, const float* up, const float* log_s, const float* sign_s, const int* perm,
                                int64_t d, int dtype, void* a_out, void* workspace, void* stream) {
  using namespace ae;
  if (!lp || !up || !log_s || !sign_s || !perm || !a_out || !workspace) return fail(AE_EINVAL, "model_lu_compose: null argument");
  AE_TRY(check_lu_size("model_lu_compose", d, dtype));
  if (((reinterpret_cast<uintptr_t>(a_out) | reinterpret_cast<uintptr_t>(workspace) | reinterpret_cast<uintptr_t>(lp) |
        reinterpret_cast<uintptr_t>(up)) & 15) != 0)
    return fail(AE_EINVAL, "model_lu_compose: the matrices and the workspace must be 16-byte aligned");
  hipStream_t s = (hipStream_t)stream;
  const int64_t mat = lu_mat_bytes(d, dtype);
  char* ws = reinterpret_cast<char*>(workspace);
  void* l = ws;                 // L                 [i][k]
  void* udt = ws + mat;         // (U + diag s)^T    [n][k]
  void* y = ws + 2 * mat;       // L (U + diag s)    [i][n]
  LuSrc q{lp, up, log_s, sign_s, nullptr, nullptr, (int)d};
  if (dtype == AE_BF16) { launch_build_rows<bf16_t, LU_L>(q, l, s); launch_build_transposed<bf16_t, LU_UD>(q, udt, s); }
  else { launch_build_rows<float, LU_L>(q, l, s); launch_build_transposed<float, LU_UD>(q, udt, s); }
  AE_TRY(launch_status("lu_build"));
  AE_TRY(dense_product(l, udt, y, (int)d, dtype, CONV_TRI_LOWER_UPPER, s));
  const int cpr = (int)(d * (int64_t)dtype_size(dtype) / 16);
  hipLaunchKernelGGL(k_lu_permute_rows, dim3(lu_grid(d * cpr)), dim3(256), 0, s, (const uint4*)y, perm, (int)d, cpr, (uint4*)a_out);
  return launch_status("lu_permute_rows");
}

extern "C" int model_lu_backward(const void* g, const float* lp, const float* up, const float* log_s, const float* sign_s,
                                 const int* perm, int64_t d, int dtype, float* d_lp, float* d_up, float* d_log_s,
                                 void* workspace, void* stream) {
  using namespace ae;
  if (!g || !lp || !up || !log_s || !sign_s || !perm || !d_lp || !d_up || !d_log_s || !workspace)
    return fail(AE_EINVAL, "model_lu_backward: null argument");
  AE_TRY(check_lu_size("model_lu_backward", d, dtype));
  if (((reinterpret_cast<uintptr_t>(g) | reinterpret_cast<uintptr_t>(workspace) | reinterpret_cast<uintptr_t>(lp) |
        reinterpret_cast<uintptr_t>(up) | reinterpret_cast<uintptr_t>(d_lp) | reinterpret_cast<uintptr_t>(d_up)) & 15) != 0)
    return fail(AE_EINVAL, "model_lu_backward: the matrices and the workspace must be 16-byte aligned");
  hipStream_t s = (hipStream_t)stream;
  const int64_t mat = lu_mat_bytes(d, dtype);
  char* ws = reinterpret_cast<char*>(workspace);
  void* lt = ws;                // L^T               [k][i]
  void* bt = ws + mat;          // B^T = (P^T G)^T   [n][i]
  void* ud = ws + 2 * mat;      // U + diag s        [k][n]
  void* b = ws + 3 * mat;       // B = P^T G         [r][n]
  void* dud = ws + 4 * mat;     // L^T B             [k][n]  (on and above the diagonal)
  void* dl = ws + 5 * mat;      // B (U + diag s)^T  [r][k]  (below the diagonal)
  int* inv = reinterpret_cast<int*>(ws + 6 * mat);
  const unsigned pg = (unsigned)((d + 255) / 256);
  hipLaunchKernelGGL(k_lu_iota, dim3(pg), dim3(256), 0, s, inv, (int)d);
  hipLaunchKernelGGL(k_lu_invert_perm, dim3(pg), dim3(256), 0, s, perm, inv, (int)d);
  LuSrc q{lp, up, log_s, sign_s, inv, g, (int)d};
  // The two gradient branches share nothing but their inputs, and a product with triangular K ranges ends on a few long
  // tiles that leave most of the chip idle: the lower-triangle branch runs on a stream of the library's own beside the
  // upper-triangle branch (not while model_lu_timing brackets every product with events on one stream).
  SideBranch br;
  AE_TRY(br.begin(s, !g_timing, "model_lu_backward"));
  hipStream_t s2 = br.side;
  int rc = AE_OK;
  const unsigned grid = lu_grid(d * d / 8 * 4);
  if (dtype == AE_BF16) {
    launch_build_transposed<bf16_t, LU_L>(q, lt, s); launch_build_transposed<bf16_t, LU_B>(q, bt, s);
    launch_build_rows<bf16_t, LU_UD>(q, ud, s2); launch_build_rows<bf16_t, LU_B>(q, b, s2);
  } else {
    launch_build_transposed<float, LU_L>(q, lt, s); launch_build_transposed<float, LU_B>(q, bt, s);
    launch_build_rows<float, LU_UD>(q, ud, s2); launch_build_rows<float, LU_B>(q, b, s2);
  }
  rc = launch_status("lu_build");
  if (rc == AE_OK) rc = dense_product(lt, bt, dud, (int)d, dtype, CONV_TRI_UPPER_X, s);
  if (rc == AE_OK) rc = dense_product(b, ud, dl, (int)d, dtype, CONV_TRI_UPPER_W, s2);
  if (rc == AE_OK) {
    if (dtype == AE_BF16) {
      hipLaunchKernelGGL((k_lu_grad_upper<bf16_t>), dim3(grid), dim3(256), 0, s, (const bf16_t*)dud, log_s, sign_s, (int)d, d_up, d_log_s);
      hipLaunchKernelGGL((k_lu_grad_lower<bf16_t>), dim3(grid), dim3(256), 0, s2, (const bf16_t*)dl, (int)d, d_lp);
    } else {
      hipLaunchKernelGGL((k_lu_grad_upper<float>), dim3(grid), dim3(256), 0, s, (const float*)dud, log_s, sign_s, (int)d, d_up, d_log_s);
      hipLaunchKernelGGL((k_lu_grad_lower<float>), dim3(grid), dim3(256), 0, s2, (const float*)dl, (int)d, d_lp);
    }
    rc = launch_status("lu_backward");
  }
  return br.end(rc, "model_lu_backward");
}

extern "C" int model_qr_workspace(int64_t d, int squarings, int64_t* bytes) {
  using namespace ae;
  if (!bytes) return fail(AE_EINVAL, "model_qr_workspace: null argument");
  AE_TRY(check_qr_args("model_qr_workspace", d, AE_F32, squarings));
  *bytes = QrSlots::count(squarings) * d * d * 4 + 1024;
  return AE_OK;
}

extern "C" int model_qr_squarings(const float* g, int64_t d, void* workspace, int* squarings, void* stream) {
  using namespace ae;
  if (!g || !workspace || !squarings) return fail(AE_EINVAL, "model_qr_squarings: null argument");
  AE_TRY(check_qr_args("model_qr_squarings", d, AE_F32, 0));
  if ((reinterpret_cast<uintptr_t>(workspace) & 15) != 0) return fail(AE_EINVAL, "model_qr_squarings: the workspace must be 16-byte aligned");
  hipStream_t s = (hipStream_t)stream;
  const int n = (int)d;
  float* skew = reinterpret_cast<float*>(workspace);          // S = (G - G^T) / 2
  float* rowsum = skew + d * d;                               // then d row sums and the maximum
  hipLaunchKernelGGL(k_qr_skew, dim3(n / 32, n / 32), dim3(256), 0, s, g, 0.5f, n, skew);
  hipLaunchKernelGGL(k_row_abs_sum, dim3((n + 3) / 4), dim3(256), 0, s, (const float*)skew, n, rowsum);
  hipLaunchKernelGGL(k_vec_max, dim3(1), dim3(256), 0, s, (const float*)rowsum, n, rowsum + d);
  AE_TRY(launch_status("qr_squarings"));
  float norm = 0.0f;
  AE_HIP(hipMemcpyAsync(&norm, rowsum + d, sizeof(float), hipMemcpyDeviceToHost, s));
  AE_HIP(hipStreamSynchronize(s));
  if (!(norm < INFINITY)) return fail(AE_EINVAL, "model_qr_squarings: the generator holds a NaN or an infinity");
  int j = 0;
  while (j <= 16 && ldexpf(1.0f, j) < 2.0f * norm) ++j;       // ||S||_2 <= ||S||_inf for a skew-symmetric S
  if (j > 16) return fail(AE_EINVAL, "model_qr_squarings: ||(G - G^T)/2|| = %g needs more than 16 squarings", (double)norm);
  *squarings = j;
  return AE_OK;
}

extern "C" int model_qr_compose(const float* g, const float* rp, const float* log_s, const float* sign_s, int64_t d, int dtype,
                                int squarings, void* a_out, void* workspace, void* stream) {
  using namespace ae;
  if (!g || !rp || !log_s || !sign_s || !a_out || !workspace) return fail(AE_EINVAL, "model_qr_compose: null argument");
  AE_TRY(check_qr_args("model_qr_compose", d, dtype, squarings));
  if (((reinterpret_cast<uintptr_t>(workspace) | reinterpret_cast<uintptr_t>(a_out) | reinterpret_cast<uintptr_t>(rp)) & 15) != 0)
    return fail(AE_EINVAL, "model_qr_compose: the matrices and the workspace must be 16-byte aligned");
  hipStream_t s = (hipStream_t)stream;
  const int n = (int)d, J = squarings;
  const QrSlots w{reinterpret_cast<float*>(workspace), d * d, J};
  const dim3 tgrid(n / 32, n / 32);
  hipLaunchKernelGGL(k_qr_skew, tgrid, dim3(256), 0, s, g, 0.5f / (float)(1 << J), n, w.x());
  float* y = w.tmp(1);
  float* b = w.tmp(0);
  // (dense_product(x, w, out) = x w^T; with w skew-symmetric that is -(x w))
  AE_TRY(dense_product(w.x(), w.x(), y, n, AE_F32, CONV_TRI_NONE, s));                      // X X^T = -X2
  qr_combine(y, nullptr, -1.0f, 0.0f, 0.0f, n, w.x2(), nullptr, s);
  AE_TRY(dense_product(w.x2(), w.x(), y, n, AE_F32, CONV_TRI_NONE, s));                     // X2 X^T = -Y
  qr_combine(y, nullptr, -1.0f, 0.0f, 0.0f, n, w.y3(), nullptr, s);
  qr_combine(w.x(), w.x2(), 1.0f / 5040.0f, 1.0f / 40320.0f, 1.0f / 720.0f, n, w.b2(), w.b2t(), s);
  AE_TRY(launch_status("qr_powers"));
  AE_TRY(dense_product(w.b2(), w.y3(), y, n, AE_F32, CONV_TRI_NONE, s));                    // B2 Y^T = -B2 Y
  qr_combine(w.x(), w.x2(), 1.0f / 24.0f, 1.0f / 120.0f, 1.0f / 6.0f, n, b, nullptr, s);    // B1
  qr_combine(y, b, -1.0f, 1.0f, 0.0f, n, w.u(), w.ut(), s);                                 // U = B1 + B2 Y
  AE_TRY(launch_status("qr_u"));
  AE_TRY(dense_product(w.u(), w.y3(), y, n, AE_F32, CONV_TRI_NONE, s));                     // U Y^T = -U Y
  qr_combine(w.x(), w.x2(), 1.0f, 0.5f, 1.0f, n, b, nullptr, s);                            // B0
  qr_combine(y, b, -1.0f, 1.0f, 0.0f, n, w.q(0), w.qt(0), s);                               // Q_0 = B0 + U Y
  AE_TRY(launch_status("qr_polynomial"));
  for (int i = 0; i < J; ++i) {
    AE_TRY(dense_product(w.q(i), w.qt(i), w.q(i + 1), n, AE_F32, CONV_TRI_NONE, s));        // Q_{i+1} = Q_i Q_i
    qr_combine(w.q(i + 1), nullptr, 1.0f, 0.0f, 0.0f, n, nullptr, w.qt(i + 1), s);
    AE_TRY(launch_status("qr_square"));
  }
  float* rdt = w.tmp(2);                                                                     // (R + diag s)^T
  LuSrc q{nullptr, rp, log_s, sign_s, nullptr, nullptr, n};
  launch_build_transposed<float, LU_UD>(q, rdt, s);
  AE_TRY(launch_status("qr_build"));
  if (dtype == AE_F32) return dense_product(w.q(J), rdt, a_out, n, AE_F32, CONV_TRI_NONE, s);
  AE_TRY(dense_product(w.q(J), rdt, y, n, AE_F32, CONV_TRI_NONE, s));
  hipLaunchKernelGGL((k_from_f32<bf16_t>), dim3(lu_grid(d * d)), dim3(256), 0, s, (const float*)y, (bf16_t*)a_out, d * d);
  return launch_status("qr_compose");
}

extern "C" int model_qr_backward(const void* g_a, const float* rp, const float* log_s, const float* sign_s, int64_t d, int dtype,
                                 int squarings, float* d_g, float* d_rp, float* d_log_s, void* workspace, void* stream) {
  using namespace ae;
  if (!g_a || !rp || !log_s || !sign_s || !d_g || !d_rp || !d_log_s || !workspace) return fail(AE_EINVAL, "model_qr_backward: null argument");
  AE_TRY(check_qr_args("model_qr_backward", d, dtype, squarings));
  if (((reinterpret_cast<uintptr_t>(workspace) | reinterpret_cast<uintptr_t>(g_a) | reinterpret_cast<uintptr_t>(rp) |
        reinterpret_cast<uintptr_t>(d_rp)) & 15) != 0)
    return fail(AE_EINVAL, "model_qr_backward: the matrices and the workspace must be 16-byte aligned");
  hipStream_t s = (hipStream_t)stream;
  const int n = (int)d, J = squarings;
  const int64_t dd = d * d;
  const QrSlots w{reinterpret_cast<float*>(workspace), dd, J};
  float *t0 = w.tmp(0), *t1 = w.tmp(1), *t2 = w.tmp(2), *t3 = w.tmp(3), *t4 = w.tmp(4), *t5 = w.tmp(5);
  // dA in binary32 (t0) and its transpose (t1)
  if (dtype == AE_BF16) hipLaunchKernelGGL((k_to_f32<bf16_t>), dim3(lu_grid(dd)), dim3(256), 0, s, (const bf16_t*)g_a, t0, dd);
  else hipLaunchKernelGGL((k_to_f32<float>), dim3(lu_grid(dd)), dim3(256), 0, s, (const float*)g_a, t0, dd);
  qr_combine(t0, nullptr, 1.0f, 0.0f, 0.0f, n, nullptr, t1, s);
  AE_TRY(launch_status("qr_backward_in"));
  // d(R + diag s) = Q^T dA: strictly upper part and diagonal
  AE_TRY(dense_product(w.qt(J), t1, t2, n, AE_F32, CONV_TRI_NONE, s));
  hipLaunchKernelGGL((k_lu_grad_upper<float>), dim3(lu_grid(dd / 8 * 4)), dim3(256), 0, s, (const float*)t2, log_s, sign_s, n, d_rp, d_log_s);
  // dQ_J = dA (R + diag s)^T  -> cur (t3), cur^T (t4)
  LuSrc q{nullptr, rp, log_s, sign_s, nullptr, nullptr, n};
  launch_build_rows<float, LU_UD>(q, t2, s);
  AE_TRY(launch_status("qr_build"));
  AE_TRY(dense_product(t0, t2, t3, n, AE_F32, CONV_TRI_NONE, s));
  qr_combine(t3, nullptr, 1.0f, 0.0f, 0.0f, n, nullptr, t4, s);
  float *cur = t3, *cur_t = t4;
  // squarings in reverse: dQ_i = dQ_{i+1} Q_i^T + Q_i^T dQ_{i+1}
  for (int i = J - 1; i >= 0; --i) {
    AE_TRY(dense_product(cur, w.q(i), t0, n, AE_F32, CONV_TRI_NONE, s));
    AE_TRY(dense_product(w.qt(i), cur_t, t1, n, AE_F32, CONV_TRI_NONE, s));
    qr_combine(t0, t1, 1.0f, 1.0f, 0.0f, n, cur, cur_t, s);
    AE_TRY(launch_status("qr_backward_square"));
  }
  // the polynomial in reverse; A = dQ_0, B = its transpose, C .. G free
  float *A = cur, *B = cur_t, *C = t0, *D = t1, *E = t2, *F = w.spare(), *G = t5;
  const dim3 eg(lu_grid(dd)), eb(256);
  AE_TRY(dense_product(A, w.y3(), C, n, AE_F32, CONV_TRI_NONE, s));                         // dU = dQ_0 Y^T
  qr_combine(C, nullptr, 1.0f, 0.0f, 0.0f, n, nullptr, D, s);                               // dU^T
  AE_TRY(dense_product(w.ut(), B, E, n, AE_F32, CONV_TRI_NONE, s));                         // U^T dQ_0        (Q_0 = B0 + U Y)
  AE_TRY(dense_product(w.b2t(), D, F, n, AE_F32, CONV_TRI_NONE, s));                        // B2^T dU         (U = B1 + B2 Y)
  qr_combine(E, F, 1.0f, 1.0f, 0.0f, n, E, D, s);                                           // dY = their sum (E) and dY^T (D)
  AE_TRY(launch_status("qr_backward_dy"));
  AE_TRY(dense_product(C, w.y3(), F, n, AE_F32, CONV_TRI_NONE, s));                         // dB2 = dU Y^T
  // dX  = dB0 + dB1/4! + dB2/7!  + ...,   dX2 = dB0/2 + dB1/5! + dB2/8! + ...   with dB0 = dQ_0, dB1 = dU
  hipLaunchKernelGGL(k_qr_axpy, eg, eb, 0, s, G, (const float*)A, 1.0f, 1, dd);
  hipLaunchKernelGGL(k_qr_axpy, eg, eb, 0, s, G, (const float*)C, 1.0f / 24.0f, 0, dd);
  hipLaunchKernelGGL(k_qr_axpy, eg, eb, 0, s, G, (const float*)F, 1.0f / 5040.0f, 0, dd);
  hipLaunchKernelGGL(k_qr_axpy, eg, eb, 0, s, B, (const float*)A, 0.5f, 1, dd);
  hipLaunchKernelGGL(k_qr_axpy, eg, eb, 0, s, B, (const float*)C, 1.0f / 120.0f, 0, dd);
  hipLaunchKernelGGL(k_qr_axpy, eg, eb, 0, s, B, (const float*)F, 1.0f / 40320.0f, 0, dd);
  AE_TRY(launch_status("qr_backward_db"));
  AE_TRY(dense_product(E, w.x(), A, n, AE_F32, CONV_TRI_NONE, s));                          // Y = X2 X:  dX2 += dY X^T
  hipLaunchKernelGGL(k_qr_axpy, eg, eb, 0, s, B, (const float*)A, 1.0f, 0, dd);
  AE_TRY(dense_product(w.x2(), D, C, n, AE_F32, CONV_TRI_NONE, s));                         //            dX  += X2^T dY = X2 dY
  hipLaunchKernelGGL(k_qr_axpy, eg, eb, 0, s, G, (const float*)C, 1.0f, 0, dd);
  qr_combine(B, nullptr, 1.0f, 0.0f, 0.0f, n, nullptr, F, s);                               // dX2^T
  AE_TRY(launch_status("qr_backward_dx2"));
  AE_TRY(dense_product(B, w.x(), A, n, AE_F32, CONV_TRI_NONE, s));                          // X2 = X X:  dX += dX2 X^T
  hipLaunchKernelGGL(k_qr_axpy, eg, eb, 0, s, G, (const float*)A, 1.0f, 0, dd);
  AE_TRY(dense_product(w.x(), F, C, n, AE_F32, CONV_TRI_NONE, s));                          //            dX += X^T dX2 = -(X dX2)
  hipLaunchKernelGGL(k_qr_axpy, eg, eb, 0, s, G, (const float*)C, -1.0f, 0, dd);
  float* dx = G;
  // X = (G - G^T) / (2 * 2^J):  dG = (dX - dX^T) / (2 * 2^J)
  hipLaunchKernelGGL(k_qr_skew, dim3(n / 32, n / 32), dim3(256), 0, s, (const float*)dx, 0.5f / (float)(1 << J), n, d_g);
  return launch_status("qr_backward");
}

extern "C" int model_qr_inverse(const float* rp, const float* log_s, const float* sign_s, int64_t d, int dtype, int squarings,
                                const void* qr_workspace, void* a_inv_out, void* workspace, void* stream) {
  using namespace ae;
  if (!rp || !log_s || !sign_s || !qr_workspace || !a_inv_out || !workspace) return fail(AE_EINVAL, "model_qr_inverse: null argument");
  AE_TRY(check_qr_args("model_qr_inverse", d, dtype, squarings));
  if (d < 128 || d % 128 != 0) return fail(AE_EINVAL, "model_qr_inverse: d must be a multiple of 128, at most 16384");
  if (((reinterpret_cast<uintptr_t>(workspace) | reinterpret_cast<uintptr_t>(qr_workspace) | reinterpret_cast<uintptr_t>(a_inv_out)) & 15) != 0)
    return fail(AE_EINVAL, "model_qr_inverse: the matrices and the workspaces must be 16-byte aligned");
  hipStream_t s = (hipStream_t)stream;
  const int64_t dd = d * d, dp = tri_padded_size(d), pp = dp * dp;
  const QrSlots w{const_cast<float*>(reinterpret_cast<const float*>(qr_workspace)), dd, squarings};
  float* f = reinterpret_cast<float*>(workspace);
  float *mneg = f, *tt = f + pp, *rdinv_t = f + 2 * pp, *rdinv = f + 3 * pp, *z = f + 4 * pp;
  LuSrc q{nullptr, rp, log_s, sign_s, nullptr, nullptr, (int)d};
  AE_TRY(tri_inverse<1>(q, (int)dp, mneg, tt, rdinv_t, rdinv, s));        // ((R + diag s)^T)^-1 and its transpose (R + diag s)^-1
  if (dp != d) {                                                          // drop the identity padding
    hipLaunchKernelGGL(k_tri_compact, dim3(lu_grid(dd)), dim3(256), 0, s, (const float*)rdinv, (int)dp, (int)d, mneg);
    AE_TRY(launch_status("tri_compact"));
    rdinv = mneg;
  }
  // A^-1 = (R + diag s)^-1 Q^T = x w^T with w = Q
  if (dtype == AE_F32) return dense_product(rdinv, w.q(squarings), a_inv_out, (int)d, AE_F32, CONV_TRI_NONE, s);
  AE_TRY(dense_product(rdinv, w.q(squarings), z, (int)d, AE_F32, CONV_TRI_NONE, s));
  hipLaunchKernelGGL((k_from_f32<bf16_t>), dim3(lu_grid(dd)), dim3(256), 0, s, (const float*)z, (bf16_t*)a_inv_out, dd);
  return launch_status("qr_inverse");
}

extern "C" int model_lu_inverse_workspace(int64_t d, int64_t* bytes) {
  using namespace ae;
  if (!bytes) return fail(AE_EINVAL, "model_lu_inverse_workspace: null argument");
  if (d < 128 || d > 16384 || d % 128 != 0) return fail(AE_EINVAL, "model_lu_inverse_workspace: d must be a multiple of 128, at most 16384");
  const int64_t dp = tri_padded_size(d);
  *bytes = 8 * dp * dp * 4 + 1024;
  return AE_OK;
}

extern "C" int model_lu_inverse(const float* lp, const float* up, const float* log_s, const float* sign_s, const int* perm,
                                int64_t d, int dtype, void* a_inv_out, void* workspace, void* stream) {
  using namespace ae;
  if (!lp || !up || !log_s || !sign_s || !perm || !a_inv_out || !workspace) return fail(AE_EINVAL, "model_lu_inverse: null argument");
  if (dtype != AE_F32 && dtype != AE_BF16) return fail(AE_EINVAL, "model_lu_inverse: bad dtype");
  if (d < 128 || d > 16384 || d % 128 != 0) return fail(AE_EINVAL, "model_lu_inverse: d must be a multiple of 128, at most 16384");
  if ((reinterpret_cast<uintptr_t>(workspace) & 15) != 0) return fail(AE_EINVAL, "model_lu_inverse: the workspace must be 16-byte aligned");
  hipStream_t s = (hipStream_t)stream;
  const int64_t dd = d * d, dp = tri_padded_size(d), pp = dp * dp;
  float* f = reinterpret_cast<float*>(workspace);
  float* mneg = f;                  // -M of the factor being inverted and the scratch of its recursion: for L ...
  float* tt = f + pp;
  float* linv = f + 2 * pp;         // L^-1 and its transpose; afterwards (U + diag s)^-1 L^-1
  float* linv_t = f + 3 * pp;
  float* udinv_t = f + 4 * pp;      // ((U + diag s)^T)^-1 = ((U + diag s)^-1)^T and its transpose (U + diag s)^-1
  float* udinv = f + 5 * pp;
  float* mneg_u = f + 6 * pp;       // ... and for (U + diag s)^T: the two inversions run side by side on two streams
  float* tt_u = f + 7 * pp;         // (the lower levels of the recursion have too few tiles to fill the chip alone)
  LuSrc q{lp, up, log_s, sign_s, nullptr, nullptr, (int)d};
  SideBranch br;
  AE_TRY(br.begin(s, !g_timing, "model_lu_inverse"));
  int rc = tri_inverse<0>(q, (int)dp, mneg, tt, linv, linv_t, s);
  if (rc == AE_OK) rc = tri_inverse<1>(q, (int)dp, mneg_u, tt_u, udinv_t, udinv, br.side);
  rc = br.end(rc, "model_lu_inverse");
  if (rc != AE_OK) return rc;
  if (dp != d) {                    // drop the identity padding: the two factors of the last product as d x d matrices
    hipLaunchKernelGGL(k_tri_compact, dim3(lu_grid(dd)), dim3(256), 0, s, (const float*)udinv, (int)dp, (int)d, mneg);
    hipLaunchKernelGGL(k_tri_compact, dim3(lu_grid(dd)), dim3(256), 0, s, (const float*)linv_t, (int)dp, (int)d, tt);
    AE_TRY(launch_status("tri_compact"));
    udinv = mneg;
    linv_t = tt;
  }
  float* z = linv;
  AE_TRY(dense_product(udinv, linv_t, z, (int)d, AE_F32, CONV_TRI_UPPER_LOWER, s));
  if (dtype == AE_BF16) hipLaunchKernelGGL((k_lu_inverse_out<bf16_t>), dim3(lu_grid(dd)), dim3(256), 0, s, (const float*)z, perm, (int)d, (int)d, (bf16_t*)a_inv_out);
  else hipLaunchKernelGGL((k_lu_inverse_out<float>), dim3(lu_grid(dd)), dim3(256), 0, s, (const float*)z, perm, (int)d, (int)d, (float*)a_inv_out);
  return launch_status("lu_inverse_out");
}

extern "C" int model_lu_timing(int enable, double* gemm_ms, int64_t* launches) {
  using namespace ae;
  if (gemm_ms) *gemm_ms = g_timing_ms;
  if (launches) *launches = g_timing_launches;
  if (enable && !g_ev0) {
    AE_HIP(hipEventCreate(&g_ev0));
    AE_HIP(hipEventCreate(&g_ev1));
  }
  g_timing = enable != 0;
  g_timing_ms = 0.0;
  g_timing_launches = 0;
  return AE_OK;
}

extern "C" int model_vol_penalty(const float* log_s, int64_t d, float* value, float* d_log_s, void* stream) {
  using namespace ae;
  if (!log_s || !value) return fail(AE_EINVAL, "model_vol_penalty: null argument");
  if (d < 1 || d > (1 << 24)) return fail(AE_EINVAL, "model_vol_penalty: bad size");
  hipLaunchKernelGGL(k_vol_penalty, dim3(1), dim3(256), 0, (hipStream_t)stream, log_s, (int)d, value, d_log_s);
  return launch_status("vol_penalty");
}
