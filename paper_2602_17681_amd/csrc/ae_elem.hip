// ae_elem.hip — the bandwidth-bound kernels around the convolutions:
// layout changes, weight repacking, per-channel reductions, the fused
// batch-norm / activation / max-pool second pass and its backward, the 2x2
// gradient sum of the upsample, and the MSE loss.  All tensors are
// [rows][C] with channels innermost; each thread moves 16-byte vectors along C.
#include "ae_device.h"
#include "ae_internal.h"

namespace ae {
namespace {

constexpr int NT = 256;

inline int grid_for(int64_t items, int per_block = NT, int cap = 65535 * 8) {
  int64_t g = (items + per_block - 1) / per_block;
  if (g < 1) g = 1;
  if (g > cap) g = cap;
  return (int)g;
}

// ---------------------------------------------------------------------------
// per-sample transpose [rows][cols] -> [cols][rows]
// ---------------------------------------------------------------------------
template <typename TI, typename TO>
__global__ void k_transpose(const TI* __restrict__ in, TO* __restrict__ out, int rows, int cols) {
  __shared__ float tile[32][33];
  const int64_t base = (int64_t)blockIdx.z * rows * cols;
  const int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
  for (int i = ty; i < 32; i += 8) {
    int r = r0 + i, c = c0 + tx;
    if (r < rows && c < cols) tile[i][tx] = Store<TI>::ld(in + base + (int64_t)r * cols + c);
  }
  __syncthreads();
  for (int i = ty; i < 32; i += 8) {
    int c = c0 + i, r = r0 + tx;
    if (r < rows && c < cols) Store<TO>::st(out + base + (int64_t)c * rows + r, tile[tx][i]);
  }
}

template <typename TI, typename TO>
int transpose_impl(const void* in, void* out, int64_t batch, int rows, int cols, hipStream_t s) {
  const int64_t zmax = 65535;
  for (int64_t b0 = 0; b0 < batch; b0 += zmax) {
    int nb = (int)std::min<int64_t>(zmax, batch - b0);
    dim3 grid((cols + 31) / 32, (rows + 31) / 32, nb);
    hipLaunchKernelGGL((k_transpose<TI, TO>), grid, dim3(256), 0, s, (const TI*)in + b0 * rows * cols,
                       (TO*)out + b0 * rows * cols, rows, cols);
  }
  return launch_status("transpose");
}

// ---------------------------------------------------------------------------
// weights: canonical fp32 W[co][ci][r][s] -> packed [co][r][s][ci] (forward) or
// [ci][k-1-r][k-1-s][co] (the convolution that produces the input gradient)
// ---------------------------------------------------------------------------
// Element index of (row, k) of a packed [rows][K] matrix in MFMA fragment order: 32 rows x 32 bytes of K form one
// KiB block, blocks of a row group follow each other along K, and inside a block lane 32 c + r of a wavefront
// finds the 16-byte chunk c of row r at byte 16 (32 c + r) — a wave's operand loads are then 1 KiB contiguous.
template <typename T>
__device__ __forceinline__ int64_t frag_order_index(int row, int64_t kidx, int64_t K) {
  const int64_t kbyte = kidx * (int64_t)sizeof(T), kblocks = (K * (int64_t)sizeof(T)) >> 5;
  const int64_t byte = (((int64_t)(row >> 5) * kblocks + (kbyte >> 5)) << 10) + ((((kbyte >> 4) & 1) * 32 + (row & 31)) << 4) + (kbyte & 15);
  return byte / (int64_t)sizeof(T);
}

template <typename T>
__global__ void k_pack_weights(const float* __restrict__ w, T* __restrict__ wp, int cout, int cin, int k, int dgrad, int frag) {
  const int64_t total = (int64_t)cout * cin * k * k;
  for (int64_t i = (int64_t)blockIdx.x * NT + threadIdx.x; i < total; i += (int64_t)gridDim.x * NT) {
    // i enumerates the PACKED layout so that the stores coalesce
    int64_t src;
    if (!dgrad) {
      int ci = (int)(i % cin); int64_t t = i / cin;
      int s = (int)(t % k); t /= k;
      int r = (int)(t % k); int co = (int)(t / k);
      src = (((int64_t)co * cin + ci) * k + r) * k + s;
    } else {
      int co = (int)(i % cout); int64_t t = i / cout;
      int s = (int)(t % k); t /= k;
      int r = (int)(t % k); int ci = (int)(t / k);
      src = (((int64_t)co * cin + ci) * k + (k - 1 - r)) * k + (k - 1 - s);
    }
    const int64_t K = (int64_t)(dgrad ? cout : cin) * k * k;
    Store<T>::st(wp + (frag ? frag_order_index<T>((int)(i / K), i % K, K) : i), w[src]);
  }
}

// All layers of a pass in one launch: job j owns workgroups [first_block[j], first_block[j+1]).
// Forward layout [co][tap][ci]: 256 (co, ci) pairs per workgroup, ci fastest across threads; a
// thread reads the k*k contiguous taps of its pair and scatters them — loads and stores of a
// wavefront are contiguous.  Input-gradient layout [ci][flipped tap][co]: a workgroup owns a
// 32 x 32 tile of pairs, reads it with ci fastest, turns it in LDS and writes with co fastest.
template <typename T>
__global__ void k_pack_weights_batch(PackBatch pb) {
  __shared__ float tile[32 * 33 * 9];
  int ji = 0;
  while (ji + 1 < pb.n && (int64_t)blockIdx.x >= pb.job[ji + 1].first_block) ++ji;
  const PackJob& J = pb.job[ji];
  const int cout = J.cout, cin = J.cin, kk = J.k * J.k;
  const int64_t lb = (int64_t)blockIdx.x - J.first_block;
  T* __restrict__ wp = (T*)J.wp;
  if (!J.dgrad) {
    const int64_t i = lb * NT + threadIdx.x;
    if (i >= (int64_t)cout * cin) return;
    const int ci = (int)(i % cin), co = (int)(i / cin);
    const float* __restrict__ src = J.w + ((int64_t)co * cin + ci) * kk;
    if (J.frag) {
      for (int t = 0; t < kk; ++t) Store<T>::st(wp + frag_order_index<T>(co, (int64_t)t * cin + ci, (int64_t)kk * cin), src[t]);
      return;
    }
    for (int t = 0; t < kk; ++t) Store<T>::st(wp + ((int64_t)co * kk + t) * cin + ci, src[t]);
    return;
  }
  const int tiles_ci = (cin + 31) / 32;
  const int co0 = (int)(lb / tiles_ci) * 32, ci0 = (int)(lb % tiles_ci) * 32;
  for (int it = 0; it < 4; ++it) {
    const int p = it * NT + threadIdx.x;
    const int ci_l = p & 31, co_l = p >> 5;
    if (co0 + co_l < cout && ci0 + ci_l < cin) {
      const float* __restrict__ src = J.w + ((int64_t)(co0 + co_l) * cin + ci0 + ci_l) * kk;
      for (int t = 0; t < kk; ++t) tile[(co_l * 33 + ci_l) * kk + t] = src[t];
    }
  }
  __syncthreads();
  for (int it = 0; it < 4; ++it) {
    const int p = it * NT + threadIdx.x;
    const int co_l = p & 31, ci_l = p >> 5;
    if (co0 + co_l < cout && ci0 + ci_l < cin) {
      for (int t = 0; t < kk; ++t) {   // tap (r,s) -> (k-1-r, k-1-s)
        const int64_t kidx = (int64_t)(kk - 1 - t) * cout + co0 + co_l;
        const int64_t dst = J.frag ? frag_order_index<T>(ci0 + ci_l, kidx, (int64_t)kk * cout) : (int64_t)(ci0 + ci_l) * kk * cout + kidx;
        Store<T>::st(wp + dst, tile[(co_l * 33 + ci_l) * kk + t]);
      }
    }
  }
}

// ---------------------------------------------------------------------------
// Block-level helper: every thread holds NQ x VEC partial sums for channel group
// `cg` (channels cbase + cg*VEC ...) accumulated over the rows of its row lane
// `rl`; combine over row lanes and write partial_blk[q][channel].
// ---------------------------------------------------------------------------
template <int VEC, int NQ>
__device__ __forceinline__ void block_col_combine(const float (&acc)[NQ][VEC], int cg, int rl, int nrl, int tpr,
                                                  int cbase, int C, float* partial_blk, float* smem, bool active) {
  __syncthreads();
  if (active) {
#pragma unroll
    for (int q = 0; q < NQ; ++q)
#pragma unroll
      for (int v = 0; v < VEC; ++v) smem[((rl * tpr + cg) * NQ + q) * VEC + v] = acc[q][v];
  }
  __syncthreads();
  for (int i = threadIdx.x; i < tpr * NQ * VEC; i += NT) {
    int v = i % VEC, q = (i / VEC) % NQ, g = i / (VEC * NQ);
    int c = cbase + g * VEC + v;
    if (c < C) {
      float t = 0.0f;
      for (int r = 0; r < nrl; ++r) t += smem[((r * tpr + g) * NQ + q) * VEC + v];
      partial_blk[(int64_t)q * C + c] = t;
    }
  }
}

// partial[b][0][c] = sum over the block's rows of x, partial[b][1][c] = sum of x^2
template <typename T, int VEC>
__global__ void k_col_stats(const T* __restrict__ x, int64_t rows, int rpb, int C, float* __restrict__ partial) {
  __shared__ float smem[NT * 2 * VEC];
  const int groups = (C + VEC - 1) / VEC;
  const int tpr = groups < NT ? groups : NT;
  const int nrl = NT / tpr;
  const int cg = threadIdx.x % tpr, rl = threadIdx.x / tpr;
  const bool active = rl < nrl;
  const int64_t r0 = (int64_t)blockIdx.x * rpb;
  const int64_t r1 = r0 + rpb < rows ? r0 + rpb : rows;
  float* pb = partial + (int64_t)blockIdx.x * 2 * C;
  {
    const int cbase = blockIdx.y * tpr * VEC;      // grid.y covers the columns
    float acc[2][VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[0][v] = acc[1][v] = 0.0f;
    const int c = cbase + cg * VEC;
    if (active && c < C) {
#pragma unroll 4
      for (int64_t r = r0 + rl; r < r1; r += nrl) {
        float v[VEC];
        if (VEC == 1) v[0] = Store<T>::ld(x + r * C + c);
        else Store<T>::ldv(x + r * C + c, reinterpret_cast<float(&)[Store<T>::VEC]>(v));
#pragma unroll
        for (int j = 0; j < VEC; ++j) { acc[0][j] += v[j]; acc[1][j] += v[j] * v[j]; }
      }
    }
    block_col_combine<VEC, 2>(acc, cg, rl, nrl, tpr, cbase, C, pb, smem, active);
  }
}

// one block per channel: reduce the partials in double and derive the batch-norm vectors
//   bn_vec = [scale | shift | mean | invstd | c1 | c2], scale = gamma*invstd, shift = beta - mean*scale
// The partials are sums of (x - k) and (x - k)^2 with k = about[c] (0 when about is null): the variance
// E[(x-k)^2] - (E[x-k])^2 does not depend on k, and with k the layer's bias the binary32 partial sums of a
// channel whose mean is far from zero because of its bias no longer cancel against each other.
__global__ void k_bn_finalize(const float* __restrict__ partial, int nblocks, double inv_rows, int C,
                              const float* __restrict__ gamma_beta, const float* __restrict__ stored_mean_var,
                              const float* __restrict__ about, float* __restrict__ bn_vec) {
  __shared__ double sm[NT / 64 + 1];
  const int c = blockIdx.x;
  double mean, var;
  if (stored_mean_var) {
    mean = (double)stored_mean_var[c];
    var = (double)stored_mean_var[C + c];
  } else {
    double s1 = 0.0, s2 = 0.0;
#pragma unroll 8
    for (int b = threadIdx.x; b < nblocks; b += NT) {
      s1 += (double)partial[((int64_t)b * 2) * C + c];
      s2 += (double)partial[((int64_t)b * 2 + 1) * C + c];
    }
    s1 = block_sum<NT>(s1, sm);
    s2 = block_sum<NT>(s2, sm);
    const double dm = s1 * inv_rows;
    var = s2 * inv_rows - dm * dm;
    if (var < 0.0) var = 0.0;
    mean = dm + (about ? (double)about[c] : 0.0);
  }
  if (threadIdx.x == 0) {
    double invstd = 1.0 / sqrt(var + 1e-5);
    double scale = (double)gamma_beta[c] * invstd;
    bn_vec[c] = (float)scale;
    bn_vec[C + c] = (float)((double)gamma_beta[C + c] - mean * scale);
    bn_vec[2 * C + c] = (float)mean;
    bn_vec[3 * C + c] = (float)invstd;
    bn_vec[4 * C + c] = 0.0f;
    bn_vec[5 * C + c] = 0.0f;
  }
}

template <typename T, int VEC>
__device__ __forceinline__ void load_vec(const T* p, float (&v)[VEC]) {
  if (VEC == 1) v[0] = Store<T>::ld(p);
  else Store<T>::ldv(p, reinterpret_cast<float(&)[Store<T>::VEC]>(v));
}
template <typename T, int VEC>
__device__ __forceinline__ void store_vec(T* p, const float (&v)[VEC]) {
  if (VEC == 1) Store<T>::st(p, v[0]);
  else Store<T>::stv(p, reinterpret_cast<const float(&)[Store<T>::VEC]>(v));
}

template <int VEC>
__device__ __forceinline__ void load_f32(const float* p, float (&v)[VEC]) {
#pragma unroll
  for (int j = 0; j < VEC; ++j) v[j] = p[j];
}

// Thread layout shared by the second-pass kernels: a workgroup owns `rpb` consecutive output
// pixels (rows); thread (cg, rl) keeps its channel group's batch-norm vectors in registers and
// walks over rows rl, rl + nrl, ...
struct RowWalk {
  int tpr, nrl, cg, rl;
  bool active;
  __device__ __forceinline__ RowWalk(int groups) {
    tpr = groups < NT ? groups : NT;
    nrl = NT / tpr;
    cg = threadIdx.x % tpr;
    rl = threadIdx.x / tpr;
    active = rl < nrl;
  }
};

// out = pool?( act( scale*raw + shift ) ); bn_vec == null means scale 1, shift 0
template <typename T, int VEC>
__global__ void k_post_forward(const T* __restrict__ raw, const float* __restrict__ bn_vec, T* __restrict__ out,
                               int64_t n, int H, int W, int C, int act, int pool, int rpb) {
  const int groups = C / VEC;
  const int Ho = H >> pool, Wo = W >> pool;
  const int64_t rows = n * Ho * Wo;
  const RowWalk t(groups);
  const int64_t r0 = (int64_t)blockIdx.x * rpb;
  const int64_t r1 = r0 + rpb < rows ? r0 + rpb : rows;
  for (int cbase = 0; cbase < C; cbase += t.tpr * VEC) {
    const int c = cbase + t.cg * VEC;
    if (!t.active || c >= C) continue;
    float sc[VEC], sh[VEC];
    if (bn_vec) { load_f32<VEC>(bn_vec + c, sc); load_f32<VEC>(bn_vec + C + c, sh); }
    else {
#pragma unroll
      for (int j = 0; j < VEC; ++j) { sc[j] = 1.0f; sh[j] = 0.0f; }
    }
#pragma unroll 2
    for (int64_t r = r0 + t.rl; r < r1; r += t.nrl) {
      const unsigned ru = (unsigned)r;              // rows < 2^31 (checked by the launcher): 32-bit divisions
      const int wo = (int)(ru % (unsigned)Wo);
      const unsigned q = ru / (unsigned)Wo;
      const int ho = (int)(q % (unsigned)Ho);
      const int64_t b = q / (unsigned)Ho;
      float res[VEC];
      if (pool) {
        float v[4][VEC];
#pragma unroll
        for (int k = 0; k < 4; ++k) load_vec<T, VEC>(raw + ((b * H + 2 * ho + (k >> 1)) * W + 2 * wo + (k & 1)) * C + c, v[k]);
#pragma unroll
        for (int k = 0; k < 4; ++k)
#pragma unroll
          for (int j = 0; j < VEC; ++j) {
            const float a = apply_act(fmaf(sc[j], v[k][j], sh[j]), act);
            res[j] = (k == 0 || a > res[j]) ? a : res[j];
          }
      } else {
        float v[VEC];
        load_vec<T, VEC>(raw + r * C + c, v);
#pragma unroll
        for (int j = 0; j < VEC; ++j) res[j] = apply_act(fmaf(sc[j], v[j], sh[j]), act);
      }
      store_vec<T, VEC>(out + r * C + c, res);
    }
  }
}

__device__ __forceinline__ float act_grad(float pre, float a, int act) {
  if (act == 1) return pre > 0.0f ? 1.0f : 0.0f;
  if (act == 2) return a * (1.0f - a);
  return 1.0f;
}

template <int VEC>
__device__ __forceinline__ void load_bn4(const float* __restrict__ bn_vec, int C, int c, float (&sc)[VEC], float (&sh)[VEC],
                                         float (&mu)[VEC], float (&is)[VEC]) {
  if (bn_vec) {
    load_f32<VEC>(bn_vec + c, sc); load_f32<VEC>(bn_vec + C + c, sh);
    load_f32<VEC>(bn_vec + 2 * C + c, mu); load_f32<VEC>(bn_vec + 3 * C + c, is);
  } else {
#pragma unroll
    for (int j = 0; j < VEC; ++j) { sc[j] = 1.0f; sh[j] = 0.0f; mu[j] = 0.0f; is[j] = 1.0f; }
  }
}

// Backward of the second pass, shared by the reduction and the apply kernels: for
// one output pixel (a 2x2 window when pooling) and VEC channels, find the routed
// gradient dy_j at each raw position j and xhat_j.  Everything is unrolled at compile
// time so that the per-position arrays stay in registers.
template <typename T, int VEC, bool POOL>
struct PostBwdWindow {
  static constexpr int NQ = POOL ? 4 : 1;
  float dy[NQ][VEC];
  float xh[NQ][VEC];
  __device__ __forceinline__ void compute(const T* __restrict__ raw, const T* __restrict__ dout, const float (&sc)[VEC],
                                          const float (&sh)[VEC], const float (&mu)[VEC], const float (&is)[VEC],
                                          int64_t b, int ho, int wo, int H, int W, int C, int c, int act) {
    const int Ho = POOL ? H >> 1 : H, Wo = POOL ? W >> 1 : W;
    float g[VEC];
    load_vec<T, VEC>(dout + ((b * Ho + ho) * Wo + wo) * C + c, g);
    float best[VEC], dbest[VEC];
    int arg[VEC];
    float v[NQ][VEC];
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
      const int hh = POOL ? 2 * ho + (q >> 1) : ho, ww = POOL ? 2 * wo + (q & 1) : wo;
      load_vec<T, VEC>(raw + ((b * H + hh) * W + ww) * C + c, v[q]);
    }
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
#pragma unroll
      for (int j = 0; j < VEC; ++j) {
        const float pre = fmaf(sc[j], v[q][j], sh[j]);
        const float a = apply_act(pre, act);
        xh[q][j] = (v[q][j] - mu[j]) * is[j];
        if (q == 0 || a > best[j]) { best[j] = a; arg[j] = q; dbest[j] = act_grad(pre, a, act); }
      }
    }
#pragma unroll
    for (int q = 0; q < NQ; ++q)
#pragma unroll
      for (int j = 0; j < VEC; ++j) dy[q][j] = (arg[j] == q) ? g[j] * dbest[j] : 0.0f;
  }
};

// partial[b][0][c] = sum dy, partial[b][1][c] = sum dy*xhat over the block's output pixels.
// With ReLU (out_act given) the sums need no pass over the conv output: the gradient reaches only
// the position that produced the stored activation a = max(pre, 0) > 0 of each (pooled) output,
// where pre = a, and xhat follows from pre = scale*raw + shift: xhat = a*p1 + p0 with
// p1 = invstd/scale, p0 = -(shift/scale + mean)*invstd.  Channels with scale == 0 take the
// general path.
template <typename T, int VEC, bool POOL>
__global__ void k_post_bwd_reduce(const T* __restrict__ raw, const T* __restrict__ dout, const T* __restrict__ out_act,
                                  const float* __restrict__ bn_vec, int64_t n, int H, int W, int C, int act,
                                  int rpb, float* __restrict__ partial) {
  __shared__ float smem[NT * 2 * VEC];
  const int Ho = POOL ? H >> 1 : H, Wo = POOL ? W >> 1 : W;
  const int64_t rows = n * Ho * Wo;
  const int groups = (C + VEC - 1) / VEC;
  const int tpr = groups < NT ? groups : NT;
  const int nrl = NT / tpr;
  const int cg = threadIdx.x % tpr, rl = threadIdx.x / tpr;
  const bool active = rl < nrl;
  const int64_t r0 = (int64_t)blockIdx.x * rpb;
  const int64_t r1 = r0 + rpb < rows ? r0 + rpb : rows;
  float* pb = partial + (int64_t)blockIdx.x * 2 * C;
  for (int cbase = 0; cbase < C; cbase += tpr * VEC) {
    float acc[2][VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[0][v] = acc[1][v] = 0.0f;
    const int c = cbase + cg * VEC;
    if (active && c < C) {
      float sc[VEC], sh[VEC], mu[VEC], is[VEC];
      load_bn4<VEC>(bn_vec, C, c, sc, sh, mu, is);
      bool from_act = out_act != nullptr;
#pragma unroll
      for (int j = 0; j < VEC; ++j) from_act = from_act && sc[j] != 0.0f;
      if (from_act) {
        float p1[VEC], p0[VEC];
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
          const float inv = 1.0f / sc[j];
          p1[j] = is[j] * inv;
          p0[j] = -(sh[j] * inv + mu[j]) * is[j];
        }
#pragma unroll 4
        for (int64_t r = r0 + rl; r < r1; r += nrl) {
          float a[VEC], g[VEC];
          load_vec<T, VEC>(out_act + r * C + c, a);
          load_vec<T, VEC>(dout + r * C + c, g);
#pragma unroll
          for (int j = 0; j < VEC; ++j) {
            const float dyv = a[j] > 0.0f ? g[j] : 0.0f;
            acc[0][j] += dyv;
            acc[1][j] = fmaf(dyv, fmaf(a[j], p1[j], p0[j]), acc[1][j]);
          }
        }
      } else {
        for (int64_t r = r0 + rl; r < r1; r += nrl) {
          const unsigned ru = (unsigned)r;              // rows < 2^31 (checked by the launcher)
          const int wo = (int)(ru % (unsigned)Wo);
          const int ho = (int)((ru / (unsigned)Wo) % (unsigned)Ho);
          const int64_t b = ru / ((unsigned)Wo * (unsigned)Ho);
          PostBwdWindow<T, VEC, POOL> win;
          win.compute(raw, dout, sc, sh, mu, is, b, ho, wo, H, W, C, c, act);
#pragma unroll
          for (int q = 0; q < PostBwdWindow<T, VEC, POOL>::NQ; ++q)
#pragma unroll
            for (int j = 0; j < VEC; ++j) { acc[0][j] += win.dy[q][j]; acc[1][j] = fmaf(win.dy[q][j], win.xh[q][j], acc[1][j]); }
        }
      }
    }
    block_col_combine<VEC, 2>(acc, cg, rl, nrl, tpr, cbase, C, pb, smem, active);
  }
}

// one block per channel: dgamma = sum dy*xhat, dbeta = sum dy; c1 = dbeta/M, c2 = dgamma/M (batch statistics)
// fix_raw / fix_dout (bfloat16 [n][H][W][C] and [n][H>>pool][W>>pool][C], optional): the partials came from an
// epilogue that derives xhat from the saved ReLU output, which a channel of scale 0 does not allow; such a channel's
// sums are taken here from the definition (all pre-activations equal the shift: the first position of a window wins
// and passes the gradient if the shift is positive).
__global__ void k_bn_bwd_finalize(const float* __restrict__ partial, int nblocks, double inv_rows, int C,
                                  float* __restrict__ bn_vec, float* __restrict__ dgamma_dbeta,
                                  float* __restrict__ dbias, int batch_stats, int stored_slots,
                                  const bf16_t* __restrict__ fix_raw, const bf16_t* __restrict__ fix_dout, int64_t n,
                                  int H, int W, int pool) {
  __shared__ double sm[NT / 64 + 1];
  const int c = blockIdx.x;
  double s1 = 0.0, s2 = 0.0;
  if (fix_raw && bn_vec[c] == 0.0f) {
    if (bn_vec[C + c] > 0.0f) {
      const int Ho = H >> pool, Wo = W >> pool;
      const float mu = bn_vec[2 * C + c], is = bn_vec[3 * C + c];
      for (int64_t r = threadIdx.x; r < n * Ho * Wo; r += NT) {
        const int wo = (int)(r % Wo);
        const int ho = (int)((r / Wo) % Ho);
        const int64_t b = r / ((int64_t)Wo * Ho);
        const float g = bf16_to_f32(fix_dout[r * C + c]);
        const float x = bf16_to_f32(fix_raw[((b * H + ((int64_t)ho << pool)) * W + ((int64_t)wo << pool)) * C + c]);
        s1 += (double)g;
        s2 += (double)(g * ((x - mu) * is));
      }
    }
  } else {
#pragma unroll 8
    for (int b = threadIdx.x; b < nblocks; b += NT) {
      s1 += (double)partial[((int64_t)b * 2) * C + c];
      s2 += (double)partial[((int64_t)b * 2 + 1) * C + c];
    }
  }
  s1 = block_sum<NT>(s1, sm);
  s2 = block_sum<NT>(s2, sm);
  if (threadIdx.x == 0) {
    dgamma_dbeta[c] = (float)s2;
    dgamma_dbeta[C + c] = (float)s1;
    if (stored_slots) { dgamma_dbeta[2 * C + c] = 0.0f; dgamma_dbeta[3 * C + c] = 0.0f; }
    bn_vec[4 * C + c] = batch_stats ? (float)(s1 * inv_rows) : 0.0f;
    bn_vec[5 * C + c] = batch_stats ? (float)(s2 * inv_rows) : 0.0f;
    // gradient of the bias of the conv that feeds this batch-norm: sum over pixels of the
    // conv-output gradient = scale*(sum dy - M*c1 - c2*sum xhat).  With batch statistics
    // sum xhat = 0 and M*c1 = sum dy: exactly zero.  With stored statistics: scale * sum dy.
    if (dbias) dbias[c] = batch_stats ? 0.0f : (float)((double)bn_vec[c] * s1);
  }
}

// draw_j = scale*(dy_j - c1 - xhat_j*c2) with batch-norm, dy_j without
template <typename T, int VEC, bool POOL>
__global__ void k_post_bwd_apply(const T* __restrict__ raw, const T* __restrict__ dout,
                                 const float* __restrict__ bn_vec, T* __restrict__ draw, int64_t n, int H, int W,
                                 int C, int act, int has_bn, int rpb) {
  const int groups = C / VEC;
  const int Ho = POOL ? H >> 1 : H, Wo = POOL ? W >> 1 : W;
  const int64_t rows = n * Ho * Wo;
  const RowWalk t(groups);
  const int64_t r0 = (int64_t)blockIdx.x * rpb;
  const int64_t r1 = r0 + rpb < rows ? r0 + rpb : rows;
  for (int cbase = 0; cbase < C; cbase += t.tpr * VEC) {
    const int c = cbase + t.cg * VEC;
    if (!t.active || c >= C) continue;
    float sc[VEC], sh[VEC], mu[VEC], is[VEC], c1[VEC], c2[VEC];
    load_bn4<VEC>(bn_vec, C, c, sc, sh, mu, is);
    if (has_bn) { load_f32<VEC>(bn_vec + 4 * C + c, c1); load_f32<VEC>(bn_vec + 5 * C + c, c2); }
    for (int64_t r = r0 + t.rl; r < r1; r += t.nrl) {
      const unsigned ru = (unsigned)r;              // rows < 2^31 (checked by the launcher): 32-bit divisions
      const int wo = (int)(ru % (unsigned)Wo);
      const unsigned q_ = ru / (unsigned)Wo;
      const int ho = (int)(q_ % (unsigned)Ho);
      const int64_t b = q_ / (unsigned)Ho;
      PostBwdWindow<T, VEC, POOL> win;
      win.compute(raw, dout, sc, sh, mu, is, b, ho, wo, H, W, C, c, act);
#pragma unroll
      for (int q = 0; q < PostBwdWindow<T, VEC, POOL>::NQ; ++q) {
        float o[VEC];
#pragma unroll
        for (int j = 0; j < VEC; ++j)
          o[j] = has_bn ? sc[j] * (win.dy[q][j] - c1[j] - win.xh[q][j] * c2[j]) : win.dy[q][j];
        const int hh = POOL ? 2 * ho + (q >> 1) : ho, ww = POOL ? 2 * wo + (q & 1) : wo;
        store_vec<T, VEC>(draw + ((b * H + hh) * W + ww) * C + c, o);
      }
    }
  }
}

// draw = dout * act'(out), from the saved activation output
template <typename T>
__global__ void k_act_bwd(const T* __restrict__ out, const float* __restrict__ out_f32, const T* __restrict__ dout,
                          T* __restrict__ draw, int64_t n, int act) {
  for (int64_t i = (int64_t)blockIdx.x * NT + threadIdx.x; i < n; i += (int64_t)gridDim.x * NT) {
    float a = out_f32 ? out_f32[i] : Store<T>::ld(out + i), g = Store<T>::ld(dout + i);
    float d = act == 1 ? (a > 0.0f ? 1.0f : 0.0f) : (act == 2 ? a * (1.0f - a) : 1.0f);
    Store<T>::st(draw + i, g * d);
  }
}

// draw = dout * act'(out) for a [rows][C] tensor, and partial[b][0][c] = column sums of draw
// over the block's rows (the bias gradient) in the same pass
template <typename T, int VEC>
__global__ void k_act_bwd_colsum(const T* __restrict__ out, const float* __restrict__ out_f32,
                                 const T* __restrict__ dout, T* __restrict__ draw, int64_t rows, int rpb, int C,
                                 int act, float* __restrict__ partial) {
  __shared__ float smem[NT * VEC];
  const int groups = (C + VEC - 1) / VEC;
  const int tpr = groups < NT ? groups : NT;
  const int nrl = NT / tpr;
  const int cg = threadIdx.x % tpr, rl = threadIdx.x / tpr;
  const bool active = rl < nrl;
  const int64_t r0 = (int64_t)blockIdx.x * rpb;
  const int64_t r1 = r0 + rpb < rows ? r0 + rpb : rows;
  float* pb = partial + (int64_t)blockIdx.x * 2 * C;
  for (int cbase = 0; cbase < C; cbase += tpr * VEC) {
    float acc[1][VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[0][v] = 0.0f;
    const int c = cbase + cg * VEC;
    if (active && c < C) {
      for (int64_t r = r0 + rl; r < r1; r += nrl) {
        float a[VEC], g[VEC], d[VEC];
        if (out_f32) load_f32<VEC>(out_f32 + r * C + c, a);
        else load_vec<T, VEC>(out + r * C + c, a);
        load_vec<T, VEC>(dout + r * C + c, g);
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
          const float dd = act == 1 ? (a[j] > 0.0f ? 1.0f : 0.0f) : (act == 2 ? a[j] * (1.0f - a[j]) : 1.0f);
          d[j] = round_to_storage<T>(g[j] * dd);
          acc[0][j] += d[j];
        }
        store_vec<T, VEC>(draw + r * C + c, d);
      }
    }
    block_col_combine<VEC, 1>(acc, cg, rl, nrl, tpr, cbase, C, pb, smem, active);
  }
}

__global__ void k_colsum_finalize(const float* __restrict__ partial, int nblocks, int C, float* __restrict__ out) {
  __shared__ double sm[NT / 64 + 1];
  const int c = blockIdx.x;
  double s1 = 0.0;
#pragma unroll 8
  for (int b = threadIdx.x; b < nblocks; b += NT) s1 += (double)partial[((int64_t)b * 2) * C + c];
  s1 = block_sum<NT>(s1, sm);
  if (threadIdx.x == 0) out[c] = (float)s1;
}

// dx[n,i,j,c] = sum of the four copies' gradients
template <typename T, int VEC>
__global__ void k_upsum(const T* __restrict__ dfull, T* __restrict__ dx, int64_t n, int H, int W, int C) {
  const int groups = C / VEC;
  const int64_t total = n * H * W * groups;
  for (int64_t it = (int64_t)blockIdx.x * NT + threadIdx.x; it < total; it += (int64_t)gridDim.x * NT) {
    const unsigned iu = (unsigned)it;
    const int c = (int)(iu % (unsigned)groups) * VEC;
    unsigned p = iu / (unsigned)groups;
    const int j = (int)(p % (unsigned)W); p /= (unsigned)W;
    const int i = (int)(p % (unsigned)H);
    const int64_t b = p / (unsigned)H;
    float acc[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = 0.0f;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      float v[VEC];
      load_vec<T, VEC>(dfull + ((b * 2 * H + 2 * i + (q >> 1)) * 2 * W + 2 * j + (q & 1)) * C + c, v);
#pragma unroll
      for (int t = 0; t < VEC; ++t) acc[t] += v[t];
    }
    store_vec<T, VEC>(dx + ((b * H + i) * W + j) * C + c, acc);
  }
}

__global__ void k_fill_zero(uint32_t* p, int64_t n_words) {
  for (int64_t i = (int64_t)blockIdx.x * NT + threadIdx.x; i < n_words; i += (int64_t)gridDim.x * NT) p[i] = 0u;
}

// loss += sum((y-t)^2)/n over the block's slice; dy = 2 (y-t)/n.  16 bytes per thread and
// access when the tensors allow it (vec), several independent accesses in flight.
template <typename T>
__global__ void k_mse(const T* __restrict__ y, const T* __restrict__ t, int64_t n, float inv_n, float* __restrict__ loss,
                      T* __restrict__ dy, int vec) {
  __shared__ float sm[NT / 64 + 1];
  constexpr int V = Store<T>::VEC;
  float acc = 0.0f;
  const int64_t nv = vec ? n / V : 0;
#pragma unroll 4
  for (int64_t i = (int64_t)blockIdx.x * NT + threadIdx.x; i < nv; i += (int64_t)gridDim.x * NT) {
    float a[V], b[V], d[V];
    Store<T>::ldv(y + i * V, a);
    Store<T>::ldv(t + i * V, b);
#pragma unroll
    for (int j = 0; j < V; ++j) { d[j] = a[j] - b[j]; acc = fmaf(d[j], d[j], acc); d[j] = 2.0f * d[j] * inv_n; }
    if (dy) Store<T>::stv(dy + i * V, d);
  }
  for (int64_t i = nv * V + (int64_t)blockIdx.x * NT + threadIdx.x; i < n; i += (int64_t)gridDim.x * NT) {
    float d = Store<T>::ld(y + i) - Store<T>::ld(t + i);
    acc = fmaf(d, d, acc);
    if (dy) Store<T>::st(dy + i, 2.0f * d * inv_n);
  }
  acc = block_sum<NT>(acc, sm);
  if (threadIdx.x == 0) atomicAdd(loss, acc * inv_n);
}

// Summed weights of the two cheaper forms of a 3x3 convolution behind a x2 upsample.
// Rows (or columns) r of the filter that read the same stored input row collapse:
//   forward, output parity a:  input offset di = 0 gets rows {0} (a = 0) or {0,1} (a = 1),
//                              di = 1 gets rows {1,2} (a = 0) or {2} (a = 1);
//   input gradient, tap e = 0..3 (output row 2i + e - 1):  rows {2}, {1,2}, {0,1}, {0}.
// One thread per (co, ci) pair reads the nine weights and writes all sixteen sums (added in
// fp32 in ascending (r, s) order, then rounded once to the storage type).
//   geom 1: wp[phase][co][di][dj][ci]      geom 2: wp[ci][e][f][co]
template <typename T>
__global__ void k_pack_weights_up(const float* __restrict__ w, T* __restrict__ wp, int cout, int cin, int geom) {
  const int64_t total = (int64_t)cout * cin;
  for (int64_t idx = (int64_t)blockIdx.x * NT + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * NT) {
    int co, ci;
    if (geom == 1) { ci = (int)(idx % cin); co = (int)(idx / cin); }
    else { co = (int)(idx % cout); ci = (int)(idx / cout); }
    float f[3][3];
    const float* src = w + ((int64_t)co * cin + ci) * 9;
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
      for (int q = 0; q < 3; ++q) f[r][q] = src[r * 3 + q];
    if (geom == 1) {
#pragma unroll
      for (int ph = 0; ph < 4; ++ph) {
        const int a = ph >> 1, b = ph & 1;
#pragma unroll
        for (int di = 0; di < 2; ++di)
#pragma unroll
          for (int dj = 0; dj < 2; ++dj) {
            const int r0 = di == 0 ? 0 : (a == 0 ? 1 : 2), r1 = di == 0 ? (a == 0 ? 0 : 1) : 2;
            const int s0 = dj == 0 ? 0 : (b == 0 ? 1 : 2), s1 = dj == 0 ? (b == 0 ? 0 : 1) : 2;
            float t = 0.0f;
#pragma unroll
            for (int r = 0; r < 3; ++r)
#pragma unroll
              for (int q = 0; q < 3; ++q)
                if (r >= r0 && r <= r1 && q >= s0 && q <= s1) t += f[r][q];
            Store<T>::st(wp + ((((int64_t)ph * cout + co) * 2 + di) * 2 + dj) * cin + ci, t);
          }
      }
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int r0 = e == 0 ? 2 : (e == 1 ? 1 : 0), r1 = e == 0 ? 2 : (e == 1 ? 2 : (e == 2 ? 1 : 0));
          const int s0 = g == 0 ? 2 : (g == 1 ? 1 : 0), s1 = g == 0 ? 2 : (g == 1 ? 2 : (g == 2 ? 1 : 0));
          float t = 0.0f;
#pragma unroll
          for (int r = 0; r < 3; ++r)
#pragma unroll
            for (int q = 0; q < 3; ++q)
              if (r >= r0 && r <= r1 && q >= s0 && q <= s1) t += f[r][q];
          Store<T>::st(wp + (((int64_t)ci * 4 + e) * 4 + g) * cout + co, t);
        }
    }
  }
}

}  // namespace

// ===========================================================================
// launchers
// ===========================================================================
#define DISPATCH_T(dtype, ...)                                  \
  do {                                                          \
    if ((dtype) == AE_BF16) { typedef bf16_t T; __VA_ARGS__; }  \
    else { typedef float T; __VA_ARGS__; }                      \
  } while (0)

// rows per workgroup of the row-walking kernels: up to 8 rows per thread, fewer when that
// would leave the machine with fewer than about 2048 workgroups
static int walk_rows_per_block(int64_t rows, int groups) {
  const int tpr = groups < NT ? groups : NT;
  const int nrl = NT / tpr;
  int it = 8;
  while (it > 1 && rows / ((int64_t)nrl * it) < 2048) it >>= 1;
  return nrl * it;
}

#define DISPATCH_T_VEC(dtype, C, ...)                                                       \
  do {                                                                                      \
    if ((dtype) == AE_BF16) {                                                               \
      typedef bf16_t T;                                                                     \
      if ((C) % 8 == 0) { constexpr int VEC = 8; __VA_ARGS__; } else { constexpr int VEC = 1; __VA_ARGS__; } \
    } else {                                                                                \
      typedef float T;                                                                      \
      if ((C) % 4 == 0) { constexpr int VEC = 4; __VA_ARGS__; } else { constexpr int VEC = 1; __VA_ARGS__; } \
    }                                                                                       \
  } while (0)

int launch_transpose(const void* in, void* out, int64_t batch, int rows, int cols, int dtype, hipStream_t s) {
  if (dtype == AE_BF16) return transpose_impl<bf16_t, bf16_t>(in, out, batch, rows, cols, s);
  return transpose_impl<float, float>(in, out, batch, rows, cols, s);
}

int launch_to_f32_nchw(const void* in_nhwc, float* out_nchw, int64_t batch, int c, int hw, int dtype, hipStream_t s) {
  // stored [hw][c] -> [c][hw]
  if (dtype == AE_BF16) return transpose_impl<bf16_t, float>(in_nhwc, out_nchw, batch, hw, c, s);
  return transpose_impl<float, float>(in_nhwc, out_nchw, batch, hw, c, s);
}

// 1x1 layers: the forward packing is a plain conversion, the input-gradient packing a transpose
template <typename T>
__global__ void k_convert_f32(const float* __restrict__ w, T* __restrict__ wp, int64_t n) {
  const int64_t n8 = n / 8;
#pragma unroll 2
  for (int64_t i = (int64_t)blockIdx.x * NT + threadIdx.x; i < n8; i += (int64_t)gridDim.x * NT) {
    const float4 a = *reinterpret_cast<const float4*>(w + i * 8), b = *reinterpret_cast<const float4*>(w + i * 8 + 4);
    Store<T>::st(wp + i * 8 + 0, a.x); Store<T>::st(wp + i * 8 + 1, a.y); Store<T>::st(wp + i * 8 + 2, a.z); Store<T>::st(wp + i * 8 + 3, a.w);
    Store<T>::st(wp + i * 8 + 4, b.x); Store<T>::st(wp + i * 8 + 5, b.y); Store<T>::st(wp + i * 8 + 6, b.z); Store<T>::st(wp + i * 8 + 7, b.w);
  }
  for (int64_t i = n8 * 8 + (int64_t)blockIdx.x * NT + threadIdx.x; i < n; i += (int64_t)gridDim.x * NT) Store<T>::st(wp + i, w[i]);
}

int launch_pack_weights_1x1(const float* w, void* wp, int cout, int cin, int dtype, bool for_dgrad, hipStream_t s) {
  if (for_dgrad) {
    if (dtype == AE_BF16) return transpose_impl<float, bf16_t>(w, wp, 1, cout, cin, s);
    return transpose_impl<float, float>(w, wp, 1, cout, cin, s);
  }
  const int64_t n = (int64_t)cout * cin;
  const bool aligned = (((uintptr_t)w | (uintptr_t)wp) & 15) == 0;
  if (!aligned) return launch_pack_weights(w, wp, cout, cin, 1, dtype, false, s);
  DISPATCH_T(dtype, hipLaunchKernelGGL((k_convert_f32<T>), dim3(grid_for(n, NT * 8, 16384)), dim3(NT), 0, s, w, (T*)wp, n));
  return launch_status("convert_f32");
}

int launch_pack_weights_batch(PackBatch& pb, int dtype, hipStream_t s) {
  if (pb.n <= 0) return AE_OK;
  int64_t blocks = 0;
  for (int j = 0; j < pb.n; ++j) {
    pb.job[j].first_block = blocks;
    const int64_t pairs = (int64_t)pb.job[j].cout * pb.job[j].cin;
    if (pb.job[j].k > 3) return fail(AE_EINVAL, "pack_weights: filters larger than 3x3 are not batched");
    blocks += pb.job[j].dgrad ? (int64_t)((pb.job[j].cout + 31) / 32) * ((pb.job[j].cin + 31) / 32) : (pairs + NT - 1) / NT;
  }
  if (blocks > 0x7FFFFFFF) return fail(AE_EINVAL, "pack_weights: too many elements");
  DISPATCH_T(dtype, hipLaunchKernelGGL((k_pack_weights_batch<T>), dim3((unsigned)blocks), dim3(NT), 0, s, pb));
  return launch_status("pack_weights_batch");
}

int launch_pack_weights(const float* w, void* wp, int cout, int cin, int k, int dtype, bool for_dgrad, hipStream_t s, bool frag) {
  int64_t total = (int64_t)cout * cin * k * k;
  if (frag && ((for_dgrad ? cin : cout) % 32 != 0 || ((int64_t)(for_dgrad ? cout : cin) * k * k * (int64_t)dtype_size(dtype)) % 32 != 0))
    return fail(AE_EINVAL, "pack_weights: fragment order needs rows in 32s and K in 32-byte blocks");
  DISPATCH_T(dtype, hipLaunchKernelGGL((k_pack_weights<T>), dim3(grid_for(total, NT, 4096)), dim3(NT), 0, s, w, (T*)wp,
                                       cout, cin, k, for_dgrad ? 1 : 0, frag ? 1 : 0));
  return launch_status("pack_weights");
}

int launch_pack_weights_up(const float* w, void* wp, int cout, int cin, int dtype, int geom, hipStream_t s) {
  if (geom != CONV_UP_PHASES && geom != CONV_UP_DGRAD) return fail(AE_EINVAL, "pack_weights_up: bad form");
  const int64_t total = (int64_t)cout * cin;
  DISPATCH_T(dtype, hipLaunchKernelGGL((k_pack_weights_up<T>), dim3(grid_for(total, NT, 4096)), dim3(NT), 0, s, w, (T*)wp,
                                       cout, cin, geom));
  return launch_status("pack_weights_up");
}

int launch_col_stats(const void* x, int64_t rows, int c, int dtype, float* partial, hipStream_t s) {
  const int rpb = reduce_rows_per_block(rows);
  const int nblocks = reduce_blocks(rows);
  DISPATCH_T_VEC(dtype, c, {
    const int groups = (c + VEC - 1) / VEC;
    const int tpr = groups < NT ? groups : NT;
    hipLaunchKernelGGL((k_col_stats<T, VEC>), dim3(nblocks, (c + tpr * VEC - 1) / (tpr * VEC)), dim3(NT), 0, s, (const T*)x,
                       rows, rpb, c, partial);
  });
  return launch_status("col_stats");
}

int launch_bn_finalize(const float* partial, int nblocks, int64_t rows, int c, const float* gamma_beta,
                       const float* stored_mean_var, const float* about, float* bn_vec, hipStream_t s) {
  hipLaunchKernelGGL(k_bn_finalize, dim3(c), dim3(NT), 0, s, partial, nblocks, 1.0 / (double)rows, c, gamma_beta,
                     stored_mean_var, about, bn_vec);
  return launch_status("bn_finalize");
}

int launch_post_forward(const void* raw, const float* bn_vec, void* out, int64_t n, int h, int w, int c, int act,
                        int pool, int dtype, hipStream_t s) {
  DISPATCH_T_VEC(dtype, c, {
    const int64_t rows = n * (h >> pool) * (w >> pool);
    if (rows * (c / VEC) >= 0x7FFFFFFF) return fail(AE_EINVAL, "post_forward: tensor too large");
    const int rpb = walk_rows_per_block(rows, c / VEC);
    hipLaunchKernelGGL((k_post_forward<T, VEC>), dim3((unsigned)((rows + rpb - 1) / rpb)), dim3(NT), 0, s, (const T*)raw,
                       bn_vec, (T*)out, n, h, w, c, act, pool, rpb);
  });
  return launch_status("post_forward");
}

// out_act: the step's stored output (after activation and pooling); used when act is ReLU
int launch_post_bwd_reduce(const void* raw, const void* dout, const void* out_act, const float* bn_vec, int64_t n, int h,
                           int w, int c, int act, int pool, int dtype, float* partial, hipStream_t s) {
  if (act != ACT_RELU || !bn_vec) out_act = nullptr;
  int64_t rows = n * (h >> pool) * (w >> pool);
  if (rows >= 0x7FFFFFFF) return fail(AE_EINVAL, "post_bwd_reduce: tensor too large");
  const int rpb = reduce_rows_per_block(rows);
  const int nblocks = reduce_blocks(rows);
  DISPATCH_T_VEC(dtype, c, {
    if (pool)
      hipLaunchKernelGGL((k_post_bwd_reduce<T, VEC, true>), dim3(nblocks), dim3(NT), 0, s, (const T*)raw,
                         (const T*)dout, (const T*)out_act, bn_vec, n, h, w, c, act, rpb, partial);
    else
      hipLaunchKernelGGL((k_post_bwd_reduce<T, VEC, false>), dim3(nblocks), dim3(NT), 0, s, (const T*)raw,
                         (const T*)dout, (const T*)out_act, bn_vec, n, h, w, c, act, rpb, partial);
  });
  return launch_status("post_bwd_reduce");
}

int launch_bn_bwd_finalize(const float* partial, int nblocks, int64_t rows, int c, float* dbias, float* bn_vec,
                           float* dgamma_dbeta, int batch_stats, hipStream_t s, const void* fix_raw, const void* fix_dout,
                           int64_t n, int h, int w, int pool) {
  hipLaunchKernelGGL(k_bn_bwd_finalize, dim3(c), dim3(NT), 0, s, partial, nblocks, 1.0 / (double)rows, c, bn_vec,
                     dgamma_dbeta, dbias, batch_stats, batch_stats ? 0 : 1, (const bf16_t*)fix_raw, (const bf16_t*)fix_dout,
                     n, h, w, pool);
  return launch_status("bn_bwd_finalize");
}

int launch_post_bwd_apply(const void* raw, const void* dout, const float* bn_vec, void* draw, int64_t n, int h, int w,
                          int c, int act, int pool, int has_bn, int dtype, hipStream_t s) {
  DISPATCH_T_VEC(dtype, c, {
    const int64_t rows = n * (h >> pool) * (w >> pool);
    if (rows * (c / VEC) >= 0x7FFFFFFF) return fail(AE_EINVAL, "post_bwd_apply: tensor too large");
    const int rpb = walk_rows_per_block(rows, c / VEC);
    const dim3 grid((unsigned)((rows + rpb - 1) / rpb));
    if (pool)
      hipLaunchKernelGGL((k_post_bwd_apply<T, VEC, true>), grid, dim3(NT), 0, s, (const T*)raw, (const T*)dout, bn_vec,
                         (T*)draw, n, h, w, c, act, has_bn, rpb);
    else
      hipLaunchKernelGGL((k_post_bwd_apply<T, VEC, false>), grid, dim3(NT), 0, s, (const T*)raw, (const T*)dout, bn_vec,
                         (T*)draw, n, h, w, c, act, has_bn, rpb);
  });
  return launch_status("post_bwd_apply");
}

int launch_act_bwd(const void* out, const float* out_f32, const void* dout, void* draw, int64_t n_elem, int act,
                   int dtype, hipStream_t s) {
  DISPATCH_T(dtype, hipLaunchKernelGGL((k_act_bwd<T>), dim3(grid_for(n_elem, NT, 16384)), dim3(NT), 0, s,
                                       (const T*)out, out_f32, (const T*)dout, (T*)draw, n_elem, act));
  return launch_status("act_bwd");
}

int launch_act_bwd_colsum(const void* out, const float* out_f32, const void* dout, void* draw, int64_t rows, int c,
                          int act, int dtype, float* partial, hipStream_t s) {
  const int rpb = reduce_rows_per_block(rows);
  const int nblocks = reduce_blocks(rows);
  DISPATCH_T_VEC(dtype, c, hipLaunchKernelGGL((k_act_bwd_colsum<T, VEC>), dim3(nblocks), dim3(NT), 0, s, (const T*)out,
                                              out_f32, (const T*)dout, (T*)draw, rows, rpb, c, act, partial));
  return launch_status("act_bwd_colsum");
}

int launch_colsum_finalize(const float* partial, int nblocks, int c, float* out, hipStream_t s) {
  hipLaunchKernelGGL(k_colsum_finalize, dim3(c), dim3(NT), 0, s, partial, nblocks, c, out);
  return launch_status("colsum_finalize");
}

int launch_upsum(const void* dfull, void* dx, int64_t n, int h, int w, int c, int dtype, hipStream_t s) {
  DISPATCH_T_VEC(dtype, c, {
    int64_t items = n * h * w * (c / VEC);
    if (items >= 0x7FFFFFFF) return fail(AE_EINVAL, "upsum: tensor too large");
    hipLaunchKernelGGL((k_upsum<T, VEC>), dim3(grid_for(items)), dim3(NT), 0, s, (const T*)dfull, (T*)dx, n, h, w, c);
  });
  return launch_status("upsum");
}

int launch_fill_zero(void* p, int64_t bytes, hipStream_t s) {
  int64_t words = (bytes + 3) / 4;  // buffers are 4-byte multiples
  hipLaunchKernelGGL(k_fill_zero, dim3(grid_for(words, NT, 8192)), dim3(NT), 0, s, (uint32_t*)p, words);
  return launch_status("fill_zero");
}

int launch_mse(const void* y, const void* t, int64_t n, int dtype, float* loss, void* dy, hipStream_t s) {
  AE_TRY(launch_fill_zero(loss, 4, s));
  const int vec = (((uintptr_t)y | (uintptr_t)t | (uintptr_t)dy) & 15) == 0 ? 1 : 0;
  // at most 512 workgroups: each ends with one atomic add to the loss scalar, and same-address atomics serialise
  DISPATCH_T(dtype, hipLaunchKernelGGL((k_mse<T>), dim3(grid_for(n, NT * 16, 512)), dim3(NT), 0, s, (const T*)y,
                                       (const T*)t, n, (float)(1.0 / (double)n), loss, (T*)dy, vec));
  return launch_status("mse");
}

}  // namespace ae
