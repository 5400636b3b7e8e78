// ae_conv_thin.hip — 3x3 convolutions with a "thin" side: the first layer (1..4
// input channels) and the last layer (1..4 output channels) of the autoencoders, for
// fp32 models and for the shapes the matrix-core versions (ae_conv_thin_mfma.hip) do not take.
// With K = 9*C_in <= 36 or N = C_out <= 4 these layers are bound by HBM, not by the
// matrix cores:
//
//   thin-in  conv : out[m][cw]  = b[cw] + sum_{ct,r,s} thin[n][ct][h+r-1][w+s-1] * Wk[cw][ct][r][s]
//                   (forward of the first layer; input gradient of the last layer)
//   thin-out conv : out[n][ct][h][w] = b[ct] + sum_{r,s,cw} wide[src(h+r-1,w+s-1)][cw] * W[ct][cw][r][s]
//                   (forward of the last layer, optionally through the x2 upsample)
//   thin wgrad    : dW[tap][ct][cw] = sum over wide pixels q of wide[q][cw] * G(q,tap,ct)
//                   (weight gradient of both), G gathered from the thin tensor.
//
// The thin tensor is always planar [n][ct][H][W] — the layout of the library's
// boundary — so the first / last layout change of the pipeline disappears into these
// kernels; the wide tensor is [pixels][cw] like every other activation.  Also here: the
// per-plane sums that give the bias gradient of the planar last layer.
#include "ae_device.h"
#include "ae_internal.h"

namespace ae {
namespace {

constexpr int NT = 256;
constexpr int THIN_ROWS = 256;   // pixels per block of the thin-in conv (= partial-sum granularity)

// ---------------------------------------------------------------------------
// thin-in conv.  Each thread owns 4 output channels (their 9*CT weights live in
// registers) and walks over the block's pixels; the CW/4 threads of one pixel read the
// same 9*CT inputs (served as broadcasts by the vector cache).
// Wk(cw,ct,r,s) = W[cw][ct][r][s]            (forward; W canonical [CW][CT][3][3])
//              = W[ct][cw][2-r][2-s]         (flip: input gradient; W canonical [CT][CW][3][3])
// ---------------------------------------------------------------------------
template <typename T, int CT>
__global__ __launch_bounds__(NT) void k_thin_in_conv(const T* __restrict__ thin, const float* __restrict__ wcanon,
                                                     const float* __restrict__ bias, T* __restrict__ out,
                                                     float* __restrict__ partial, int64_t M, int H, int W, int CW,
                                                     int flip, int act) {
  __shared__ float sred[NT * 8];
  const int groups = CW >> 2;                  // threads per pixel
  const int g = threadIdx.x % groups;          // this thread's channel group
  const int pl = threadIdx.x / groups;         // pixel lane
  const int ppp = NT / groups;                 // pixels per pass
  float wk[4][CT * 9];
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const int cw = 4 * g + c;
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
      for (int t = 0; t < 9; ++t) {
        const int r = t / 3, s = t % 3;
        wk[c][ct * 9 + t] = flip ? wcanon[(((int64_t)ct * CW + cw) * 3 + (2 - r)) * 3 + (2 - s)]
                                 : wcanon[(((int64_t)cw * CT + ct) * 3 + r) * 3 + s];
      }
  }
  float bs[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) bs[c] = bias ? bias[4 * g + c] : 0.0f;
  float s1[4] = {0.f, 0.f, 0.f, 0.f}, s2[4] = {0.f, 0.f, 0.f, 0.f};
  const int64_t m0 = (int64_t)blockIdx.x * THIN_ROWS;
  const int64_t HW = (int64_t)H * W;
  for (int pp = pl; pp < THIN_ROWS; pp += ppp) {
    const int64_t m = m0 + pp;
    if (m >= M) break;
    const unsigned mu = (unsigned)m;             // M < 2^31 (checked by the launcher): 32-bit divisions
    const int w = (int)(mu % (unsigned)W);
    const int h = (int)((mu / (unsigned)W) % (unsigned)H);
    const int64_t n = mu / ((unsigned)H * (unsigned)W);
    // all 9*CT loads first, unconditionally and from clamped (valid) coordinates, so that
    // they are in flight together; the zero padding is applied to the loaded values
    float xv[CT * 9];
    int roff[3], coff[3];
    bool rok[3], cok[3];
#pragma unroll
    for (int t = 0; t < 3; ++t) {
      const int hh = h + t - 1, ww = w + t - 1;
      rok[t] = hh >= 0 && hh < H;
      cok[t] = ww >= 0 && ww < W;
      roff[t] = min(max(hh, 0), H - 1) * W;
      coff[t] = min(max(ww, 0), W - 1);
    }
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
      const T* plane = thin + (n * CT + ct) * HW;
#pragma unroll
      for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int s = 0; s < 3; ++s) xv[ct * 9 + r * 3 + s] = Store<T>::ld(plane + roff[r] + coff[s]);
    }
    float acc[4] = {bs[0], bs[1], bs[2], bs[3]};
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
      for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int s = 0; s < 3; ++s) {
          const float x = (rok[r] && cok[s]) ? xv[ct * 9 + r * 3 + s] : 0.0f;
#pragma unroll
          for (int c = 0; c < 4; ++c) acc[c] = fmaf(x, wk[c][ct * 9 + r * 3 + s], acc[c]);
        }
    float o[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const float v = round_to_storage<T>(acc[c]);
      const float d = v - bs[c];                 // statistics about the channel's bias (see k_bn_finalize)
      s1[c] += d;
      s2[c] = fmaf(d, d, s2[c]);
      o[c] = apply_act(v, act);
    }
    T* dst = out + m * CW + 4 * g;
    if (sizeof(T) == 2) {
      uint2 pk;
      pk.x = (uint32_t)f32_to_bf16(o[0]) | ((uint32_t)f32_to_bf16(o[1]) << 16);
      pk.y = (uint32_t)f32_to_bf16(o[2]) | ((uint32_t)f32_to_bf16(o[3]) << 16);
      *reinterpret_cast<uint2*>(dst) = pk;
    } else {
      *reinterpret_cast<float4*>(dst) = make_float4(o[0], o[1], o[2], o[3]);
    }
  }
  if (partial) {
    // combine the pixel lanes: sred[pl][g][8]
#pragma unroll
    for (int c = 0; c < 4; ++c) { sred[threadIdx.x * 8 + c] = s1[c]; sred[threadIdx.x * 8 + 4 + c] = s2[c]; }
    __syncthreads();
    for (int i = threadIdx.x; i < 2 * CW; i += NT) {
      const int q = i / CW, cw = i % CW;
      float t = 0.0f;
      for (int l = 0; l < ppp; ++l) t += sred[(l * groups + (cw >> 2)) * 8 + q * 4 + (cw & 3)];
      partial[((int64_t)blockIdx.x * 2 + q) * CW + cw] = t;
    }
  }
}

// ---------------------------------------------------------------------------
// thin-out conv: one thread per output pixel, CT <= 4 accumulators; the pixel's
// 9 x CW inputs stream from the vector cache in 16-byte pieces, the CT*9*CW weights
// sit in LDS as fp32 (broadcast reads).  Output planar [n][ct][H][W] (+ fp32 copy).
// ---------------------------------------------------------------------------
template <typename T, int CT>
__global__ __launch_bounds__(NT) void k_thin_out_conv(const T* __restrict__ wide, const float* __restrict__ wcanon,
                                                      const float* __restrict__ bias, T* __restrict__ out,
                                                      float* __restrict__ out_f32, int64_t M, int Hc, int Wc, int CW,
                                                      int up, int act) {
  extern __shared__ float sw[];                // [ct][tap][cw]
  constexpr int V = Store<T>::VEC;
  for (int i = threadIdx.x; i < CT * CW * 9; i += NT) {
    // canonical W[ct][cw][r][s]
    const int t = i % 9, cw = (i / 9) % CW, ct = i / (9 * CW);
    sw[(ct * 9 + t) * CW + cw] = wcanon[i];
  }
  __syncthreads();
  const int64_t m = (int64_t)blockIdx.x * NT + threadIdx.x;
  if (m >= M) return;
  const unsigned mu = (unsigned)m;
  const int w = (int)(mu % (unsigned)Wc);
  const int h = (int)((mu / (unsigned)Wc) % (unsigned)Hc);
  const int64_t n = mu / ((unsigned)Wc * (unsigned)Hc);
  const int Hin = Hc >> up, Win = Wc >> up;
  float acc[CT];
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) acc[ct] = bias ? bias[ct] : 0.0f;
  // channels in groups of 32 elements: the group's loads are issued together (from a
  // clamped, always valid source pixel), then consumed
  constexpr int GRP = 32 / V;                  // 16-byte loads per group
  for (int r = 0; r < 3; ++r) {
    const int hh = h + r - 1;
    const bool rok = hh >= 0 && hh < Hc;
    const int hs = min(max(hh, 0), Hc - 1) >> up;
    for (int s = 0; s < 3; ++s) {
      const int ww = w + s - 1;
      const float keep = (rok && ww >= 0 && ww < Wc) ? 1.0f : 0.0f;
      const int ws = min(max(ww, 0), Wc - 1) >> up;
      const T* src = wide + ((n * Hin + hs) * Win + ws) * CW;
      const float* wt = sw + (r * 3 + s) * CW;
      for (int c0 = 0; c0 < CW; c0 += 32) {
        float xv[GRP][V];
#pragma unroll
        for (int g = 0; g < GRP; ++g) Store<T>::ldv(src + c0 + g * V, xv[g]);
#pragma unroll
        for (int g = 0; g < GRP; ++g)
#pragma unroll
          for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int j = 0; j < V; j += 4) {
              const float4 w4 = *reinterpret_cast<const float4*>(wt + ct * 9 * CW + c0 + g * V + j);
              float t = xv[g][j] * w4.x;
              t = fmaf(xv[g][j + 1], w4.y, t);
              t = fmaf(xv[g][j + 2], w4.z, t);
              t = fmaf(xv[g][j + 3], w4.w, t);
              acc[ct] = fmaf(keep, t, acc[ct]);
            }
      }
    }
  }
  const int64_t HW = (int64_t)Hc * Wc;
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) {
    const float a = apply_act(round_to_storage<T>(acc[ct]), act);
    const int64_t o = (n * CT + ct) * HW + (int64_t)h * Wc + w;
    Store<T>::st(out + o, a);
    if (out_f32) out_f32[o] = a;
  }
}

// ---------------------------------------------------------------------------
// thin wgrad.  mode 0 (first layer): q = conv pixel (n,h,w), G[tap][ct] = thin[n][ct][h+r-1][w+s-1].
// mode 1 (last layer): q = wide pixel (n,i,j) at the stored resolution, thin is the
// output gradient at conv resolution, G[tap][ct] = sum_{a,b<=up} thin[n][ct][(i<<up)+a-(r-1)][(j<<up)+b-(s-1)].
// A block walks PIX wide pixels; G of 64 pixels at a time is built cooperatively in
// LDS, then each thread (one wide channel cw, one pixel lane) accumulates its
// 9*CT sums.  Block partials [block][9*CT][CW] are summed by k_thin_wgrad_reduce.
// ---------------------------------------------------------------------------
template <typename T, int CT>
__global__ __launch_bounds__(NT) void k_thin_wgrad(const T* __restrict__ thin, const T* __restrict__ wide,
                                                   float* __restrict__ partial, int64_t Q, int pix_per_block, int Hq,
                                                   int Wq, int Ht, int Wt, int CW, int cw0_stride, int mode, int up) {
  constexpr int G = 9 * CT;
  constexpr int GP = (G + 3) & ~3;               // row padded for 16-byte LDS reads
  constexpr int CHUNK = 64;
  __shared__ __attribute__((aligned(16))) float sg[CHUNK][GP];
  __shared__ float sacc[NT][G + 1];
  const int cwl = threadIdx.x % cw0_stride;      // channel within the block's channel slice
  const int pl = threadIdx.x / cw0_stride;
  const int lanes = NT / cw0_stride;
  const int cw = blockIdx.y * cw0_stride + cwl;
  float acc[G];
#pragma unroll
  for (int i = 0; i < G; ++i) acc[i] = 0.0f;
  const int64_t q0 = (int64_t)blockIdx.x * pix_per_block;
  const int64_t q1 = (q0 + pix_per_block < Q) ? q0 + pix_per_block : Q;
  const int64_t HWt = (int64_t)Ht * Wt;
  for (int64_t qc = q0; qc < q1; qc += CHUNK) {
    __syncthreads();
    // build G for pixels qc .. qc+CHUNK-1
    // fixed trip count, unrolled: the loads of all passes are in flight together
#pragma unroll
    for (int k = 0; k < (CHUNK * G + NT - 1) / NT; ++k) {
      const int i = threadIdx.x + k * NT;
      if (i >= CHUNK * G) break;
      const int p = i / G, gi = i % G;
      const int ct = gi % CT, tap = gi / CT;
      const int r = tap / 3, s = tap % 3;
      const int64_t q = qc + p;
      float v = 0.0f;
      if (q < q1) {
        const unsigned qu = (unsigned)q;
        const int j = (int)(qu % (unsigned)Wq);
        const int ii = (int)((qu / (unsigned)Wq) % (unsigned)Hq);
        const int64_t n = qu / ((unsigned)Wq * (unsigned)Hq);
        const T* plane = thin + (n * CT + ct) * HWt;
        if (mode == 0) {
          const int hh = ii + r - 1, ww = j + s - 1;
          const float x = Store<T>::ld(plane + (int64_t)min(max(hh, 0), Ht - 1) * Wt + min(max(ww, 0), Wt - 1));
          v = (hh >= 0 && hh < Ht && ww >= 0 && ww < Wt) ? x : 0.0f;
        } else {
          for (int a = 0; a <= up; ++a)
            for (int b = 0; b <= up; ++b) {
              const int hh = (ii << up) + a - (r - 1), ww = (j << up) + b - (s - 1);
              const float x = Store<T>::ld(plane + (int64_t)min(max(hh, 0), Ht - 1) * Wt + min(max(ww, 0), Wt - 1));
              v += (hh >= 0 && hh < Ht && ww >= 0 && ww < Wt) ? x : 0.0f;
            }
        }
      }
      sg[p][gi] = v;
    }
    if (GP > G)
      for (int i = threadIdx.x; i < CHUNK * (GP - G); i += NT) sg[i / (GP - G)][G + i % (GP - G)] = 0.0f;
    __syncthreads();
    if (cw < CW) {
      // the wide values of all the thread's pixels first (lanes >= 4: at most 16 of them), then the sums
      float wvs[16];
#pragma unroll
      for (int k = 0; k < 16; ++k) {
        const int p = pl + k * lanes;
        const int64_t q = qc + p;
        wvs[k] = (p < CHUNK && q < q1) ? Store<T>::ld(wide + q * CW + cw) : 0.0f;
      }
#pragma unroll
      for (int k = 0; k < 16; ++k) {
        const int p = pl + k * lanes;
        if (p >= CHUNK) break;
        const float wv = wvs[k];
#pragma unroll
        for (int i = 0; i < GP; i += 4) {
          const float4 g4 = *reinterpret_cast<const float4*>(&sg[p][i]);
          acc[i] = fmaf(wv, g4.x, acc[i]);
          if (i + 1 < G) acc[i + 1] = fmaf(wv, g4.y, acc[i + 1]);
          if (i + 2 < G) acc[i + 2] = fmaf(wv, g4.z, acc[i + 2]);
          if (i + 3 < G) acc[i + 3] = fmaf(wv, g4.w, acc[i + 3]);
        }
      }
    }
  }
  // combine pixel lanes, write the block partial [G][CW]
#pragma unroll
  for (int i = 0; i < G; ++i) sacc[threadIdx.x][i] = acc[i];
  __syncthreads();
  for (int i = threadIdx.x; i < cw0_stride * G; i += NT) {
    const int c = i % cw0_stride, gi = i / cw0_stride;
    const int cwo = blockIdx.y * cw0_stride + c;
    if (cwo < CW) {
      float t = 0.0f;
      for (int l = 0; l < lanes; ++l) t += sacc[l * cw0_stride + c][gi];
      partial[((int64_t)blockIdx.x * G + gi) * CW + cwo] = t;
    }
  }
}

// dW canonical: mode 0: [cw][ct][r][s]; mode 1: [ct][cw][r][s]
template <int CT>
__global__ void k_thin_wgrad_reduce(const float* __restrict__ partial, int nblocks, int CW, int mode,
                                    float* __restrict__ dw) {
  constexpr int G = 9 * CT;
  const int total = G * CW;
  // eight lanes per output: lane q sums blocks q, q+8, ...; then a fixed-order shuffle tree
  const int gid = (blockIdx.x * NT + threadIdx.x) >> 3, sub = threadIdx.x & 7;
  const int i = gid < total ? gid : total - 1;
  float acc = 0.0f;
  for (int b = sub; b < nblocks; b += 8) acc += partial[(int64_t)b * total + i];
  acc += __shfl_xor(acc, 1, 64);
  acc += __shfl_xor(acc, 2, 64);
  acc += __shfl_xor(acc, 4, 64);
  if (gid < total && sub == 0) {
    const int cw = i % CW, gi = i / CW;
    const int ct = gi % CT, tap = gi / CT;
    const int64_t o = mode == 0 ? ((int64_t)cw * CT + ct) * 9 + tap : ((int64_t)ct * CW + cw) * 9 + tap;
    dw[o] = acc;
  }
}

// per-plane sums of a planar tensor [n][C][HW], each plane cut into `split` pieces:
// partial[(n*split + piece)][0][c] = sum, [..][1][c] = sum of squares
template <typename T>
__global__ void k_plane_sums(const T* __restrict__ x, int C, int64_t HW, int split, int vec, float* __restrict__ partial) {
  __shared__ float sm[NT / 64 + 1];
  constexpr int V = Store<T>::VEC;
  const int piece = blockIdx.y;
  const int c = blockIdx.x % C;
  const int64_t n = blockIdx.x / C;
  const int64_t len = (HW + split - 1) / split;
  const int64_t i0 = piece * len, i1 = i0 + len < HW ? i0 + len : HW;
  const T* p = x + (n * C + c) * HW;
  float s1 = 0.0f, s2 = 0.0f;
  int64_t i = i0 + threadIdx.x;
  if (vec && len % V == 0) {                     // pieces start on 16-byte boundaries
#pragma unroll 4
    for (int64_t q = i0 + (int64_t)threadIdx.x * V; q + V <= i1; q += (int64_t)NT * V) {
      float v[V];
      Store<T>::ldv(p + q, v);
#pragma unroll
      for (int j = 0; j < V; ++j) { s1 += v[j]; s2 = fmaf(v[j], v[j], s2); }
    }
    i = i0 + (i1 - i0) / V * V + threadIdx.x;
  }
  for (; i < i1; i += NT) { const float v = Store<T>::ld(p + i); s1 += v; s2 = fmaf(v, v, s2); }
  s1 = block_sum<NT>(s1, sm);
  s2 = block_sum<NT>(s2, sm);
  if (threadIdx.x == 0) {
    const int64_t row = n * split + piece;
    partial[(row * 2) * C + c] = s1;
    partial[(row * 2 + 1) * C + c] = s2;
  }
}

}  // namespace

bool thin_in_supported(int ct, int cw, int k, int up) {
  if (k != 3 || up || ct < 1 || ct > 4) return false;
  if (cw % 4 != 0 || cw < 8 || cw > 1024) return false;
  const int groups = cw / 4;
  return (groups & (groups - 1)) == 0;          // the 256 threads split evenly into channel groups
}

bool thin_out_supported(int ct, int cw, int k, int dtype) {
  (void)dtype;
  return k == 3 && ct >= 1 && ct <= 4 && cw % 32 == 0 && (int64_t)ct * 9 * cw * 4 <= 60 * 1024;
}

int thin_in_partial_rows() { return THIN_ROWS; }

#define THIN_DISPATCH(dtype, CTV, ...)                                             \
  do {                                                                             \
    if ((dtype) == AE_BF16) { typedef bf16_t T; THIN_CT(CTV, __VA_ARGS__); }       \
    else { typedef float T; THIN_CT(CTV, __VA_ARGS__); }                           \
  } while (0)
#define THIN_CT(CTV, ...)                                          \
  switch (CTV) {                                                   \
    case 1: { constexpr int CT = 1; __VA_ARGS__; break; }          \
    case 2: { constexpr int CT = 2; __VA_ARGS__; break; }          \
    case 3: { constexpr int CT = 3; __VA_ARGS__; break; }          \
    default: { constexpr int CT = 4; __VA_ARGS__; break; }         \
  }

// thin: planar [n][ct][H][W]; out: [n*H*W][cw]
int launch_thin_in_conv(const void* thin, const float* wcanon, const float* bias, void* out, float* partial, int n,
                        int h, int w, int ct, int cw, int flip, int act, int dtype, hipStream_t s) {
  if (!thin_in_supported(ct, cw, 3, 0)) return fail(AE_EINVAL, "thin_in_conv: shape not supported");
  const int64_t M = (int64_t)n * h * w;
  if (M >= 0x7FFFFFFF) return fail(AE_EINVAL, "thin_in_conv: tensor too large");
  const unsigned grid = (unsigned)((M + THIN_ROWS - 1) / THIN_ROWS);
  THIN_DISPATCH(dtype, ct, hipLaunchKernelGGL((k_thin_in_conv<T, CT>), dim3(grid), dim3(NT), 0, s, (const T*)thin,
                                              wcanon, bias, (T*)out, partial, M, h, w, cw, flip, act));
  return launch_status("thin_in_conv");
}

// wide: [n*(hc>>up)*(wc>>up)][cw]; out: planar [n][ct][hc][wc]
int launch_thin_out_conv(const void* wide, const float* wcanon, const float* bias, void* out, float* out_f32, int n,
                         int hc, int wc, int ct, int cw, int up, int act, int dtype, hipStream_t s) {
  if (!thin_out_supported(ct, cw, 3, dtype)) return fail(AE_EINVAL, "thin_out_conv: shape not supported");
  const int64_t M = (int64_t)n * hc * wc;
  if (M >= 0x7FFFFFFF) return fail(AE_EINVAL, "thin_out_conv: tensor too large");
  const unsigned grid = (unsigned)((M + NT - 1) / NT);
  const size_t smem = (size_t)ct * 9 * cw * sizeof(float);
  THIN_DISPATCH(dtype, ct, hipLaunchKernelGGL((k_thin_out_conv<T, CT>), dim3(grid), dim3(NT), smem, s, (const T*)wide,
                                              wcanon, bias, (T*)out, out_f32, M, hc, wc, cw, up, act));
  return launch_status("thin_out_conv");
}

// pixels per block of the VALU weight-gradient kernel: about 1024 blocks, at least 512 pixels each
static int thin_wgrad_ppb(int64_t q_pixels) {
  int64_t ppb = (q_pixels + 1023) / 1024;
  ppb = (ppb + 63) / 64 * 64;
  if (ppb < 512) ppb = 512;
  return (int)ppb;
}

int64_t thin_wgrad_workspace_floats(int64_t q_pixels, int ct, int cw) {
  const int64_t ppb = thin_wgrad_ppb(q_pixels);
  return ((q_pixels + ppb - 1) / ppb) * 9 * ct * cw;
}

// mode 0: thin planar [n][ct][hq][wq] (the layer input), wide [n*hq*wq][cw] (output gradient)
// mode 1: thin planar [n][ct][hq<<up][wq<<up] (output gradient), wide [n*hq*wq][cw] (the layer input)
int launch_thin_wgrad(const void* thin, const void* wide, float* workspace, float* dw_canonical, int n, int hq, int wq,
                      int ct, int cw, int mode, int up, int dtype, hipStream_t s) {
  if (ct < 1 || ct > 4) return fail(AE_EINVAL, "thin_wgrad: thin side must have 1..4 channels");
  const int64_t Q = (int64_t)n * hq * wq;
  if (Q >= 0x7FFFFFFF) return fail(AE_EINVAL, "thin_wgrad: tensor too large");
  const int ppb = thin_wgrad_ppb(Q);
  const int nblocks = (int)((Q + ppb - 1) / ppb);
  int slice = 64;                               // wide channels per block
  while (slice > cw && slice > 1) slice >>= 1;
  const int ht = mode == 0 ? hq : hq << up, wt = mode == 0 ? wq : wq << up;
  dim3 grid((unsigned)nblocks, (unsigned)((cw + slice - 1) / slice));
  THIN_DISPATCH(dtype, ct, hipLaunchKernelGGL((k_thin_wgrad<T, CT>), grid, dim3(NT), 0, s, (const T*)thin,
                                              (const T*)wide, workspace, Q, ppb, hq, wq, ht, wt, cw, slice, mode, up));
  AE_TRY(launch_status("thin_wgrad"));
  const int total = 9 * ct * cw;
  switch (ct) {
    case 1: hipLaunchKernelGGL(k_thin_wgrad_reduce<1>, dim3((total * 8 + NT - 1) / NT), dim3(NT), 0, s, workspace, nblocks, cw, mode, dw_canonical); break;
    case 2: hipLaunchKernelGGL(k_thin_wgrad_reduce<2>, dim3((total * 8 + NT - 1) / NT), dim3(NT), 0, s, workspace, nblocks, cw, mode, dw_canonical); break;
    case 3: hipLaunchKernelGGL(k_thin_wgrad_reduce<3>, dim3((total * 8 + NT - 1) / NT), dim3(NT), 0, s, workspace, nblocks, cw, mode, dw_canonical); break;
    default: hipLaunchKernelGGL(k_thin_wgrad_reduce<4>, dim3((total * 8 + NT - 1) / NT), dim3(NT), 0, s, workspace, nblocks, cw, mode, dw_canonical); break;
  }
  return launch_status("thin_wgrad_reduce");
}

int plane_sums_split(int64_t hw) {
  int split = (int)(hw / 8192);                  // about 8192 elements per workgroup
  if (split < 1) split = 1;
  if (split > 64) split = 64;
  return split;
}

// writes n*plane_sums_split(hw) partial rows
int launch_plane_sums(const void* x, int64_t n, int c, int64_t hw, int dtype, float* partial, hipStream_t s) {
  if (n * c > 0x7FFFFFFF) return fail(AE_EINVAL, "plane_sums: too many planes");
  const int split = plane_sums_split(hw);
  const int vec = (((uintptr_t)x & 15) == 0 && hw % 8 == 0) ? 1 : 0;
  dim3 grid((unsigned)(n * c), (unsigned)split);
  if (dtype == AE_BF16)
    hipLaunchKernelGGL((k_plane_sums<bf16_t>), grid, dim3(NT), 0, s, (const bf16_t*)x, c, hw, split, vec, partial);
  else
    hipLaunchKernelGGL((k_plane_sums<float>), grid, dim3(NT), 0, s, (const float*)x, c, hw, split, vec, partial);
  return launch_status("plane_sums");
}

}  // namespace ae
