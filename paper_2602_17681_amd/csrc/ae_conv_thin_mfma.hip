// ae_conv_thin_mfma.hip — bf16 matrix-core kernels for the 3x3 convolutions with a
// "thin" side (1..4 channels): the first and the last layer of the autoencoders.
//
//   thin-in conv  : out[q][cw] = b[cw] + sum_{ct,r,s} thin[n][ct][h+r-1][w+s-1] * Wk[cw][ct][r][s]
//                   forward of the first layer; input gradient of the last layer (flipped
//                   weights), optionally summed over 2x2 pixel groups (the backward of the
//                   x2 upsample the last conv reads through).
//   thin wgrad    : dW = sum over wide pixels q of wide[q][cw] * G(q)[tap][ct]
//                   weight gradient of the first layer (G gathered from the layer input)
//                   and of the last layer (G gathered from the output gradient).
//
// The thin tensor is planar [n][ct][H][W] (the layout of the library's boundary); the wide
// tensor is [pixels][cw].  All kernels work on a patch of the thin tensor held in LDS as
// pixels of 4 interleaved channels (8 bytes): the three taps (s = 0,1,2) of one filter row
// of a pixel are then 12 consecutive values, i.e. one K = 16 MFMA step with
//   k = 4*s + ci   (s = 3 and ci >= CT carry zero weights / are ignored).
// These layers are bound by HBM (the wide tensor) — the kernels issue all their global loads
// of a patch at once, and never loop over dependent loads.
#include "ae_device.h"
#include "ae_internal.h"

namespace ae {
namespace {

constexpr int NT = 256;
typedef __bf16 t_bf16x8 __attribute__((ext_vector_type(8)));
typedef float t_floatx16 __attribute__((ext_vector_type(16)));
typedef short t_short4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) t_short4 t_lds_short4;

// ---------------------------------------------------------------------------
// LDS patch of one sample's planar thin tensor img[CT][H][W].
// Cell (pr, pc), pr < rows, pc < IW + 4, holds pixel (h_first + pr, w_first - 2 + pc):
// pc = 1 is the left halo column, pc = 2 .. IW+1 the interior (IW a multiple of 8,
// w_first a multiple of 8), pc = IW+2 the right halo, pc = 0 and IW+3 are zero.
// Pixels outside the image and channels >= CT are zero.
// vec: W % 8 == 0 and img 16-byte aligned — the interior moves as 16-byte loads.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void thin_fill_patch(bf16_t* __restrict__ tile, const bf16_t* __restrict__ img, int H, int W,
                                                int CT, int h_first, int w_first, int rows, int IW, bool vec) {
  const int PW = IW + 4;
  const int tid = threadIdx.x;
  const int64_t HW = (int64_t)H * W;
  if (vec) {
    const int cpr = IW >> 3, cshift = 31 - __clz(cpr);   // IW is a power of two
    for (int idx = tid; idx < rows * cpr; idx += NT) {
      const int pr = idx >> cshift, c = idx & (cpr - 1);
      const int hh = h_first + pr, ww = w_first + 8 * c;
      const bool ok = hh >= 0 && hh < H && ww < W;
      const int64_t off = (int64_t)min(max(hh, 0), H - 1) * W + min(ww, W - 8);
      uint32_t v[4][4];
#pragma unroll
      for (int ci = 0; ci < 4; ++ci) {
        const uint4 t = *reinterpret_cast<const uint4*>(img + (int64_t)min(ci, CT - 1) * HW + off);
        const bool keep = ok && ci < CT;
        v[ci][0] = keep ? t.x : 0u; v[ci][1] = keep ? t.y : 0u; v[ci][2] = keep ? t.z : 0u; v[ci][3] = keep ? t.w : 0u;
      }
      bf16_t* dst = tile + ((int64_t)pr * PW + 2 + 8 * c) * 4;
#pragma unroll
      for (int k = 0; k < 4; ++k) {              // word k holds pixels 2k (low half) and 2k+1 (high half)
        uint4 o;
        o.x = (v[0][k] & 0xFFFFu) | (v[1][k] << 16);
        o.y = (v[2][k] & 0xFFFFu) | (v[3][k] << 16);
        o.z = (v[0][k] >> 16) | (v[1][k] & 0xFFFF0000u);
        o.w = (v[2][k] >> 16) | (v[3][k] & 0xFFFF0000u);
        *reinterpret_cast<uint4*>(dst + 8 * k) = o;
      }
    }
    // halo columns (and the two zero columns), by the high threads so that they overlap the interior
    for (int idx = NT - 1 - tid; idx < rows * 2; idx += NT) {
      const int pr = idx >> 1, side = idx & 1;
      const int hh = h_first + pr, ww = side ? w_first + IW : w_first - 1;
      const bool ok = hh >= 0 && hh < H && ww >= 0 && ww < W;
      const int64_t off = (int64_t)min(max(hh, 0), H - 1) * W + min(max(ww, 0), W - 1);
      uint32_t e[4];
#pragma unroll
      for (int ci = 0; ci < 4; ++ci) {
        const bf16_t t = img[(int64_t)min(ci, CT - 1) * HW + off];
        e[ci] = (ok && ci < CT) ? (uint32_t)t : 0u;
      }
      const uint32_t lo = e[0] | (e[1] << 16), hi = e[2] | (e[3] << 16);
      if (side) *reinterpret_cast<uint4*>(tile + ((int64_t)pr * PW + IW + 2) * 4) = make_uint4(lo, hi, 0u, 0u);
      else *reinterpret_cast<uint4*>(tile + (int64_t)pr * PW * 4) = make_uint4(0u, 0u, lo, hi);
    }
  } else {
    for (int i = tid; i < rows * PW * 4; i += NT) {
      const int ci = i & 3, cell = i >> 2;
      const int pc = cell % PW, pr = cell / PW;
      const int hh = h_first + pr, ww = w_first - 2 + pc;
      const bool ok = ci < CT && pc >= 1 && pc <= IW + 2 && hh >= 0 && hh < H && ww >= 0 && ww < W;
      const bf16_t t = img[(int64_t)min(ci, CT - 1) * HW + (int64_t)min(max(hh, 0), H - 1) * W + min(max(ww, 0), W - 1)];
      tile[i] = ok ? t : (bf16_t)0;
    }
  }
}

// The same patch for binary32: a cell is a pixel of 4 interleaved floats (16 bytes); the interior moves as 16-byte
// loads of 4 pixels of one channel.
__device__ __forceinline__ void thin_fill_patch(float* __restrict__ tile, const float* __restrict__ img, int H, int W,
                                                int CT, int h_first, int w_first, int rows, int IW, bool vec) {
  const int PW = IW + 4;
  const int tid = threadIdx.x;
  const int64_t HW = (int64_t)H * W;
  if (vec) {
    const int cpr = IW >> 2, cshift = 31 - __clz(cpr);   // IW is a power of two
    for (int idx = tid; idx < rows * cpr; idx += NT) {
      const int pr = idx >> cshift, c = idx & (cpr - 1);
      const int hh = h_first + pr, ww = w_first + 4 * c;
      const bool ok = hh >= 0 && hh < H && ww < W;
      const int64_t off = (int64_t)min(max(hh, 0), H - 1) * W + min(ww, W - 4);
      float v[4][4];
#pragma unroll
      for (int ci = 0; ci < 4; ++ci) {
        const float4 t = *reinterpret_cast<const float4*>(img + (int64_t)min(ci, CT - 1) * HW + off);
        const bool keep = ok && ci < CT;
        v[ci][0] = keep ? t.x : 0.0f; v[ci][1] = keep ? t.y : 0.0f; v[ci][2] = keep ? t.z : 0.0f; v[ci][3] = keep ? t.w : 0.0f;
      }
      float* dst = tile + ((int64_t)pr * PW + 2 + 4 * c) * 4;
#pragma unroll
      for (int k = 0; k < 4; ++k) *reinterpret_cast<float4*>(dst + 4 * k) = make_float4(v[0][k], v[1][k], v[2][k], v[3][k]);
    }
    for (int idx = NT - 1 - tid; idx < rows * 2; idx += NT) {
      const int pr = idx >> 1, side = idx & 1;
      const int hh = h_first + pr, ww = side ? w_first + IW : w_first - 1;
      const bool ok = hh >= 0 && hh < H && ww >= 0 && ww < W;
      const int64_t off = (int64_t)min(max(hh, 0), H - 1) * W + min(max(ww, 0), W - 1);
      float e[4];
#pragma unroll
      for (int ci = 0; ci < 4; ++ci) {
        const float t = img[(int64_t)min(ci, CT - 1) * HW + off];
        e[ci] = (ok && ci < CT) ? t : 0.0f;
      }
      float* cell = tile + ((int64_t)pr * PW + (side ? IW + 2 : 0)) * 4;
      const float4 px = make_float4(e[0], e[1], e[2], e[3]), zero = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
      *reinterpret_cast<float4*>(cell) = side ? px : zero;
      *reinterpret_cast<float4*>(cell + 4) = side ? zero : px;
    }
  } else {
    for (int i = tid; i < rows * PW * 4; i += NT) {
      const int ci = i & 3, cell = i >> 2;
      const int pc = cell % PW, pr = cell / PW;
      const int hh = h_first + pr, ww = w_first - 2 + pc;
      const bool ok = ci < CT && pc >= 1 && pc <= IW + 2 && hh >= 0 && hh < H && ww >= 0 && ww < W;
      const float t = img[(int64_t)min(ci, CT - 1) * HW + (int64_t)min(max(hh, 0), H - 1) * W + min(max(ww, 0), W - 1)];
      tile[i] = ok ? t : 0.0f;
    }
  }
}

// Weights of a thin-side conv as bf16 MFMA operand rows: wfrag[co][r][k], k = 4*s + ci
// (zero where ci >= CT, s == 3 or co >= CW).
//   Wk(co,ci,r,s) = W[co][ci][r][s]             (W canonical [CW][CT][3][3])
//                 = W[ci][co][2-r][2-s]         (flip: W canonical [CT][CW][3][3], input gradient)
template <typename T>
__global__ void k_thin_pack_wfrag(const float* __restrict__ wcanon, T* __restrict__ wfrag, int CT, int CW,
                                  int rows, int flip) {
  const int i = blockIdx.x * NT + threadIdx.x;
  if (i >= rows * 48) return;
  const int k = i & 15, r = (i >> 4) % 3, co = i / 48;
  const int s_ = k >> 2, ci = k & 3;
  float v = 0.0f;
  if (co < CW && ci < CT && s_ < 3)
    v = flip ? wcanon[(((int64_t)ci * CW + co) * 3 + (2 - r)) * 3 + (2 - s_)]
             : wcanon[(((int64_t)co * CT + ci) * 3 + r) * 3 + s_];
  Store<T>::st(wfrag + i, v);
}

// Row L (0..255) of a workgroup's 256 x CW output tile -> pixel of the TH x TW patch.
// Linear: row-major.  Grouped (GROUP2): rows 4G..4G+3 are the 2x2 pixel group G, so that the
// four accumulator values a lane holds for one row quad are one group.
template <bool GROUP2>
__device__ __forceinline__ void thin_row_pixel(int L, int TW, int tw_shift, int& th, int& tw) {
  if (GROUP2) {
    const int G = L >> 2;
    th = 2 * (G >> (tw_shift - 1)) + ((L >> 1) & 1);
    tw = 2 * (G & ((TW >> 1) - 1)) + (L & 1);
  } else {
    th = L >> tw_shift;
    tw = L & (TW - 1);
  }
}

// Epilogue of the thin-in conv.  MODE 0: every check at run time (ragged patches, any activation);
// MODE 1: interior patch, column statistics of the stored value, no activation;
// MODE 2: interior, ReLU;  MODE 3: interior, no activation.
// Element e of lane l in tile (i,j): row wave*64 + i*32 + (e/4)*8 + (l/32)*4 + e%4, channel j*32 + l%32.
// Rows are staged through wave-private LDS so that global stores are 16 bytes wide.
template <typename T, int NJ, int MODE, bool UPSUM>
__device__ __forceinline__ void thin_epilogue(const t_floatx16 (&acc)[2][NJ], const float (&bs)[NJ],
                                              T* __restrict__ stage, T* __restrict__ out_n, int H, int W,
                                              int CW, int h0, int w0, int TW, int tw_shift, int act, bool want_stats,
                                              float (&s1)[NJ], float (&s2)[NJ]) {
  constexpr int EPC = 16 / (int)sizeof(T);       // elements per 16-byte chunk
  constexpr int SW = NJ * 32 + EPC;              // staging row stride
  constexpr int CPR = NJ * 32 / EPC;             // 16-byte chunks per pixel
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col_lane = lane & 31, row_lane = (lane >> 5) * 4;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    if (!UPSUM) {
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int lr = (e >> 2) * 8 + row_lane + (e & 3);
          float v = acc[i][j][e] + bs[j];
          if (MODE == 0) {
            v = round_to_storage<T>(v);
            if (want_stats) {
              int th, tw;
              thin_row_pixel<false>(wave * 64 + i * 32 + lr, TW, tw_shift, th, tw);
              if (j * 32 + col_lane < CW && h0 + th < H && w0 + tw < W) {
                const float d = v - bs[j];       // statistics about the channel's bias (see k_bn_finalize)
                s1[j] += d;
                s2[j] = fmaf(d, d, s2[j]);
              }
            }
            v = apply_act(v, act);
          } else if (MODE == 1) {
            v = round_to_storage<T>(v);
            const float d = v - bs[j];
            s1[j] += d;
            s2[j] = fmaf(d, d, s2[j]);
          } else if (MODE == 2) {
            v = fmaxf(v, 0.0f);                  // rounding is monotonic and keeps 0
          }
          Store<T>::st(&stage[lr * SW + j * 32 + col_lane], v);
        }
      }
#pragma unroll
      for (int c = 0; c < (32 * CPR) / 64; ++c) {
        const int idx = c * 64 + lane;
        const int lr = idx / CPR, ch = idx % CPR;
        int th, tw;
        thin_row_pixel<false>(wave * 64 + i * 32 + lr, TW, tw_shift, th, tw);
        const int hh = h0 + th, ww = w0 + tw;
        if (MODE != 0 || (hh < H && ww < W && ch * EPC < CW))
          *reinterpret_cast<uint4*>(out_n + ((int64_t)hh * W + ww) * CW + ch * EPC) =
              *reinterpret_cast<const uint4*>(&stage[lr * SW + ch * EPC]);
      }
    } else {
      // 2x2 sums: the row quad (e%4 = 0..3) of a lane is one pixel group
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
#pragma unroll
        for (int eg = 0; eg < 4; ++eg) {
          const float v = ((acc[i][j][4 * eg] + bs[j]) + (acc[i][j][4 * eg + 1] + bs[j])) +
                          ((acc[i][j][4 * eg + 2] + bs[j]) + (acc[i][j][4 * eg + 3] + bs[j]));
          Store<T>::st(&stage[(eg * 2 + (lane >> 5)) * SW + j * 32 + col_lane], v);
        }
      }
      const int Hq = H >> 1, Wq = W >> 1;
#pragma unroll
      for (int c = 0; c < (8 * CPR + 63) / 64; ++c) {
        const int idx = c * 64 + lane;
        const int g8 = idx / CPR, ch = idx % CPR;
        const int G = wave * 16 + i * 8 + g8;
        const int hq = (h0 >> 1) + (G >> (tw_shift - 1)), wq = (w0 >> 1) + (G & ((TW >> 1) - 1));
        if (idx < 8 * CPR && (MODE != 0 || (hq < Hq && wq < Wq && ch * EPC < CW)))
          *reinterpret_cast<uint4*>(out_n + ((int64_t)hq * Wq + wq) * CW + ch * EPC) =
              *reinterpret_cast<const uint4*>(&stage[g8 * SW + ch * EPC]);
      }
    }
  }
}

// ---------------------------------------------------------------------------
// thin-in conv.  A workgroup owns a TH x TW patch of one image (TH*TW = 256 pixels); each
// wave computes 64 pixels x NJ*32 channels with three MFMA steps (one per filter row) per
// 32x32 tile.  out: [n][H][W][CW], or with UPSUM [n][H/2][W/2][CW] holding 2x2 sums.
// partial (optional): [patch][sum | sum of squares][CW] of the stored values.
// ---------------------------------------------------------------------------
// T = float: a filter row is K = 16 as eight v_mfma_f32_32x32x2_f32: a lane's 16-byte read is one patch cell (a tap's four
// channels), the low half-wave takes taps 0 and 2, the high one taps 1 and 3, and component c of both halves is one
// MFMA's pair of K values (the weights are read the same way).
template <typename T, int NJ, bool UPSUM>
__global__ __launch_bounds__(NT) void k_thin_in_mfma(const T* __restrict__ thin, const T* __restrict__ wfrag,
                                                     const float* __restrict__ bias, T* __restrict__ out,
                                                     float* __restrict__ partial, int H, int W, int CT, int CW, int act,
                                                     int TW, int tw_shift, int tiles_w, int tiles_h, int vec) {
  constexpr int MAXT = 408;                     // (TH+2)*(TW+4) cells for every TW in {8,...,64}
  constexpr int SW = NJ * 32 + 16 / (int)sizeof(T);
  constexpr bool F32 = sizeof(T) == 4;
  __shared__ __attribute__((aligned(16))) T tile[MAXT * 4];
  __shared__ __attribute__((aligned(16))) T stage_all[4 * 32 * SW];
  __shared__ float sRed[4][2][NJ * 32];
  const int TH = NT >> tw_shift;
  const int PW = TW + 4;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int b = blockIdx.x;
  const int tx = b % tiles_w; b /= tiles_w;
  const int ty = b % tiles_h;
  const int n = b / tiles_h;
  const int h0 = ty * TH, w0 = tx * TW;
  const int frag_row = lane & 31, g = lane >> 5;
  const int col_lane = lane & 31;

  union Frag { uint4 u; t_bf16x8 v; float f[4]; };
  Frag bfrag[3][NJ][F32 ? 2 : 1];
#pragma unroll
  for (int r = 0; r < 3; ++r)
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const T* wrow = &wfrag[((j * 32 + frag_row) * 3 + r) * 16];
      if constexpr (F32) {
        bfrag[r][j][0].u = *reinterpret_cast<const uint4*>(wrow + g * 4);
        bfrag[r][j][1].u = *reinterpret_cast<const uint4*>(wrow + 8 + g * 4);
      } else {
        bfrag[r][j][0].u = *reinterpret_cast<const uint4*>(wrow + g * 8);
      }
    }
  float bs[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) bs[j] = (bias && j * 32 + col_lane < CW) ? bias[j * 32 + col_lane] : 0.0f;

  thin_fill_patch(tile, thin + (int64_t)n * CT * H * W, H, W, CT, h0 - 1, w0, TH + 2, TW, vec != 0);
  __syncthreads();

  t_floatx16 acc[2][NJ];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    int th, tw;
    thin_row_pixel<UPSUM>(wave * 64 + i * 32 + frag_row, TW, tw_shift, th, tw);
#pragma unroll
    for (int r = 0; r < 3; ++r) {
      if constexpr (F32) {
        // taps g and 2 + g = cells tw + 1 + g and tw + 3 + g of patch row th + r
        const float* src = &tile[((th + r) * PW + tw + 1 + g) * 4];
        Frag a0, a1;
        a0.u = *reinterpret_cast<const uint4*>(src);
        a1.u = *reinterpret_cast<const uint4*>(src + 8);
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
#pragma unroll
          for (int c = 0; c < 4; ++c) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.f[c], bfrag[r][j][0].f[c], acc[i][j], 0, 0, 0);
#pragma unroll
          for (int c = 0; c < 4; ++c) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.f[c], bfrag[r][j][F32 ? 1 : 0].f[c], acc[i][j], 0, 0, 0);
        }
      } else {
        // k-chunk g: taps s = 2g, 2g+1 = cells tw + 1 + 2g, tw + 2 + 2g of patch row th + r
        const T* src = &tile[((th + r) * PW + tw + 1 + 2 * g) * 4];
        union { uint2 u[2]; t_bf16x8 v; } a;
        a.u[0] = *reinterpret_cast<const uint2*>(src);
        a.u[1] = *reinterpret_cast<const uint2*>(src + 4);
#pragma unroll
        for (int j = 0; j < NJ; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, bfrag[r][j][0].v, acc[i][j], 0, 0, 0);
      }
    }
  }

  float s1[NJ], s2[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) { s1[j] = 0.0f; s2[j] = 0.0f; }
  T* stage = stage_all + wave * (32 * SW);
  const bool interior = h0 + TH <= H && w0 + TW <= W && CW == NJ * 32;
  if (UPSUM) {
    T* out_n = out + (int64_t)n * (H >> 1) * (W >> 1) * CW;
    if (interior) thin_epilogue<T, NJ, 3, true>(acc, bs, stage, out_n, H, W, CW, h0, w0, TW, tw_shift, act, false, s1, s2);
    else thin_epilogue<T, NJ, 0, true>(acc, bs, stage, out_n, H, W, CW, h0, w0, TW, tw_shift, act, false, s1, s2);
  } else {
    T* out_n = out + (int64_t)n * H * W * CW;
    const bool stats = partial != nullptr;
    if (!interior || act == ACT_SIGMOID || (stats && act != ACT_NONE))
      thin_epilogue<T, NJ, 0, false>(acc, bs, stage, out_n, H, W, CW, h0, w0, TW, tw_shift, act, stats, s1, s2);
    else if (stats) thin_epilogue<T, NJ, 1, false>(acc, bs, stage, out_n, H, W, CW, h0, w0, TW, tw_shift, act, true, s1, s2);
    else if (act == ACT_RELU) thin_epilogue<T, NJ, 2, false>(acc, bs, stage, out_n, H, W, CW, h0, w0, TW, tw_shift, act, false, s1, s2);
    else thin_epilogue<T, NJ, 3, false>(acc, bs, stage, out_n, H, W, CW, h0, w0, TW, tw_shift, act, false, s1, s2);
    if (stats) {
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const float t1 = s1[j] + __shfl_xor(s1[j], 32, 64);
        const float t2 = s2[j] + __shfl_xor(s2[j], 32, 64);
        if (lane < 32) { sRed[wave][0][j * 32 + col_lane] = t1; sRed[wave][1][j * 32 + col_lane] = t2; }
      }
      __syncthreads();
      for (int i = tid; i < 2 * NJ * 32; i += NT) {
        const int q = i / (NJ * 32), c = i % (NJ * 32);
        if (c < CW)
          partial[((int64_t)blockIdx.x * 2 + q) * CW + c] = sRed[0][q][c] + sRed[1][q][c] + sRed[2][q][c] + sRed[3][q][c];
      }
    }
  }
}

// ---------------------------------------------------------------------------
// thin weight gradient:  D[cw][k] = sum over wide pixels q = (n,i,j) of wide[q][cw] * B[q][k],
//   k = 16*r + 4*s + ct,   B[q][k] = sum_{a,b <= up} thin[n][ct][(i<<up) + r - 1 + a][(j<<up) + s - 1 + b].
// first layer (up = 0): thin is the layer input, wide the output gradient: dW[cw][ct][r][s] = D[cw][k];
// last layer: thin is the output gradient (at the resolution of the conv), wide the layer input
// (at the stored resolution, which the conv reads through the x2 upsample if up = 1), and the
// taps come out mirrored: dW[ct][cw][2-r][2-s] = D[cw][k].
// The pixel is the reduction index of the MFMA; both operands are pixel-major in LDS (the wide
// slab as loaded, the thin patch as described above, where B[q][16r .. 16r+11] is a contiguous
// run and the next pixel starts 4 << up values later) and are read with the transposing LDS load:
// within 16 lanes, lane 4*j+q supplies the address of 4 values of pixel j, lane i receives
// value i of pixels 0..3.  A workgroup walks over patches of 256 wide pixels, each wave owning
// 64 of them, and accumulates in registers; at the end the four waves are summed through LDS
// in a fixed order and one partial [cw][64] is written.
// ---------------------------------------------------------------------------
__device__ __forceinline__ t_bf16x8 thin_tr_frag(const bf16_t* p0, const bf16_t* p1) {
  t_short4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((t_lds_short4*)p0);
  t_short4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((t_lds_short4*)p1);
  union { short s[8]; t_bf16x8 v; } u;
  u.s[0] = lo[0]; u.s[1] = lo[1]; u.s[2] = lo[2]; u.s[3] = lo[3];
  u.s[4] = hi[0]; u.s[5] = hi[1]; u.s[6] = hi[2]; u.s[7] = hi[3];
  return u.v;
}

// T = float: v_mfma_f32_32x32x2_f32, two pixels per step: lane l supplies pixel l/32 of the pair — wide channel l%32 of
// it for one operand, column k = l%32 of B for the other, both plain 4-byte LDS reads (no transposition needed: the
// 32 lanes of a half-wave read 32 consecutive channels, or the 2 x 16 values of two patch rows).  Behind an upsample
// the four terms of B are added before the MFMA.
template <typename T, int MI>   // CW = 32*MI wide channels
__global__ __launch_bounds__(NT) void k_thin_wgrad_mfma(const T* __restrict__ thin, const T* __restrict__ wide,
                                                        float* __restrict__ partial, int Hq, int Wq, int CT, int up,
                                                        int TW, int tw_shift, int tiles_w, int tiles_h, int ntiles,
                                                        int vec) {
  constexpr bool F32 = sizeof(T) == 4;
  constexpr int EPC = 16 / (int)sizeof(T);      // elements per 16-byte chunk
  constexpr int CW = 32 * MI;
  constexpr int LA = CW + (F32 ? 32 : 16);      // (binary32: the two pixels of a pair fall into different halves of the banks)
  constexpr int MAXT = 1320;                    // ((TH<<up)+2) * ((TW<<up)+4) cells for every TW in {16,32,64}, up in {0,1}
  __shared__ __attribute__((aligned(16))) T tile[MAXT * 4];
  __shared__ __attribute__((aligned(16))) T sW[NT * LA];
  const int TH = NT >> tw_shift;
  const int IW = TW << up, PW = IW + 4, rows = (TH << up) + 2;
  const int Ht = Hq << up, Wt = Wq << up;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int grp = lane >> 4, sl = lane & 15;

  t_floatx16 acc[MI][2];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  for (int t = blockIdx.x; t < ntiles; t += gridDim.x) {
    int b = t;
    const int tx = b % tiles_w; b /= tiles_w;
    const int ty = b % tiles_h;
    const int n = b / tiles_h;
    const int h0 = ty * TH, w0 = tx * TW;
    // wide slab first (its loads are the long ones): patch pixel p = th*TW + tw -> row p of sW
    constexpr int CPP = CW / EPC;               // 16-byte chunks per pixel
    uint4 wv[CPP];
#pragma unroll
    for (int c = 0; c < CPP; ++c) {
      const int idx = c * NT + tid;
      const int p = idx / CPP, ch = idx % CPP;
      const int hh = h0 + (p >> tw_shift), ww = w0 + (p & (TW - 1));
      const bool ok = hh < Hq && ww < Wq;
      wv[c] = *reinterpret_cast<const uint4*>(wide + (((int64_t)n * Hq + min(hh, Hq - 1)) * Wq + min(ww, Wq - 1)) * CW + ch * EPC);
      if (!ok) { wv[c].x = 0u; wv[c].y = 0u; wv[c].z = 0u; wv[c].w = 0u; }
    }
    __syncthreads();                            // previous patch fully consumed
    thin_fill_patch(tile, thin + (int64_t)n * CT * Ht * Wt, Ht, Wt, CT, (h0 << up) - 1, w0 << up, rows, IW, vec != 0);
#pragma unroll
    for (int c = 0; c < CPP; ++c) {
      const int idx = c * NT + tid;
      *reinterpret_cast<uint4*>(&sW[(idx / CPP) * LA + (idx % CPP) * EPC]) = wv[c];
    }
    __syncthreads();
    if constexpr (F32) {
      const int half = lane >> 5, nl = lane & 31;
      int boff[2];                              // column k = 32 j + nl of B: k = 16 r + 4 s + ct (columns 48..63 unused: any finite data)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int kq = 32 * j + nl;
        boff[j] = (min(kq >> 4, 2) * PW + ((kq >> 2) & 3)) * 4 + (kq & 3);
      }
      const float* tf = reinterpret_cast<const float*>(tile);
      const float* wf = reinterpret_cast<const float*>(sW);
#pragma unroll 4
      for (int ks = 0; ks < 32; ++ks) {         // this wave's 64 pixels, two per step
        const int p = wave * 64 + 2 * ks + half;
        const int th = p >> tw_shift, tw = p & (TW - 1);
        float a[MI], b[2];
#pragma unroll
        for (int i = 0; i < MI; ++i) a[i] = wf[p * LA + i * 32 + nl];
        const float* q0 = tf + ((th << up) * PW + 1 + (tw << up)) * 4;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const float* q = q0 + boff[j];
          b[j] = up ? (q[0] + q[4]) + (q[PW * 4] + q[PW * 4 + 4]) : q[0];
        }
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
      }
    } else {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int p0 = wave * 64 + ks * 16;       // 16 consecutive pixels of one patch row
      const int th = p0 >> tw_shift, tw0 = p0 & (TW - 1);
      const int psub = 8 * (grp >> 1) + (sl >> 2);
      t_bf16x8 a[MI];
#pragma unroll
      for (int i = 0; i < MI; ++i) {
        const bf16_t* q = &sW[(p0 + psub) * LA + i * 32 + 16 * (grp & 1) + 4 * (sl & 3)];
        a[i] = thin_tr_frag(q, q + 4 * LA);
      }
      for (int ab = 0; ab < (1 << (2 * up)); ++ab) {
        const int a_ = ab >> 1, b_ = ab & 1;
        t_bf16x8 bfr[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int r = min(2 * j + (grp & 1), 2);  // columns 48..63 are unused: any finite data
          const bf16_t* q = &tile[(((th << up) + r + a_) * PW + 1 + ((tw0 + psub) << up) + (sl & 3) + b_) * 4];
          bfr[j] = thin_tr_frag(q, q + (16 << up));
        }
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], bfr[j], acc[i][j], 0, 0, 0);
      }
    }
    }
  }
  // sum the four waves in a fixed order through LDS (reusing the slab), then write [cw][64]
  float* sF = reinterpret_cast<float*>(sW);     // MI*2*1024 floats <= NT*LA*2 bytes
  for (int wv = 0; wv < 4; ++wv) {
    __syncthreads();
    if (wave == wv) {
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int row = i * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3), col = j * 32 + (lane & 31);
            if (wv == 0) sF[row * 64 + col] = acc[i][j][e];
            else sF[row * 64 + col] += acc[i][j][e];
          }
    }
  }
  __syncthreads();
  for (int i = tid; i < CW * 64; i += NT) partial[(int64_t)blockIdx.x * CW * 64 + i] = sF[i];
}

// dW = sum over blocks of partial[b][cw][16*r + 4*s + ct]; 16 lanes per output, each summing
// every 16th block, then a fixed-order shuffle tree.
// mode 0: dW[cw][ct][r][s];  mode 1: dW[ct][cw][2-r][2-s]
__global__ void k_thin_wgrad_mfma_reduce(const float* __restrict__ partial, int nblocks, int CW, int CT, int mode,
                                         float* __restrict__ dw) {
  const int total = CW * CT * 9;
  const int gid = (blockIdx.x * NT + threadIdx.x) >> 4, sub = threadIdx.x & 15;
  const int i = gid < total ? gid : total - 1;
  const int tap = i % 9, ct = (i / 9) % CT, cw = i / (9 * CT);
  const int r = tap / 3, s = tap % 3;
  const float* src = partial + (int64_t)cw * 64 + 16 * r + 4 * s + ct;
  float acc = 0.0f;
#pragma unroll 4
  for (int b = sub; b < nblocks; b += 16) acc += src[(int64_t)b * CW * 64];
  acc += __shfl_xor(acc, 1, 64);
  acc += __shfl_xor(acc, 2, 64);
  acc += __shfl_xor(acc, 4, 64);
  acc += __shfl_xor(acc, 8, 64);
  if (gid < total && sub == 0) {
    const int64_t o = mode == 0 ? (int64_t)i : (((int64_t)ct * CW + cw) * 3 + (2 - r)) * 3 + (2 - s);
    dw[o] = acc;
  }
}

// ---------------------------------------------------------------------------
// The vector path of thin_fill_patch in two halves, so that the global loads of the next patch are
// in flight while the current one is computed.  rows * IW/8 <= NT and 2 * rows <= NT (one interior
// chunk and one halo cell per thread at most): true for every patch of 256 pixels at least 16 wide.
// ---------------------------------------------------------------------------
struct ThinPatchRegs { uint4 c[4]; uint32_t e[4]; };

__device__ __forceinline__ void thin_patch_load(ThinPatchRegs& R, const bf16_t* __restrict__ img, int H, int W, int CT,
                                                int h_first, int w_first, int rows, int IW) {
  const int tid = threadIdx.x;
  const int64_t HW = (int64_t)H * W;
  const int cpr = IW >> 3, cshift = 31 - __clz(cpr);      // IW is a power of two: no divisions
  if (tid < rows * cpr) {
    const int pr = tid >> cshift, c = tid & (cpr - 1);
    const int hh = h_first + pr, ww = w_first + 8 * c;
    const int64_t off = (int64_t)min(max(hh, 0), H - 1) * W + min(ww, W - 8);
#pragma unroll
    for (int ci = 0; ci < 4; ++ci) R.c[ci] = *reinterpret_cast<const uint4*>(img + (int64_t)min(ci, CT - 1) * HW + off);
  }
  const int hidx = NT - 1 - tid;
  if (hidx < rows * 2) {
    const int pr = hidx >> 1, side = hidx & 1;
    const int hh = h_first + pr, ww = side ? w_first + IW : w_first - 1;
    const int64_t off = (int64_t)min(max(hh, 0), H - 1) * W + min(max(ww, 0), W - 1);
#pragma unroll
    for (int ci = 0; ci < 4; ++ci) R.e[ci] = (uint32_t)img[(int64_t)min(ci, CT - 1) * HW + off];
  }
}

__device__ __forceinline__ void thin_patch_store(const ThinPatchRegs& R, bf16_t* __restrict__ tile, int H, int W, int CT,
                                                 int h_first, int w_first, int rows, int IW) {
  const int PW = IW + 4;
  const int tid = threadIdx.x;
  const int cpr = IW >> 3, cshift = 31 - __clz(cpr);
  if (tid < rows * cpr) {
    const int pr = tid >> cshift, c = tid & (cpr - 1);
    const int hh = h_first + pr, ww = w_first + 8 * c;
    const bool ok = hh >= 0 && hh < H && ww < W;
    uint32_t v[4][4];
#pragma unroll
    for (int ci = 0; ci < 4; ++ci) {
      const bool keep = ok && ci < CT;
      v[ci][0] = keep ? R.c[ci].x : 0u; v[ci][1] = keep ? R.c[ci].y : 0u;
      v[ci][2] = keep ? R.c[ci].z : 0u; v[ci][3] = keep ? R.c[ci].w : 0u;
    }
    bf16_t* dst = tile + ((int64_t)pr * PW + 2 + 8 * c) * 4;
#pragma unroll
    for (int k = 0; k < 4; ++k) {                // word k holds pixels 2k (low half) and 2k+1 (high half)
      uint4 o;
      o.x = (v[0][k] & 0xFFFFu) | (v[1][k] << 16);
      o.y = (v[2][k] & 0xFFFFu) | (v[3][k] << 16);
      o.z = (v[0][k] >> 16) | (v[1][k] & 0xFFFF0000u);
      o.w = (v[2][k] >> 16) | (v[3][k] & 0xFFFF0000u);
      *reinterpret_cast<uint4*>(dst + 8 * k) = o;
    }
  }
  const int hidx = NT - 1 - tid;
  if (hidx < rows * 2) {
    const int pr = hidx >> 1, side = hidx & 1;
    const int hh = h_first + pr, ww = side ? w_first + IW : w_first - 1;
    const bool ok = hh >= 0 && hh < H && ww >= 0 && ww < W;
    uint32_t e[4];
#pragma unroll
    for (int ci = 0; ci < 4; ++ci) e[ci] = (ok && ci < CT) ? R.e[ci] : 0u;
    const uint32_t lo = e[0] | (e[1] << 16), hi = e[2] | (e[3] << 16);
    if (side) *reinterpret_cast<uint4*>(tile + ((int64_t)pr * PW + IW + 2) * 4) = make_uint4(lo, hi, 0u, 0u);
    else *reinterpret_cast<uint4*>(tile + (int64_t)pr * PW * 4) = make_uint4(0u, 0u, lo, hi);
  }
}

// ---------------------------------------------------------------------------
// First layer followed by batch-norm, ReLU and 2x2 max-pool, with its convolution output never in
// memory.  K = 27 makes the convolution nearly free on the matrix cores, while its output is the
// largest tensor of the network (C_out/C_in times the input): every pass that needs the output
// recomputes it from the input patch instead of reading it.  Row quads of the accumulator tiles are
// 2x2 pooling windows (thin_row_pixel<true>), so a lane holds the four candidates x_0..x_3 of a window.
//   PASS 0  column statistics of the rounded convolution output -> partial[block][sum | sum sq][CW]
//   PASS 1  pooled activation  out[n][H/2][W/2][CW] = max_k relu(scale*x_k + shift)
//   PASS 2  sums of the batch-norm backward: partial[block][sum dy | sum dy*xhat][CW], dy being the
//           pooled gradient at the window's winner where its pre-activation is positive
//   PASS 3  dx_k = scale*(dy_k - c1 - xhat_k*c2), rounded to storage, kept in LDS as the pixel-major slab
//           the weight-gradient MFMAs of k_thin_wgrad_mfma read: partial[block][CW][64]
//   PASS 4  (not a first layer: the LAST layer's input gradient through its x2 upsample, flipped weights, no bias)
//           out[n][H/2][W/2][CW] = the 2x2 sums of the convolution as k_thin_in_mfma with UPSUM forms them, stored
//           as the ReLU backward of the layer below wants them: zero where that layer's saved activation
//           `dout` [n][H/2][W/2][CW] is not positive; partial[block][0][CW] = column sums of what was stored
//           (the bias gradient of the layer below)
// Rounding to storage and x -> scale*x + shift are monotonic, so the window's maximum activation is
// relu(scale*x_w + shift) with x_w the rounded maximum of the window for scale > 0, the minimum for
// scale < 0, x_0 for scale = 0 (all equal: the first wins) — passes 1 and 2 need nothing else of the
// window, and give the bits of k_post_forward / PostBwdWindow.  Pass 3 finds the winner as the first
// k whose pre-activation equals the maximum, and evaluates dx_k as alpha*x_k + beta with alpha = -scale*c2*invstd,
// beta = scale*(c2*invstd*mean - c1), and beta + scale*dy at the winner: the formula of k_post_bwd_apply up to
// binary32 rounding, before the rounding to storage.
// Patches are interior (H, W multiples of the patch); a workgroup computes CW = 32*NJ of the layer's CWT wide
// channels (blockIdx.y selects which: 128 channels run as two halves), the input is 16-byte aligned with
// W % 8 == 0; a workgroup walks over patches t = blockIdx.x, blockIdx.x + gridDim.x, ... and has the
// next patch's global loads in flight while it computes.
// ---------------------------------------------------------------------------
template <int NJ, int PASS>
__global__ __launch_bounds__(NT, (PASS == 3 && NJ == 2) ? 2 : 3) void k_thin_first(
    const bf16_t* __restrict__ thin, const bf16_t* __restrict__ wfrag, const float* __restrict__ bias,
    const float* __restrict__ bn_vec, const bf16_t* __restrict__ dout, bf16_t* __restrict__ out,
    float* __restrict__ partial, int H, int W, int CT, int CWT, int TW, int tw_shift, int tiles_w, int tiles_h,
    int ntiles) {
  constexpr int CW = NJ * 32;
  constexpr int MAXT = 408;                     // (TH+2)*(TW+4) cells for every TW in {16,32,64}
  constexpr int SW = CW + 8;                    // row stride of the staged pooled outputs
  constexpr int LA = CW + 16;                   // row stride of the gradient slab
  constexpr int CPR = CW / 8;                   // 16-byte chunks per pixel
  constexpr int GCH = 64 * CPR;                 // chunks of the pooled-gradient tile (64 windows)
  constexpr int GPT = (GCH + NT - 1) / NT;
  __shared__ __attribute__((aligned(16))) bf16_t tile[MAXT * 4];
  __shared__ __attribute__((aligned(16))) bf16_t sG[(PASS == 2 || PASS == 3) ? 64 * CW : 8];
  __shared__ __attribute__((aligned(16))) bf16_t sW[PASS == 3 ? NT * LA : ((PASS == 1 || PASS == 4) ? 4 * 8 * SW : 8)];
  __shared__ float sRed[(PASS == 0 || PASS == 2 || PASS == 4) ? 4 * 2 * CW : 1];
  const int TH = NT >> tw_shift;
  const int PW = TW + 4;
  const int Hq = H >> 1, Wq = W >> 1;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int frag_row = lane & 31, g = lane >> 5, col_lane = lane & 31;
  const int c0 = blockIdx.y * CW;               // this workgroup's CW of the layer's CWT wide channels

  t_bf16x8 bfrag[3][NJ];
#pragma unroll
  for (int r = 0; r < 3; ++r)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
      bfrag[r][j] = *reinterpret_cast<const t_bf16x8*>(&wfrag[((c0 + j * 32 + frag_row) * 3 + r) * 16 + g * 8]);
  float bs[NJ], sc[NJ], sh[NJ], mu[NJ], is[NJ], al[NJ], be[NJ], s1[NJ], s2[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int c = c0 + j * 32 + col_lane;
    bs[j] = bias ? bias[c] : 0.0f;
    sc[j] = (PASS >= 1 && PASS <= 3) ? bn_vec[c] : 1.0f;
    sh[j] = (PASS >= 1 && PASS <= 3) ? bn_vec[CWT + c] : 0.0f;
    mu[j] = (PASS == 2 || PASS == 3) ? bn_vec[2 * CWT + c] : 0.0f;
    is[j] = (PASS == 2 || PASS == 3) ? bn_vec[3 * CWT + c] : 1.0f;
    const float c1 = PASS == 3 ? bn_vec[4 * CWT + c] : 0.0f;
    const float c2 = PASS == 3 ? bn_vec[5 * CWT + c] : 0.0f;
    al[j] = -(sc[j] * c2) * is[j];
    be[j] = sc[j] * (c2 * is[j] * mu[j] - c1);
    s1[j] = 0.0f; s2[j] = 0.0f;
  }
  // Every loop-invariant load has landed before the first patch is requested: the load counter completes in order, so
  // a wait for one of these values at its first use inside the loop would, in every iteration, also wait for the
  // next patch's loads issued just before (seen in the compiled kernel: s_waitcnt vmcnt(0) in the middle of the
  // arithmetic).  A use here makes the compiler wait here, once.
#if defined(__HIP_DEVICE_COMPILE__)
#pragma unroll
  for (int r = 0; r < 3; ++r)
#pragma unroll
    for (int j = 0; j < NJ; ++j) asm volatile("" : "+v"(bfrag[r][j]));
#pragma unroll
  for (int j = 0; j < NJ; ++j)
    asm volatile("" : "+v"(bs[j]), "+v"(sc[j]), "+v"(sh[j]), "+v"(mu[j]), "+v"(is[j]), "+v"(al[j]), "+v"(be[j]));
#endif
  t_floatx16 wacc[PASS == 3 ? NJ : 1][2];
  if (PASS == 3) {
#pragma unroll
    for (int i = 0; i < NJ; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) wacc[i][j][e] = 0.0f;
  }

  // patch t: image n, rows h0 .., columns w0 ..
  auto where = [&](int t, int& n, int& h0, int& w0) {
    const int tx = t % tiles_w; t /= tiles_w;
    const int ty = t % tiles_h;
    n = t / tiles_h; h0 = ty * TH; w0 = tx * TW;
  };
  ThinPatchRegs pre;
  static_assert(GPT <= 2, "pooled-gradient tile: at most two chunks per thread");
  uint4 gv0 = make_uint4(0u, 0u, 0u, 0u), gv1 = gv0;   // pass 4: this lane's chunks of the companion tensor for i = 0, 1
  float cs[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};   // pass 4: column sums of this lane's chunk
  auto prefetch = [&](int t) {
    int n, h0, w0;
    where(t, n, h0, w0);
    thin_patch_load(pre, thin + (int64_t)n * CT * H * W, H, W, CT, h0 - 1, w0, TH + 2, TW);
    if (PASS == 4) {
      static_assert(8 * CPR <= 64, "one chunk per lane and row group");
      auto chunk = [&](int i) {
        const int G = wave * 16 + i * 8 + min(lane, 8 * CPR - 1) / CPR, ch = lane % CPR;
        const int hq = (h0 >> 1) + (G >> (tw_shift - 1)), wq = (w0 >> 1) + (G & ((TW >> 1) - 1));
        return *reinterpret_cast<const uint4*>(dout + (((int64_t)n * Hq + hq) * Wq + wq) * CWT + c0 + ch * 8);
      };
      gv0 = chunk(0);
      gv1 = chunk(1);
    } else if (PASS >= 2) {
      auto chunk = [&](int idx) {
        const int G = idx / CPR, ch = idx % CPR;
        const int hq = (h0 >> 1) + (G >> (tw_shift - 1)), wq = (w0 >> 1) + (G & ((TW >> 1) - 1));
        return *reinterpret_cast<const uint4*>(dout + (((int64_t)n * Hq + hq) * Wq + wq) * CWT + c0 + ch * 8);
      };
      gv0 = chunk(min(tid, GCH - 1));
      if (GPT == 2) gv1 = chunk(min(NT + tid, GCH - 1));
    }
  };
  prefetch(blockIdx.x);

  for (int t = blockIdx.x; t < ntiles; t += gridDim.x) {
    int n, h0, w0;
    where(t, n, h0, w0);
    __syncthreads();                            // the previous patch is fully consumed
    thin_patch_store(pre, tile, H, W, CT, h0 - 1, w0, TH + 2, TW);
    uint4 cm0 = gv0, cm1 = gv1;                 // (pass 4: the prefetch below overwrites gv0, gv1)
#if defined(__HIP_DEVICE_COMPILE__)
    // (a use here: the compiler waits for these two loads here, before the next patch is requested, instead of at
    // their first use in the arithmetic, where the same wait would also cover the loads just issued)
    if (PASS == 4)
      asm volatile("" : "+v"(cm0.x), "+v"(cm0.y), "+v"(cm0.z), "+v"(cm0.w), "+v"(cm1.x), "+v"(cm1.y), "+v"(cm1.z), "+v"(cm1.w));
#endif
    if (PASS == 2 || PASS == 3) {
      if (tid < GCH) *reinterpret_cast<uint4*>(&sG[tid * 8]) = gv0;
      if (GPT == 2 && NT + tid < GCH) *reinterpret_cast<uint4*>(&sG[(NT + tid) * 8]) = gv1;
    }
    __syncthreads();
    if (t + (int)gridDim.x < ntiles) prefetch(t + gridDim.x);

    t_floatx16 acc[2][NJ];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      int th, tw;
      thin_row_pixel<true>(wave * 64 + i * 32 + frag_row, TW, tw_shift, th, tw);
#pragma unroll
      for (int r = 0; r < 3; ++r) {
        const bf16_t* src = &tile[((th + r) * PW + tw + 1 + 2 * g) * 4];
        union { uint2 u[2]; t_bf16x8 v; } a;
        a.u[0] = *reinterpret_cast<const uint2*>(src);
        a.u[1] = *reinterpret_cast<const uint2*>(src + 4);
#pragma unroll
        for (int j = 0; j < NJ; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, bfrag[r][j], acc[i][j], 0, 0, 0);
      }
    }

    bf16_t* stage = sW + wave * (8 * SW);        // passes 1 and 4
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
#pragma unroll
        for (int eg = 0; eg < 4; ++eg) {
          float x[4];                            // the window's conv outputs before rounding
#pragma unroll
          for (int k = 0; k < 4; ++k) x[k] = acc[i][j][4 * eg + k] + ((PASS == 1 || PASS == 2) ? 0.0f : bs[j]);
          if (PASS == 0) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
              const float d = bf16_to_f32(f32_to_bf16(x[k])) - bs[j];   // statistics about the channel's bias (see k_bn_finalize)
              s1[j] += d;
              s2[j] = fmaf(d, d, s2[j]);
            }
          } else if (PASS == 4) {
            // input gradient through the x2 upsample: the sum over the 2x2 group (k_thin_in_mfma with UPSUM)
            stage[(eg * 2 + g) * SW + j * 32 + col_lane] = f32_to_bf16((x[0] + x[1]) + (x[2] + x[3]));
          } else if (PASS <= 2) {
            // (adding the bias is monotonic too: it is added to the selected accumulator only)
            const float hi = fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3]));
            const float lo = fminf(fminf(x[0], x[1]), fminf(x[2], x[3]));
            const float xw = bf16_to_f32(f32_to_bf16((sc[j] > 0.0f ? hi : (sc[j] < 0.0f ? lo : x[0])) + bs[j]));
            const float pre_w = fmaf(sc[j], xw, sh[j]);
            if (PASS == 1) {
              stage[(eg * 2 + g) * SW + j * 32 + col_lane] = f32_to_bf16(apply_act(pre_w, ACT_RELU));
            } else {
              const int G = wave * 16 + i * 8 + eg * 2 + g;
              const float gg = bf16_to_f32(sG[G * CW + j * 32 + col_lane]);
              const float dyw = pre_w > 0.0f ? gg : 0.0f;
              s1[j] += dyw;
              s2[j] = fmaf(dyw, (xw - mu[j]) * is[j], s2[j]);
            }
          } else {
            const int G = wave * 16 + i * 8 + eg * 2 + g;
            const float gg = bf16_to_f32(sG[G * CW + j * 32 + col_lane]);
            float pk[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
              x[k] = bf16_to_f32(f32_to_bf16(x[k]));
              pk[k] = fmaf(sc[j], x[k], sh[j]);
            }
            const float pm = fmaxf(fmaxf(pk[0], pk[1]), fmaxf(pk[2], pk[3]));
            // the winner (first k whose pre-activation is the maximum) gets beta + scale*dy as its constant term
            const float bw = be[j] + (pm > 0.0f ? sc[j] * gg : 0.0f);
            const bool m0 = pk[0] == pm, m1 = pk[1] == pm, m2 = pk[2] == pm;
            const bool f[4] = {m0, m1 && !m0, m2 && !(m0 || m1), !(m0 || m1 || m2)};
            int th, tw;
            thin_row_pixel<true>(wave * 64 + i * 32 + eg * 8 + g * 4, TW, tw_shift, th, tw);
            bf16_t* dst = &sW[(th * TW + tw) * LA + j * 32 + col_lane];
#pragma unroll
            for (int k = 0; k < 4; ++k)
              dst[((k >> 1) * TW + (k & 1)) * LA] = f32_to_bf16(fmaf(al[j], x[k], f[k] ? bw : be[j]));
          }
        }
      }
      if (PASS == 4) {
        // ReLU backward of the layer below while storing: its saved activation decides, column sums for its bias
        bf16_t* out_n = out + (int64_t)n * Hq * Wq * CWT + c0;
        if (lane < 8 * CPR) {
          const int g8 = lane / CPR, ch = lane % CPR;
          const int G = wave * 16 + i * 8 + g8;
          const int hq = (h0 >> 1) + (G >> (tw_shift - 1)), wq = (w0 >> 1) + (G & ((TW >> 1) - 1));
          const uint4 sv = *reinterpret_cast<const uint4*>(&stage[g8 * SW + ch * 8]);
          const uint4 av = i == 0 ? cm0 : cm1;
          const uint32_t sw[4] = {sv.x, sv.y, sv.z, sv.w}, aw[4] = {av.x, av.y, av.z, av.w};
          uint32_t ow[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const float a_lo = __uint_as_float(aw[q] << 16), a_hi = __uint_as_float(aw[q] & 0xFFFF0000u);
            const uint32_t lo = a_lo > 0.0f ? (sw[q] & 0xFFFFu) : 0u, hi = a_hi > 0.0f ? (sw[q] & 0xFFFF0000u) : 0u;
            cs[2 * q] += __uint_as_float(lo << 16);
            cs[2 * q + 1] += __uint_as_float(hi);
            ow[q] = lo | hi;
          }
          *reinterpret_cast<uint4*>(out_n + ((int64_t)hq * Wq + wq) * CWT + ch * 8) = make_uint4(ow[0], ow[1], ow[2], ow[3]);
        }
      }
      if (PASS == 1) {
        bf16_t* out_n = out + (int64_t)n * Hq * Wq * CWT + c0;
#pragma unroll
        for (int c = 0; c < (8 * CPR + 63) / 64; ++c) {
          const int idx = c * 64 + lane;
          const int g8 = idx / CPR, ch = idx % CPR;
          const int G = wave * 16 + i * 8 + g8;
          const int hq = (h0 >> 1) + (G >> (tw_shift - 1)), wq = (w0 >> 1) + (G & ((TW >> 1) - 1));
          if (idx < 8 * CPR)
            *reinterpret_cast<uint4*>(out_n + ((int64_t)hq * Wq + wq) * CWT + ch * 8) =
                *reinterpret_cast<const uint4*>(&stage[g8 * SW + ch * 8]);
        }
      }
    }

    if (PASS == 3) {
      // The pixel is the reduction index, so a wavefront may sum over any pixels as long as both operands name the
      // same ones: it takes the 64 pixels whose gradients it has just written itself (its 16 pooling windows: two rows
      // of 32 pixels, or four rows of 16 in a 16-wide patch), as four runs of 16 consecutive pixels of one patch row.
      // No workgroup barrier: LDS operations of a wavefront complete in order.
      asm volatile("" ::: "memory");          // (the compiler keeps the reads below behind the stores above)
      const int grp = lane >> 4, sl = lane & 15;
      const int wpr = TW >> 5;                  // wavefronts side by side in a row pair (0: the patch is 16 wide)
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const int th = wpr ? 2 * (wave / wpr) + (ks >> 1) : 4 * wave + ks;
        const int tw0 = wpr ? 32 * (wave % wpr) + 16 * (ks & 1) : 0;
        const int p0 = th * TW + tw0;           // 16 consecutive pixels of one patch row
        const int psub = 8 * (grp >> 1) + (sl >> 2);
        t_bf16x8 a[NJ], bfr[2];
#pragma unroll
        for (int i = 0; i < NJ; ++i) {
          const bf16_t* q = &sW[(p0 + psub) * LA + i * 32 + 16 * (grp & 1) + 4 * (sl & 3)];
          a[i] = thin_tr_frag(q, q + 4 * LA);
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int r = min(2 * j + (grp & 1), 2);  // columns 48..63 are unused: any finite data
          const bf16_t* q = &tile[((th + r) * PW + 1 + tw0 + psub + (sl & 3)) * 4];
          bfr[j] = thin_tr_frag(q, q + 16);
        }
#pragma unroll
        for (int i = 0; i < NJ; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j) wacc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], bfr[j], wacc[i][j], 0, 0, 0);
      }
    }
  }

  if (PASS == 4) {
    // lanes that share a column chunk differ in lane / CPR (lanes beyond 8*CPR hold zeros)
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      for (int off = CPR; off < 64; off <<= 1) cs[t] += __shfl_xor(cs[t], off, 64);
      if (lane < CPR) { sRed[(wave * 2 + 0) * CW + lane * 8 + t] = cs[t]; sRed[(wave * 2 + 1) * CW + lane * 8 + t] = 0.0f; }
    }
  }
  if (PASS == 0 || PASS == 2 || PASS == 4) {
    if (PASS != 4) {
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const float t1 = s1[j] + __shfl_xor(s1[j], 32, 64);
        const float t2 = s2[j] + __shfl_xor(s2[j], 32, 64);
        if (lane < 32) { sRed[(wave * 2 + 0) * CW + j * 32 + col_lane] = t1; sRed[(wave * 2 + 1) * CW + j * 32 + col_lane] = t2; }
      }
    }
    __syncthreads();
    for (int i = tid; i < 2 * CW; i += NT)
      partial[((int64_t)blockIdx.x * 2 + i / CW) * CWT + c0 + i % CW] = (sRed[i] + sRed[2 * CW + i]) + (sRed[4 * CW + i] + sRed[6 * CW + i]);
  }
  if (PASS == 3) {
    // sum the four waves in a fixed order through LDS (reusing the slab), then write [cw][64]
    float* sF = reinterpret_cast<float*>(sW);   // NJ*2*1024 floats <= NT*LA*2 bytes
    for (int wv = 0; wv < 4; ++wv) {
      __syncthreads();
      if (wave == wv) {
#pragma unroll
        for (int i = 0; i < NJ; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
              const int row = i * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3), col = j * 32 + (lane & 31);
              if (wv == 0) sF[row * 64 + col] = wacc[i][j][e];
              else sF[row * 64 + col] += wacc[i][j][e];
            }
      }
    }
    __syncthreads();
    for (int i = tid; i < CW * 64; i += NT) partial[((int64_t)blockIdx.x * CWT + c0) * 64 + i] = sF[i];
  }
}

// ---------------------------------------------------------------------------
// thin-out conv (forward of the last layer, optionally through the x2 upsample):
//   out[n][ct][y][x] = act( b[ct] + sum_{r,s,cw} wide[n][(y+r-1)>>up][(x+s-1)>>up][cw] * W[ct][cw][r][s] )
// as a small GEMM followed by a shifted sum.  For every wide pixel q of a patch (TH x TW pixels
// plus a halo of one) the matrix cores compute
//   Z[q][tap*CT + ct] = sum_cw wide[q][cw] * W[ct][cw][tap]          (N = 9*CT columns, padded to 32*NJ)
// reading each wide pixel once, straight from global memory into the MFMA operand layout (lane l:
// pixel l%32, 8 channels at 16*ks + 8*(l/32)); Z goes to LDS as fp32, and every output pixel then
// adds its nine terms Z[pixel under tap (r,s)][(r,s),ct] in a fixed order.
// wz: bf16 [32*NJ][CW], row tap*CT + ct (zero rows beyond 9*CT).  out planar (+ optional fp32 copy).
// ---------------------------------------------------------------------------
template <typename T>
__global__ void k_thin_pack_wz(const float* __restrict__ wcanon, T* __restrict__ wz, int CT, int CW, int rows) {
  const int i = blockIdx.x * NT + threadIdx.x;
  if (i >= rows * CW) return;
  const int cw = i % CW, col = i / CW;
  float v = 0.0f;
  if (col < 9 * CT) {
    const int ct = col % CT, tap = col / CT;
    v = wcanon[((int64_t)ct * CW + cw) * 9 + tap];
  }
  Store<T>::st(wz + i, v);
}

// T = bf16: one K = 16 MFMA per 16-byte load.  T = float: a 16-byte load holds four channels; component c of the low
// half-wave and component c of the high one are the two K values of a v_mfma_f32_32x32x2_f32 (wz uses the same pairing).
template <typename T, int NJ, int KS>   // 32*NJ >= 9*CT columns, CW = KS * 32/sizeof(T) wide channels
__global__ __launch_bounds__(NT) void k_thin_out_mfma(const T* __restrict__ wide, const T* __restrict__ wz,
                                                      const float* __restrict__ bias, T* __restrict__ out,
                                                      float* __restrict__ out_f32, int Hq, int Wq, int CT, int up,
                                                      int act, int TW, int tw_shift, int tiles_w, int tiles_h) {
  constexpr int CPL = 16 / (int)sizeof(T);      // channels per 16-byte load
  constexpr int CW = 2 * CPL * KS;
  constexpr int ZS = 32 * NJ + 1;               // odd row stride: conflict-free column reads
  constexpr int MAXC = 352;                     // (TH+2)*(TW+2) <= 340 cells for TW in {8,16,32}, rounded up to 32
  constexpr int TPW = 3;                        // row tiles of 32 cells per wave (11 tiles over 4 waves)
  __shared__ float sZ[MAXC * ZS];
  const int TH = NT >> tw_shift;
  const int PW = TW + 2, cells = (TH + 2) * PW;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int b = blockIdx.x;
  const int tx = b % tiles_w; b /= tiles_w;
  const int ty = b % tiles_h;
  const int n = b / tiles_h;
  const int h0 = ty * TH, w0 = tx * TW;        // wide coordinates
  const int frag_row = lane & 31, g = lane >> 5;

  // all global loads of the wave's row tiles first
  uint4 av[TPW][KS];
#pragma unroll
  for (int t = 0; t < TPW; ++t) {
    const int cell = (wave + 4 * t) * 32 + frag_row;
    const int pr = cell / PW, pc = cell - pr * PW;
    const int hh = h0 - 1 + pr, ww = w0 - 1 + pc;
    const bool ok = cell < cells && hh >= 0 && hh < Hq && ww >= 0 && ww < Wq;
    const T* src = wide + (((int64_t)n * Hq + min(max(hh, 0), Hq - 1)) * Wq + min(max(ww, 0), Wq - 1)) * CW + g * CPL;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      av[t][ks] = *reinterpret_cast<const uint4*>(src + ks * 2 * CPL);
      if (!ok) { av[t][ks].x = 0u; av[t][ks].y = 0u; av[t][ks].z = 0u; av[t][ks].w = 0u; }
    }
  }
  uint4 bw[KS][NJ];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
      bw[ks][j] = *reinterpret_cast<const uint4*>(&wz[(j * 32 + frag_row) * CW + ks * 2 * CPL + g * CPL]);

#pragma unroll
  for (int t = 0; t < TPW; ++t) {
    const int rt = wave + 4 * t;
    if (rt * 32 < cells) {                      // uniform per wave
      t_floatx16 acc[NJ];
#pragma unroll
      for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[j][e] = 0.0f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        union { uint4 u; t_bf16x8 v; float f[4]; } a;
        a.u = av[t][ks];
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
          union { uint4 u; t_bf16x8 v; float f[4]; } b;
          b.u = bw[ks][j];
          if constexpr (sizeof(T) == 2) {
            acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, b.v, acc[j], 0, 0, 0);
          } else {
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.f[c], b.f[c], acc[j], 0, 0, 0);
          }
        }
      }
#pragma unroll
      for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int row = rt * 32 + (e >> 2) * 8 + g * 4 + (e & 3);
          sZ[row * ZS + j * 32 + frag_row] = acc[j][e];
        }
    }
  }
  __syncthreads();

  // shifted sums: item -> (ct, y, x) of the output patch, x fastest (planar rows are contiguous)
  const int Hc = Hq << up, Wc = Wq << up;
  const int OW = TW << up, OH = TH << up;
  const int ow_shift = tw_shift + up;
  const int64_t HWc = (int64_t)Hc * Wc;
  // (a tap that falls outside the image reads a halo cell, whose Z row is zero because its input was loaded as
  // zeros: no per-tap bounds checks; -1 >> 1 = -1 addresses the halo as well)
  const int oh_shift = 8 - tw_shift + up;       // OH = (256 / TW) << up
#pragma unroll 2
  for (int item = tid; item < (CT << (oh_shift + ow_shift)); item += NT) {
    const int xl = item & (OW - 1), rr = item >> ow_shift;
    const int yl = rr & (OH - 1), ct = rr >> oh_shift;
    const int y = (h0 << up) + yl, x = (w0 << up) + xl;
    if (y < Hc && x < Wc) {
      float v = bias ? bias[ct] : 0.0f;
#pragma unroll
      for (int r = 0; r < 3; ++r) {
        const int prow = (((y + r - 1) >> up) - (h0 - 1)) * PW;
#pragma unroll
        for (int s_ = 0; s_ < 3; ++s_) v += sZ[(prow + ((x + s_ - 1) >> up) - (w0 - 1)) * ZS + (r * 3 + s_) * CT + ct];
      }
      const float a = apply_act(round_to_storage<T>(v), act);
      const int64_t o = ((int64_t)n * CT + ct) * HWc + (int64_t)y * Wc + x;
      Store<T>::st(out + o, a);
      if (out_f32) out_f32[o] = a;
    }
  }
}

struct ThinTile { int tw, shift, th, tiles_w, tiles_h, blocks; };
ThinTile thin_tile(int n, int h, int w, int max_tw = 64) {
  ThinTile t;
  t.tw = 8; t.shift = 3;
  while (t.tw < max_tw && t.tw < w) { t.tw <<= 1; ++t.shift; }
  t.th = NT / t.tw;
  t.tiles_w = (w + t.tw - 1) / t.tw;
  t.tiles_h = (h + t.th - 1) / t.th;
  t.blocks = n * t.tiles_h * t.tiles_w;
  return t;
}

bool vec_ok(const void* p, int w) { return w % 8 == 0 && ((uintptr_t)p & 15) == 0; }

}  // namespace

bool thin_in_mfma_supported(int ct, int cw, int k, int up, int dtype) {
  if (k != 3 || up || ct < 1 || ct > 4 || cw % 32 != 0) return false;
  // (binary32: the weight operands of 96 or 128 wide channels would not fit the registers beside the accumulators)
  return dtype == AE_BF16 ? cw <= 128 : (dtype == AE_F32 && cw <= 64);
}

int thin_in_mfma_blocks(int n, int h, int w) { return thin_tile(n, h, w).blocks; }

int64_t thin_wfrag_bytes(int cw) { return (int64_t)((cw + 31) / 32) * 32 * 48 * 4; }   // (sized for binary32)

// thin: planar [n][ct][h][w]; out: [n*h*w][cw], or with upsum (h, w even) [n*(h/2)*(w/2)][cw] holding the
// sums over 2x2 pixel groups.  wfrag: scratch of thin_wfrag_bytes(cw) bytes.
int launch_thin_in_mfma(const void* thin, const float* wcanon, void* wfrag, const float* bias, void* out, float* partial,
                        int n, int h, int w, int ct, int cw, int flip, int act, int upsum, int dtype, hipStream_t s) {
  if (!thin_in_mfma_supported(ct, cw, 3, 0, dtype)) return fail(AE_EINVAL, "thin_in_mfma: shape not supported");
  if (upsum && ((h | w) & 1 || partial || act != ACT_NONE)) return fail(AE_EINVAL, "thin_in_mfma: bad 2x2-sum request");
  if ((((uintptr_t)wfrag | (uintptr_t)out) & 15) != 0) return fail(AE_EINVAL, "thin_in_mfma: output and weight scratch must be 16-byte aligned");
  const ThinTile t = thin_tile(n, h, w);
  const int nj = cw / 32;
  const dim3 pgrid((unsigned)((nj * 32 * 48 + NT - 1) / NT));
  if (dtype == AE_BF16) hipLaunchKernelGGL((k_thin_pack_wfrag<bf16_t>), pgrid, dim3(NT), 0, s, wcanon, (bf16_t*)wfrag, ct, cw, nj * 32, flip);
  else hipLaunchKernelGGL((k_thin_pack_wfrag<float>), pgrid, dim3(NT), 0, s, wcanon, (float*)wfrag, ct, cw, nj * 32, flip);
  AE_TRY(launch_status("thin_pack_wfrag"));
  const int vec = vec_ok(thin, w) ? 1 : 0;
#define LAUNCH_TIM(T, NJV, UPV)                                                                                  \
  hipLaunchKernelGGL((k_thin_in_mfma<T, NJV, UPV>), dim3((unsigned)t.blocks), dim3(NT), 0, s, (const T*)thin,    \
                     (const T*)wfrag, bias, (T*)out, partial, h, w, ct, cw, act, t.tw, t.shift,                  \
                     t.tiles_w, t.tiles_h, vec)
#define LAUNCH_TIM_NJ(UPV)                                                              \
  if (dtype == AE_BF16) {                                                               \
    switch (nj) {                                                                       \
      case 1: LAUNCH_TIM(bf16_t, 1, UPV); break;                                        \
      case 2: LAUNCH_TIM(bf16_t, 2, UPV); break;                                        \
      case 3: LAUNCH_TIM(bf16_t, 3, UPV); break;                                        \
      default: LAUNCH_TIM(bf16_t, 4, UPV); break;                                       \
    }                                                                                   \
  } else {                                                                              \
    if (nj == 1) LAUNCH_TIM(float, 1, UPV); else LAUNCH_TIM(float, 2, UPV);             \
  }
  if (upsum) { LAUNCH_TIM_NJ(true) } else { LAUNCH_TIM_NJ(false) }
#undef LAUNCH_TIM_NJ
#undef LAUNCH_TIM
  return launch_status("thin_in_mfma");
}

// First layer + batch-norm + ReLU + 2x2 max-pool with the convolution output recomputed in every
// pass (k_thin_first).  Whole patches only; 32, 64 or 128 output channels.
bool thin_first_supported(int ct, int cw, int k, int up, int dtype, int h, int w) {
  if (dtype != AE_BF16 || !thin_in_mfma_supported(ct, cw, k, up, dtype) || (cw != 32 && cw != 64 && cw != 128) || w % 8 != 0) return false;
  const ThinTile t = thin_tile(1, h, w);
  return t.tw >= 16 && h % t.th == 0 && w % t.tw == 0;
}

// workgroups of a pass (each walks the same number of patches when the patch count is a multiple)
// channels per workgroup column: 64, but 32 in pass 3 (its 64-channel form needs 248 registers, two workgroups per
// compute unit; with 32 channels three fit and the recomputed convolution costs next to nothing)
static int thin_first_nj(int cw, int pass) { return (cw == 32 || pass == 3) ? 1 : 2; }
static int thin_first_grid(int tiles, int cw, int pass) {
  // resident workgroups: registers allow three per compute unit, shared by the workgroup columns
  const int cap = 768 / (cw / (32 * thin_first_nj(cw, pass)));
  return tiles < cap ? tiles : cap;
}
int thin_first_blocks(int n, int h, int w, int cw, int pass) { return thin_first_grid(thin_tile(n, h, w).blocks, cw, pass); }

// pass 0: partial <- column statistics (packs wfrag from wcanon first);  pass 1: out <- pooled activation;
// pass 2: partial <- batch-norm backward sums from the pooled gradient dout;
// pass 3: workspace, dw_canonical <- weight gradient.  Passes 1-3 read the wfrag an earlier pass 0 / pack left.
// pass 4 (last layer's input gradient, see k_thin_first): thin = the planar output gradient, wcanon = the layer's
// weights [ct][cw][3][3] (packed flipped), dout = saved activation of the layer below, out <- masked gradient,
// partial <- column sums ([blocks][2][cw], second row zero).
int launch_thin_first(int pass, const void* thin, const float* wcanon, void* wfrag, const float* bias,
                      const float* bn_vec, const void* dout, void* out, float* partial, float* dw_canonical, int n, int h,
                      int w, int ct, int cw, hipStream_t s) {
  if (pass < 0 || pass > 4 || !thin_first_supported(ct, cw, 3, 0, AE_BF16, h, w))
    return fail(AE_EINVAL, "thin_first: shape not supported");
  if (((uintptr_t)thin & 15) != 0) return fail(AE_EINVAL, "thin_first: input must be 16-byte aligned");
  const ThinTile t = thin_tile(n, h, w);
  const int nj = thin_first_nj(cw, pass);        // 32-channel column tiles per workgroup; more channels: several workgroup columns
  const int halves = cw / (nj * 32);
  if (wcanon) {
    hipLaunchKernelGGL((k_thin_pack_wfrag<bf16_t>), dim3((unsigned)((cw * 48 + NT - 1) / NT)), dim3(NT), 0, s, wcanon,
                       (bf16_t*)wfrag, ct, cw, cw, pass == 4 ? 1 : 0);
    AE_TRY(launch_status("thin_pack_wfrag"));
  }
  const int grid = thin_first_grid(t.blocks, cw, pass);
#define LAUNCH_TF(NJV, PASSV)                                                                                      \
  hipLaunchKernelGGL((k_thin_first<NJV, PASSV>), dim3((unsigned)grid, (unsigned)halves), dim3(NT), 0, s,             \
                     (const bf16_t*)thin, (const bf16_t*)wfrag, bias, bn_vec, (const bf16_t*)dout, (bf16_t*)out,     \
                     partial, h, w, ct, cw, t.tw, t.shift, t.tiles_w, t.tiles_h, t.blocks)
#define LAUNCH_TF_NJ(PASSV) \
  if (nj == 1) LAUNCH_TF(1, PASSV); else LAUNCH_TF(2, PASSV)
  switch (pass) {
    case 0: LAUNCH_TF_NJ(0); break;
    case 1: LAUNCH_TF_NJ(1); break;
    case 2: LAUNCH_TF_NJ(2); break;
    case 3: LAUNCH_TF_NJ(3); break;
    default: LAUNCH_TF_NJ(4); break;
  }
#undef LAUNCH_TF_NJ
#undef LAUNCH_TF
  AE_TRY(launch_status("thin_first"));
  if (pass == 3) {
    const int total = cw * ct * 9;
    hipLaunchKernelGGL(k_thin_wgrad_mfma_reduce, dim3((unsigned)((total * 16 + NT - 1) / NT)), dim3(NT), 0, s, partial,
                       grid, cw, ct, 0, dw_canonical);
    return launch_status("thin_wgrad_mfma_reduce");
  }
  return AE_OK;
}

bool thin_out_mfma_supported(int ct, int cw, int k, int dtype) {
  if (k != 3 || ct < 1 || ct > 4) return false;
  if (dtype == AE_BF16) return cw == 32 || cw == 64 || cw == 128;
  return dtype == AE_F32 && (cw == 32 || cw == 64);   // (binary32: 128 wide channels would hold 192 registers of loads)
}

int64_t thin_out_wz_bytes(int ct, int cw) { return (int64_t)((9 * ct + 31) / 32) * 32 * cw * 4; }   // (sized for binary32)

// wide: [n*hq*wq][cw] (hq = hc >> up); out: planar [n][ct][hc][wc] (+ fp32 copy); wz: scratch of thin_out_wz_bytes
int launch_thin_out_mfma(const void* wide, const float* wcanon, void* wz, const float* bias, void* out, float* out_f32,
                         int n, int hc, int wc, int ct, int cw, int up, int act, int dtype, hipStream_t s) {
  if (!thin_out_mfma_supported(ct, cw, 3, dtype) || up < 0 || up > 1) return fail(AE_EINVAL, "thin_out_mfma: shape not supported");
  if ((((uintptr_t)wide | (uintptr_t)wz) & 15) != 0) return fail(AE_EINVAL, "thin_out_mfma: input and weight scratch must be 16-byte aligned");
  const int hq = hc >> up, wq = wc >> up;
  const ThinTile t = thin_tile(n, hq, wq, 32);  // squarer patches: less halo
  const int nj = (9 * ct + 31) / 32;
  const dim3 pgrid((unsigned)((nj * 32 * cw + NT - 1) / NT));
  if (dtype == AE_BF16) hipLaunchKernelGGL((k_thin_pack_wz<bf16_t>), pgrid, dim3(NT), 0, s, wcanon, (bf16_t*)wz, ct, cw, nj * 32);
  else hipLaunchKernelGGL((k_thin_pack_wz<float>), pgrid, dim3(NT), 0, s, wcanon, (float*)wz, ct, cw, nj * 32);
  AE_TRY(launch_status("thin_pack_wz"));
#define LAUNCH_TOM(T, NJV, KSV)                                                                                  \
  hipLaunchKernelGGL((k_thin_out_mfma<T, NJV, KSV>), dim3((unsigned)t.blocks), dim3(NT), 0, s, (const T*)wide,   \
                     (const T*)wz, bias, (T*)out, out_f32, hq, wq, ct, up, act, t.tw, t.shift, t.tiles_w, t.tiles_h)
#define LAUNCH_TOM_KS(NJV)                                                         \
  if (dtype == AE_BF16) {                                                          \
    switch (cw) {                                                                  \
      case 32: LAUNCH_TOM(bf16_t, NJV, 2); break;                                  \
      case 64: LAUNCH_TOM(bf16_t, NJV, 4); break;                                  \
      default: LAUNCH_TOM(bf16_t, NJV, 8); break;                                  \
    }                                                                              \
  } else {                                                                         \
    if (cw == 32) LAUNCH_TOM(float, NJV, 4); else LAUNCH_TOM(float, NJV, 8);       \
  }
  if (nj == 1) { LAUNCH_TOM_KS(1) } else { LAUNCH_TOM_KS(2) }
#undef LAUNCH_TOM_KS
#undef LAUNCH_TOM
  return launch_status("thin_out_mfma");
}

bool thin_wgrad_mfma_supported(int ct, int cw, int wq, int dtype) {
  if (ct < 1 || ct > 4 || cw % 32 != 0 || wq < 16) return false;
  return dtype == AE_BF16 ? cw <= 128 : (dtype == AE_F32 && cw <= 64);   // (binary32: the wide slab of a patch is 256 x cw x 4 bytes of LDS)
}

int thin_wgrad_mfma_blocks(int n, int hq, int wq) {
  const int tiles = thin_tile(n, hq, wq).blocks;
  return tiles < 768 ? tiles : 768;             // upper bound of the persistent grid (sizes the partial buffer)
}
// Persistent workgroups actually launched: as many as are resident at once (registers allow
// three per compute unit for 32 wide channels, two for 64, one beyond), so that every
// workgroup walks the same number of patches and nobody waits for a second round.
static int thin_wgrad_mfma_grid(int tiles, int cw, int dtype) {
  const int per_cu = dtype == AE_F32 ? 1 : (cw <= 32 ? 3 : (cw <= 64 ? 2 : 1));   // (binary32: LDS allows one)
  const int cap = 256 * per_cu;
  return tiles < cap ? tiles : cap;
}

int64_t thin_wgrad_mfma_workspace_floats(int n, int hq, int wq, int cw) {
  return (int64_t)thin_wgrad_mfma_blocks(n, hq, wq) * cw * 64;
}

// wide: [n*hq*wq][cw].  mode 0 (first layer): thin = planar layer input [n][ct][hq][wq], up = 0.
// mode 1 (last layer): thin = planar output gradient [n][ct][hq<<up][wq<<up].
int launch_thin_wgrad_mfma(const void* thin, const void* wide, float* workspace, float* dw_canonical, int n, int hq,
                           int wq, int ct, int cw, int mode, int up, int dtype, hipStream_t s) {
  if (!thin_wgrad_mfma_supported(ct, cw, wq, dtype) || up < 0 || up > 1 || (mode == 0 && up))
    return fail(AE_EINVAL, "thin_wgrad_mfma: shape not supported");
  if (((uintptr_t)wide & 15) != 0) return fail(AE_EINVAL, "thin_wgrad_mfma: the wide tensor must be 16-byte aligned");
  const ThinTile t = thin_tile(n, hq, wq);
  const int nblk = thin_wgrad_mfma_grid(t.blocks, cw, dtype);
  const int vec = vec_ok(thin, wq << up) ? 1 : 0;
#define LAUNCH_TWM(T, MIV)                                                                                      \
  hipLaunchKernelGGL((k_thin_wgrad_mfma<T, MIV>), dim3((unsigned)nblk), dim3(NT), 0, s, (const T*)thin,          \
                     (const T*)wide, workspace, hq, wq, ct, up, t.tw, t.shift, t.tiles_w, t.tiles_h, t.blocks, vec)
  if (dtype == AE_F32) {
    if (cw == 32) LAUNCH_TWM(float, 1); else LAUNCH_TWM(float, 2);
  } else {
    switch (cw / 32) {
      case 1: LAUNCH_TWM(bf16_t, 1); break;
      case 2: LAUNCH_TWM(bf16_t, 2); break;
      case 3: LAUNCH_TWM(bf16_t, 3); break;
      default: LAUNCH_TWM(bf16_t, 4); break;
    }
  }
#undef LAUNCH_TWM
  AE_TRY(launch_status("thin_wgrad_mfma"));
  const int total = cw * ct * 9;
  hipLaunchKernelGGL(k_thin_wgrad_mfma_reduce, dim3((unsigned)((total * 16 + NT - 1) / NT)), dim3(NT), 0, s, workspace,
                     nblk, cw, ct, mode, dw_canonical);
  return launch_status("thin_wgrad_mfma_reduce");
}

}  // namespace ae
