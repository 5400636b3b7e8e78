// ae_fused_small.hip — the whole forward pass of a SMALL-IMAGE autoencoder in three launches.
//
// A network of the shape
//     conv3+bn+relu+pool2, conv3+bn+relu+pool2, flatten, fc, pnorm, awgn, fc, reshape, up2+conv3+relu, up2+conv3+sigmoid
// on images of at most 32 x 32 pixels (the smallest workload: 64 samples of 1 x 28 x 28, 0.29 GFLOP per batch)
// is bound by the launch-to-launch latency of its ~20 layer kernels, not by any roof.  Here one workgroup owns one
// sample and keeps that sample's tensors in LDS; batch-norm with batch statistics is the only coupling between
// samples, so a launch boundary stands exactly where a layer needs the statistics of the whole batch:
//   k_small_conv1   conv 1 of the sample, its output (for the next launch) and per-sample partial statistics;
//   k_small_conv2   statistics of layer 1 finished by every workgroup for itself (fixed order, double), batch-norm +
//                   ReLU + max-pool into LDS, conv 2, its output and partial statistics;
//   k_small_tail    statistics of layer 2, batch-norm + ReLU + max-pool, flatten, fc, power normalisation, noise,
//                   fc, reshape, both upsampled convolutions, sigmoid — all in LDS, y written once.
// Arithmetic is plain binary32 FMA on the vector ALUs (these layers are far too small for the matrix cores);
// definitions as in aemodel.h.  No activation is kept for a backward pass: the executor takes this path only for a
// model in inference mode.
#include <hip/hip_runtime.h>

#include "ae_device.h"
#include "ae_internal.h"
#include "ae_philox.h"

namespace ae {
namespace {

constexpr int NT_MAX = 256;     // threads per workgroup (more wavefronts per sample were measured slower)
constexpr int NT_CONV2 = 256;
constexpr int COB = 16;        // output channels per accumulator block
#define NT ((int)blockDim.x)

// sum over the workgroup of `v` (every thread contributes), result in thread 0 only; red: NT/64 floats of LDS
__device__ __forceinline__ float block_sum_to0(float v, float* red) {
  v = wave_sum(v);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  __syncthreads();
  if (lane == 0) red[wave] = v;
  __syncthreads();
  float t = 0.0f;
  if (threadIdx.x == 0)
    for (int i = 0; i < NT / 64; ++i) t += red[i];
  return t;
}

// Batch-norm vectors of a layer from the per-sample partial sums (taken about the conv bias): every workgroup
// computes them for itself in double, in a fixed order — thread (g, c) adds the samples g, g + G, ... of channel c
// (independent loads, all in flight together), then the G group sums of a channel are added in index order.
// scale[c] = gamma * invstd, shift[c] = beta - mean * scale.  The first BT = 256 threads do this; tmp: 2 * BT doubles.
__device__ __forceinline__ void bn_vectors(const float* __restrict__ partial, int B, int C, double inv_rows,
                                           const float* __restrict__ bias, const float* __restrict__ gamma_beta,
                                           float* scale, float* shift, double* tmp) {
  constexpr int BT = 256;
  const int G = BT / C > 0 ? BT / C : 1;           // sample groups per channel (C <= BT)
  const int c = threadIdx.x % C, g = threadIdx.x / C;
  double s1 = 0.0, s2 = 0.0;
  if (g < G) {
#pragma unroll 4
    for (int b = g; b < B; b += G) {
      s1 += (double)partial[((int64_t)b * 2) * C + c];
      s2 += (double)partial[((int64_t)b * 2 + 1) * C + c];
    }
  }
  if ((int)threadIdx.x < BT) {
    tmp[threadIdx.x] = s1;
    tmp[BT + threadIdx.x] = s2;
  }
  __syncthreads();
  if ((int)threadIdx.x < C) {
    double t1 = 0.0, t2 = 0.0;
    for (int q = 0; q < G; ++q) { t1 += tmp[q * C + c]; t2 += tmp[BT + q * C + c]; }
    const double dm = t1 * inv_rows;
    double var = t2 * inv_rows - dm * dm;
    if (var < 0.0) var = 0.0;
    const double mean = dm + (double)bias[c];
    const double invstd = 1.0 / sqrt(var + 1e-5);
    const double sc = (double)gamma_beta[c] * invstd;
    scale[c] = (float)sc;
    shift[c] = (float)((double)gamma_beta[C + c] - mean * sc);
  }
}

// One 3x3 convolution (zero padding) of a planar LDS image src[cin][hs*ws], read through an optional x2
// nearest-neighbour upsample (UP: the convolution runs at 2hs x 2ws), for the output channels [co0, co0 + NCO):
// weights wl[(ci*9 + tap)*NCO + k] in LDS (every lane reads the same address: a broadcast; scalar loads of the
// weights straight from global memory were measured slower).  Thread-per-pixel; acc holds the NCO results of (y, x).
template <int NCO, bool UP>
__device__ __forceinline__ void conv3_pixel(const float* src, const float* wl, int cin, int hs, int ws, int y, int x,
                                            float (&acc)[NCO]) {
  const int hc = UP ? 2 * hs : hs, wc = UP ? 2 * ws : ws;
  int off[9];
  bool ok[9];
#pragma unroll
  for (int r = 0; r < 3; ++r)
#pragma unroll
    for (int s = 0; s < 3; ++s) {
      const int yy = y + r - 1, xx = x + s - 1;
      ok[r * 3 + s] = yy >= 0 && yy < hc && xx >= 0 && xx < wc;
      const int ys = UP ? (yy >> 1) : yy, xs = UP ? (xx >> 1) : xx;
      off[r * 3 + s] = ok[r * 3 + s] ? ys * ws + xs : 0;
    }
  const int plane = hs * ws;
  for (int ci = 0; ci < cin; ++ci) {
    const float* sp = src + ci * plane;
    const float* wp = wl + ci * 9 * NCO;
#pragma unroll
    for (int t = 0; t < 9; ++t) {
      const float v = ok[t] ? sp[off[t]] : 0.0f;
#pragma unroll
      for (int k = 0; k < NCO; ++k) acc[k] = fmaf(v, wp[t * NCO + k], acc[k]);
    }
  }
}

// The 2x2 block of output pixels (rows 2*by, 2*by + 1, columns 2*bx, 2*bx + 1) of a plain 3x3 convolution of
// src[cin][hs][ws] (hs, ws even): the block's 36 taps read the 4x4 source window around it, loaded once per input
// channel; a weight serves four pixels.  Each output adds its taps in the order (ci, r, s) as conv3_pixel does.
// wl: [ci*9 + tap][wstride], this thread's NCO channels first.  acc[2*a + b] is pixel (2*by + a, 2*bx + b).
template <int NCO>
__device__ __forceinline__ void conv3_block(const float* src, const float* wl, int wstride, int cin, int hs, int ws,
                                            int by, int bx, float (&acc)[4][NCO]) {
  int off[16];
  bool ok[16];
#pragma unroll
  for (int q = 0; q < 16; ++q) {
    const int yy = 2 * by + q / 4 - 1, xx = 2 * bx + q % 4 - 1;
    ok[q] = yy >= 0 && yy < hs && xx >= 0 && xx < ws;
    off[q] = ok[q] ? yy * ws + xx : 0;
  }
  const int plane = hs * ws;
  for (int ci = 0; ci < cin; ++ci) {
    const float* sp = src + ci * plane;
    const float* wp = wl + ci * 9 * wstride;
    float sv[16];
#pragma unroll
    for (int q = 0; q < 16; ++q) sv[q] = ok[q] ? sp[off[q]] : 0.0f;
#pragma unroll
    for (int t = 0; t < 9; ++t) {
      float w[NCO];
      if constexpr (NCO == 4) {
        const float4 w4 = *reinterpret_cast<const float4*>(wp + t * wstride);
        w[0] = w4.x; w[1] = w4.y; w[2] = w4.z; w[3] = w4.w;
      } else {
#pragma unroll
        for (int k = 0; k < NCO; ++k) w[k] = wp[t * wstride + k];
      }
#pragma unroll
      for (int ab = 0; ab < 4; ++ab) {
        const float v = sv[((ab >> 1) + t / 3) * 4 + (ab & 1) + t % 3];
#pragma unroll
        for (int k = 0; k < NCO; ++k) acc[ab][k] = fmaf(v, w[k], acc[ab][k]);
      }
    }
  }
}

// The 2x2 block of output pixels (rows 2*by, 2*by + 1, columns 2*bx, 2*bx + 1) of a 3x3 convolution behind a x2
// nearest upsample of src[cin][hs][ws]: the block's 36 taps read only the 3x3 source cells around (by, bx), which
// are loaded once per input channel, and a weight serves four pixels.  (One pixel per thread, conv3_pixel, is bound
// by the LDS reads: a value and NCO weights per NCO multiply-adds.)  Each output adds its taps in the order
// (ci, r, s): the sums are those of conv3_pixel<NCO, true> bit for bit.
// wl: [ci*9 + tap][wstride], this thread's NCO channels first.  acc[2*a + b] is pixel (2*by + a, 2*bx + b).
template <int NCO>
__device__ __forceinline__ void conv3_up_block(const float* src, const float* wl, int wstride, int cin, int hs, int ws,
                                               int by, int bx, float (&acc)[4][NCO]) {
  int off[9];
  bool ok[9];
#pragma unroll
  for (int q = 0; q < 9; ++q) {
    const int yy = by + q / 3 - 1, xx = bx + q % 3 - 1;
    ok[q] = yy >= 0 && yy < hs && xx >= 0 && xx < ws;
    off[q] = ok[q] ? yy * ws + xx : 0;
  }
  const int plane = hs * ws;
  for (int ci = 0; ci < cin; ++ci) {
    const float* sp = src + ci * plane;
    const float* wp = wl + ci * 9 * wstride;
    float sv[9];
#pragma unroll
    for (int q = 0; q < 9; ++q) sv[q] = ok[q] ? sp[off[q]] : 0.0f;
#pragma unroll
    for (int t = 0; t < 9; ++t) {
      float w[NCO];
      if constexpr (NCO == 4) {
        const float4 w4 = *reinterpret_cast<const float4*>(wp + t * wstride);
        w[0] = w4.x; w[1] = w4.y; w[2] = w4.z; w[3] = w4.w;
      } else {
#pragma unroll
        for (int k = 0; k < NCO; ++k) w[k] = wp[t * wstride + k];
      }
#pragma unroll
      for (int ab = 0; ab < 4; ++ab) {
        // output row 2*by + a under tap row r is upsampled row 2*by + a + r - 1, i.e. source row by + ((a + r - 1) >> 1)
        const int dy = ((ab >> 1) + t / 3 - 1) >> 1, dx = ((ab & 1) + t % 3 - 1) >> 1;
        const float v = sv[(dy + 1) * 3 + dx + 1];
#pragma unroll
        for (int k = 0; k < NCO; ++k) acc[ab][k] = fmaf(v, w[k], acc[ab][k]);
      }
    }
  }
}

// canonical conv weights W[co][ci][3][3] -> wl[(ci*9 + tap)*NCO + k] for co = co0 + k (zero beyond cout)
__device__ __forceinline__ void stage_weights(const float* __restrict__ w, int cout, int cin, int co0, int nco, float* wl) {
  for (int i = threadIdx.x; i < cin * 9 * nco; i += NT) {
    const int k = i % nco, t = i / nco;           // t = ci*9 + tap
    const int co = co0 + k;
    wl[i] = co < cout ? w[(int64_t)co * cin * 9 + t] : 0.0f;
  }
}


struct SmallArgs {
  const float* x; const float* params; float* y;
  float* raw1; float* raw2; float* part1; float* part2;
  int B, c0, h, w, c1, c2, n, cr, c3, c4;       // cr: channels after the reshape (input of the first decoder conv)
  int64_t w1, b1, bn1, w2, b2, bn2, wf1, bf1, wf2, bf2, w3, b3, w4, b4;   // offsets into params
  float sigma; uint64_t seed, first_sample;
};

// ---- launch 1: conv 1 (planar input, c0 <= 4 channels) ------------------------------------------------------------
__global__ __launch_bounds__(NT_MAX) void k_small_conv1(SmallArgs a) {
  extern __shared__ float lds[];
  float* img = lds;                               // [c0][h*w]
  float* wl = img + a.c0 * a.h * a.w;             // [c0*9][COB]
  float* red = wl + a.c0 * 9 * COB;               // [NT][2*COB + 1]: per-thread statistics (odd stride: no bank conflicts)
  const int b = blockIdx.x, hw = a.h * a.w;
  const float* xb = a.x + (int64_t)b * a.c0 * hw;
  for (int i = threadIdx.x; i < a.c0 * hw; i += NT) img[i] = xb[i];
  const float* bias = a.params + a.b1;
  for (int co0 = 0; co0 < a.c1; co0 += COB) {
    __syncthreads();
    stage_weights(a.params + a.w1, a.c1, a.c0, co0, COB, wl);
    __syncthreads();
    float s1[COB], s2[COB];
#pragma unroll
    for (int k = 0; k < COB; ++k) { s1[k] = 0.0f; s2[k] = 0.0f; }
    for (int p = threadIdx.x; p < hw; p += NT) {
      float acc[COB];
#pragma unroll
      for (int k = 0; k < COB; ++k) acc[k] = bias[co0 + k];
      conv3_pixel<COB, false>(img, wl, a.c0, a.h, a.w, p / a.w, p % a.w, acc);
      float* dst = a.raw1 + ((int64_t)b * hw + p) * a.c1 + co0;    // (c1 and co0 are multiples of COB: 16-byte pieces)
#pragma unroll
      for (int k = 0; k < COB; k += 4) *reinterpret_cast<float4*>(dst + k) = make_float4(acc[k], acc[k + 1], acc[k + 2], acc[k + 3]);
#pragma unroll
      for (int k = 0; k < COB; ++k) {
        const float d = acc[k] - bias[co0 + k];
        s1[k] += d;
        s2[k] = fmaf(d, d, s2[k]);
      }
    }
    // channel sums over the threads in a fixed order, through LDS: groups of 32 threads, then the groups
    constexpr int SR = 2 * COB + 1;
    __syncthreads();
#pragma unroll
    for (int k = 0; k < COB; ++k) { red[threadIdx.x * SR + k] = s1[k]; red[threadIdx.x * SR + COB + k] = s2[k]; }
    __syncthreads();
    {
      const int c = threadIdx.x % (2 * COB), g = threadIdx.x / (2 * COB);      // NT / 32 groups of 32 threads
      float t = 0.0f;
      for (int th = g * 32; th < g * 32 + 32; ++th) t += red[th * SR + c];
      __syncthreads();
      red[g * SR + c] = t;
      __syncthreads();
      if (g == 0) {
        float u = 0.0f;
        for (int gg = 0; gg < NT / 32; ++gg) u += red[gg * SR + c];
        const int q = c / COB, k = c % COB;
        if (co0 + k < a.c1) a.part1[((int64_t)b * 2 + q) * a.c1 + co0 + k] = u;
      }
    }
  }
}

// batch-norm + ReLU + 2x2 max-pool of a [pixels][C] conv output of one sample into a planar LDS image dst[C][hp*wp]
__device__ __forceinline__ void bn_relu_pool_to_lds(const float* __restrict__ raw, int hc, int wc, int C, const float* scale,
                                                    const float* shift, float* dst) {
  const int hp = hc / 2, wp = wc / 2;
  for (int i = threadIdx.x; i < hp * wp * C; i += NT) {
    const int c = i % C, q = i / C;
    const int yy = q / wp, xx = q % wp;
    const float sc = scale[c], sh = shift[c];
    const float* r0 = raw + ((int64_t)(2 * yy) * wc + 2 * xx) * C + c;
    const float v0 = fmaf(r0[0], sc, sh), v1 = fmaf(r0[C], sc, sh);
    const float v2 = fmaf(r0[(int64_t)wc * C], sc, sh), v3 = fmaf(r0[(int64_t)wc * C + C], sc, sh);
    dst[c * (hp * wp) + q] = fmaxf(fmaxf(fmaxf(v0, v1), fmaxf(v2, v3)), 0.0f);
  }
}

// ---- launch 2: layer-1 statistics, bn + relu + pool, conv 2 (one workgroup per sample and block of COB channels) ----
__global__ __launch_bounds__(NT_CONV2) void k_small_conv2(SmallArgs a) {
  extern __shared__ float lds[];
  const int h2 = a.h / 2, w2 = a.w / 2, hw2 = h2 * w2;
  double* tmp = reinterpret_cast<double*>(lds);   // [2*256] scratch of the statistics
  float* a1 = lds + 1024;                         // [c1][hw2]
  float* wl = a1 + a.c1 * hw2;                    // [c1*9][COB]
  float* scale = wl + a.c1 * 9 * COB;             // [c1]
  float* shift = scale + a.c1;                    // [c1]
  float* red = shift + a.c1;
  const int b = blockIdx.x, co0 = blockIdx.y * COB;
  bn_vectors(a.part1, a.B, a.c1, 1.0 / ((double)a.B * a.h * a.w), a.params + a.b1, a.params + a.bn1, scale, shift, tmp);
  stage_weights(a.params + a.w2, a.c2, a.c1, co0, COB, wl);
  __syncthreads();
  bn_relu_pool_to_lds(a.raw1 + (int64_t)b * a.h * a.w * a.c1, a.h, a.w, a.c1, scale, shift, a1);
  __syncthreads();
  const float* bias = a.params + a.b2;
  // a thread owns a 2x2 block of output pixels and four of the workgroup's COB channels; the threads of a wavefront
  // share the channels (their weight reads are broadcasts)
  const int h4 = h2 / 2, w4 = w2 / 2, nblk = h4 * w4;
  float* part = red + NT / 64 * 2 * COB;          // [item][sum | sum sq][4]: statistics of each item's 16 outputs
  for (int item = threadIdx.x; item < nblk * (COB / 4); item += NT) {
    const int blk = item % nblk, g4 = item / nblk;
    const int by = blk / w4, bx = blk % w4;
    float acc[4][4], bk[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      bk[k] = bias[co0 + 4 * g4 + k];
#pragma unroll
      for (int ab = 0; ab < 4; ++ab) acc[ab][k] = bk[k];
    }
    conv3_block<4>(a1, wl + 4 * g4, COB, a.c1, h2, w2, by, bx, acc);
    float s1[4] = {0.f, 0.f, 0.f, 0.f}, s2[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ab = 0; ab < 4; ++ab) {
      const int pix = (2 * by + (ab >> 1)) * w2 + 2 * bx + (ab & 1);
      *reinterpret_cast<float4*>(a.raw2 + ((int64_t)b * hw2 + pix) * a.c2 + co0 + 4 * g4) =
          make_float4(acc[ab][0], acc[ab][1], acc[ab][2], acc[ab][3]);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const float d = acc[ab][k] - bk[k];
        s1[k] += d;
        s2[k] = fmaf(d, d, s2[k]);
      }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) { part[item * 8 + k] = s1[k]; part[item * 8 + 4 + k] = s2[k]; }
  }
  __syncthreads();
  // channel sums over the blocks in index order
  if ((int)threadIdx.x < 2 * COB) {
    const int q = threadIdx.x / COB, kk = threadIdx.x % COB;
    float t = 0.0f;
    for (int blk = 0; blk < nblk; ++blk) t += part[(blk + nblk * (kk >> 2)) * 8 + q * 4 + (kk & 3)];
    if (co0 + kk < a.c2) a.part2[((int64_t)b * 2 + q) * a.c2 + co0 + kk] = t;
  }
}

// ---- launch 3: everything from the second batch-norm to y ----------------------------------------------------------
__global__ __launch_bounds__(NT_MAX) void k_small_tail(SmallArgs a) {
  extern __shared__ float lds[];
  const int h2 = a.h / 2, w2 = a.w / 2, h4 = a.h / 4, w4 = a.w / 4, hw4 = h4 * w4, hw2 = h2 * w2, hw = a.h * a.w;
  const int F = a.c2 * hw4, FD = a.cr * hw4;      // flattened encoder output; decoder fc output
  double* tmp = reinterpret_cast<double*>(lds);   // [2*256] scratch of the statistics
  float* a2 = lds + 1024;                         // [c2][hw4]   (flatten order)
  float* dec = a2 + F;                            // [cr][hw4]   (reshape order)
  float* a3 = dec + FD;                           // [c3][hw2]
  float* lat = a3 + a.c3 * hw2;                   // [n] z, then the channel output
  float* scale = lat + a.n;                       // [c2]
  float* shift = scale + a.c2;
  float* red = shift + a.c2;                      // [NT/64 + 1]
  float* wl = reinterpret_cast<float*>((reinterpret_cast<uintptr_t>(red + NT / 64 + 4) + 15) & ~(uintptr_t)15);   // weights of the decoder convs (16-byte aligned: read four at a time)
  const int b = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  bn_vectors(a.part2, a.B, a.c2, 1.0 / ((double)a.B * hw2), a.params + a.b2, a.params + a.bn2, scale, shift, tmp);
  __syncthreads();
  bn_relu_pool_to_lds(a.raw2 + (int64_t)b * hw2 * a.c2, h2, w2, a.c2, scale, shift, a2);
  __syncthreads();
  // fc to the latent: one wavefront per output row, lanes stride over the inputs
  {
    const float* wf = a.params + a.wf1;
    constexpr int RB = 4;                         // rows per wavefront at a time: 4 * RB loads in flight per lane
    const bool vec = (F & 3) == 0 && (((uintptr_t)wf | (uintptr_t)a2) & 15) == 0;   // rows in 16-byte pieces: four times the bytes in flight
    for (int o0 = wave * RB; o0 < a.n; o0 += NT / 64 * RB) {
      float acc[RB];
#pragma unroll
      for (int r = 0; r < RB; ++r) acc[r] = 0.0f;
      for (int i0 = 4 * lane; vec && i0 < F; i0 += 256 * 4) {
        float4 wv[RB][4], av[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int i = i0 + 256 * u;
          av[u] = i < F ? *reinterpret_cast<const float4*>(&a2[i]) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
          for (int r = 0; r < RB; ++r)
            wv[r][u] = (i < F && o0 + r < a.n) ? *reinterpret_cast<const float4*>(&wf[(int64_t)(o0 + r) * F + i]) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
          for (int r = 0; r < RB; ++r)
            acc[r] = fmaf(wv[r][u].w, av[u].w, fmaf(wv[r][u].z, av[u].z, fmaf(wv[r][u].y, av[u].y, fmaf(wv[r][u].x, av[u].x, acc[r]))));
      }
      for (int i0 = lane; !vec && i0 < F; i0 += 64 * 4) {
        float wv[RB][4], av[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int i = i0 + 64 * u;
          av[u] = i < F ? a2[i] : 0.0f;
#pragma unroll
          for (int r = 0; r < RB; ++r) wv[r][u] = (i < F && o0 + r < a.n) ? wf[(int64_t)(o0 + r) * F + i] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
          for (int r = 0; r < RB; ++r) acc[r] = fmaf(wv[r][u], av[u], acc[r]);
      }
#pragma unroll
      for (int r = 0; r < RB; ++r) {
        const float t = wave_sum(acc[r]);
        if (lane == 0 && o0 + r < a.n) lat[o0 + r] = t + a.params[a.bf1 + o0 + r];
      }
    }
  }
  __syncthreads();
  // power normalisation and noise (same operation order as the stand-alone channel kernel)
  {
    float ss = 0.0f;
    for (int i = threadIdx.x; i < a.n; i += NT) ss = fmaf(lat[i], lat[i], ss);
    const float tot = block_sum_to0(ss, red);
    if (threadIdx.x == 0) {
      const float ms = tot / (float)a.n;
      red[NT / 64] = ms > 0.0f ? 1.0f / sqrtf(ms) : 0.0f;
    }
    __syncthreads();
    const float sc = red[NT / 64];
    for (int q = threadIdx.x; q < (a.n + 3) / 4; q += NT) {
      float g[4];
      normal_quad(a.seed, a.first_sample + (uint64_t)b, (uint32_t)q, g);
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (4 * q + j < a.n) lat[4 * q + j] = __fadd_rn(__fmul_rn(lat[4 * q + j], sc), __fmul_rn(a.sigma, g[j]));
    }
  }
  __syncthreads();
  // decoder fc: one thread per output, the latent from LDS; a row is read in 16-byte pieces where the blob allows
  {
    const float* wf = a.params + a.wf2;
    const bool vec = (a.n & 3) == 0 && (((uintptr_t)wf | (uintptr_t)lat) & 15) == 0;
    for (int o = threadIdx.x; o < FD; o += NT) {
      const float* row = wf + (int64_t)o * a.n;
      float acc = a.params[a.bf2 + o];
      if (vec) {
#pragma unroll 8
        for (int j = 0; j < a.n; j += 4) {
          const float4 w4 = *reinterpret_cast<const float4*>(row + j);
          const float4 l4 = *reinterpret_cast<const float4*>(lat + j);
          acc = fmaf(w4.w, l4.w, fmaf(w4.z, l4.z, fmaf(w4.y, l4.y, fmaf(w4.x, l4.x, acc))));
        }
      } else {
#pragma unroll 16
        for (int j = 0; j < a.n; ++j) acc = fmaf(row[j], lat[j], acc);
      }
      dec[o] = acc;
    }
  }
  // first decoder conv: x2 upsample of dec [cr][h4 x w4], 3x3 to c3 channels at h2 x w2, ReLU, planar into a3.
  // A thread owns a 2x2 block of output pixels and four channels; the threads of a wavefront share the channels
  // (their weight reads are broadcasts).
  for (int co0 = 0; co0 < a.c3; co0 += COB) {
    __syncthreads();
    stage_weights(a.params + a.w3, a.c3, a.cr, co0, COB, wl);
    __syncthreads();
    const int groups = (min(COB, a.c3 - co0) + 3) >> 2;
    for (int item = threadIdx.x; item < hw4 * groups; item += NT) {
      const int blk = item % hw4, g4 = item / hw4;
      const int by = blk / w4, bx = blk % w4;
      float acc[4][4];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const float bk = co0 + 4 * g4 + k < a.c3 ? a.params[a.b3 + co0 + 4 * g4 + k] : 0.0f;
#pragma unroll
        for (int ab = 0; ab < 4; ++ab) acc[ab][k] = bk;
      }
      conv3_up_block<4>(dec, wl + 4 * g4, COB, a.cr, h4, w4, by, bx, acc);
#pragma unroll
      for (int k = 0; k < 4; ++k)
        if (co0 + 4 * g4 + k < a.c3) {
#pragma unroll
          for (int ab = 0; ab < 4; ++ab)
            a3[(co0 + 4 * g4 + k) * hw2 + (2 * by + (ab >> 1)) * w2 + 2 * bx + (ab & 1)] = fmaxf(acc[ab][k], 0.0f);
        }
    }
  }
  // last conv: x2 upsample of a3, 3x3 to c4 <= 4 channels at h x w, sigmoid, planar output; 2x2 blocks again
  __syncthreads();
  float* yb = a.y + (int64_t)b * a.c4 * hw;
  if (a.c4 == 1) {                                 // a single output channel: one accumulator per pixel, not four
    stage_weights(a.params + a.w4, 1, a.c3, 0, 1, wl);
    __syncthreads();
    for (int blk = threadIdx.x; blk < hw2; blk += NT) {
      const int by = blk / w2, bx = blk % w2;
      float acc[4][1];
#pragma unroll
      for (int ab = 0; ab < 4; ++ab) acc[ab][0] = a.params[a.b4];
      conv3_up_block<1>(a3, wl, 1, a.c3, h2, w2, by, bx, acc);
#pragma unroll
      for (int ab = 0; ab < 4; ++ab) yb[(2 * by + (ab >> 1)) * a.w + 2 * bx + (ab & 1)] = apply_act(acc[ab][0], ACT_SIGMOID);
    }
    return;
  }
  stage_weights(a.params + a.w4, a.c4, a.c3, 0, 4, wl);
  __syncthreads();
  for (int blk = threadIdx.x; blk < hw2; blk += NT) {
    const int by = blk / w2, bx = blk % w2;
    float acc[4][4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
      for (int ab = 0; ab < 4; ++ab) acc[ab][k] = k < a.c4 ? a.params[a.b4 + k] : 0.0f;
    conv3_up_block<4>(a3, wl, 4, a.c3, h2, w2, by, bx, acc);
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (k < a.c4) {
#pragma unroll
        for (int ab = 0; ab < 4; ++ab)
          yb[(int64_t)k * hw + (2 * by + (ab >> 1)) * a.w + 2 * bx + (ab & 1)] = apply_act(acc[ab][k], ACT_SIGMOID);
      }
  }
}

size_t lds1(const SmallArgs& a) { return sizeof(float) * ((size_t)a.c0 * a.h * a.w + (size_t)a.c0 * 9 * COB + (size_t)NT_MAX * (2 * COB + 1)); }
size_t lds2(const SmallArgs& a) {
  return sizeof(float) * (1024 + (size_t)a.c1 * (a.h / 2) * (a.w / 2) + (size_t)a.c1 * 9 * COB + 2 * a.c1 + NT_CONV2 / 64 * 2 * COB +
                          (size_t)(a.h / 4) * (a.w / 4) * (COB / 4) * 8);
}
size_t lds3(const SmallArgs& a) {
  const size_t F = (size_t)(a.c2 + a.cr) * (a.h / 4) * (a.w / 4);
  const size_t wmax = (size_t)a.cr * 9 * COB > (size_t)a.c3 * 9 * 4 ? (size_t)a.cr * 9 * COB : (size_t)a.c3 * 9 * 4;
  return sizeof(float) * (1024 + F + (size_t)a.c3 * (a.h / 2) * (a.w / 2) + a.n + 2 * a.c2 + NT_MAX / 64 + 4 + 4 + wmax);
}

#undef NT
}  // namespace

// Does the plan have the shape and the sizes of the three-launch path?  (binary32, batch statistics, channel
// counts that are multiples of the accumulator block, every per-sample tensor inside 64 KiB of LDS.)
bool fused_small_match(const Plan& P, FusedSmall* f) {
  if (P.dtype != AE_F32 || P.bn_mode != 0) return false;
  const std::vector<Step>& S = P.steps;
  if (S.size() != 9) return false;
  const StepKind kinds[9] = {ST_CONV, ST_CONV, ST_TRANSPOSE, ST_CONV, ST_CHANNEL, ST_CONV, ST_TRANSPOSE, ST_CONV, ST_CONV};
  for (int i = 0; i < 9; ++i)
    if (S[i].kind != kinds[i]) return false;
  auto enc = [](const Step& s) { return s.k == 3 && !s.up && s.has_bn && s.act == ACT_RELU && s.pool; };
  auto fc = [](const Step& s) { return s.k == 1 && !s.up && !s.has_bn && s.act == ACT_NONE && !s.pool && s.hin == 1 && s.win == 1; };
  auto dec = [](const Step& s, int act) { return s.k == 3 && s.up && !s.has_bn && s.act == act && !s.pool; };
  // (nine steps: the planar boundary tensors are read / written by the first / last convolution itself, either
  // through the thin kernels or because a single channel has the same layout either way)
  if (!enc(S[0]) || (S[0].thin != 1 && P.c0 != 1) || !enc(S[1]) || !fc(S[3]) || !S[4].do_pnorm || !S[4].do_awgn || !fc(S[5]) ||
      !dec(S[7], ACT_RELU) || !dec(S[8], ACT_SIGMOID) || (S[8].thin != 2 && P.cl != 1))
    return false;
  SmallArgs a{};
  a.B = P.batch; a.c0 = P.c0; a.h = P.h0; a.w = P.w0;
  a.c1 = S[0].cout; a.c2 = S[1].cout; a.n = S[3].cout; a.cr = S[7].cin; a.c3 = S[7].cout; a.c4 = S[8].cout;
  if (a.h % 4 || a.w % 4 || a.h > 32 || a.w > 32 || a.c0 > 4 || a.c4 > 4) return false;
  if (a.c1 % COB || a.c2 % COB || a.c3 % COB || a.c1 > 64 || a.c2 > 128 || a.c3 > 64 || a.n > 1024) return false;
  // the flatten and the reshape keep the (c,h,w) order of the pooled maps
  if (S[3].cin != a.c2 * (a.h / 4) * (a.w / 4) || S[5].cin != a.n || S[7].hin != a.h / 4 || S[7].win != a.w / 4 ||
      a.cr * (a.h / 4) * (a.w / 4) != S[5].cout || S[8].cin != a.c3 || S[8].hin != a.h / 2)
    return false;
  if (lds1(a) > 65536 || lds2(a) > 65536 || lds3(a) > 65536) return false;
  if ((int64_t)P.batch * 2 * (a.c1 + a.c2) > P.max_partial_floats) return false;   // the per-sample statistics live in the partial-sum buffer
  if (f) {
    f->w1 = S[0].w_off; f->b1 = S[0].b_off; f->bn1 = S[0].bn_off; f->w2 = S[1].w_off; f->b2 = S[1].b_off; f->bn2 = S[1].bn_off;
    f->wf1 = S[3].w_off; f->bf1 = S[3].b_off; f->wf2 = S[5].w_off; f->bf2 = S[5].b_off;
    f->w3 = S[7].w_off; f->b3 = S[7].b_off; f->w4 = S[8].w_off; f->b4 = S[8].b_off;
    f->c1 = a.c1; f->c2 = a.c2; f->n = a.n; f->cr = a.cr; f->c3 = a.c3; f->c4 = a.c4;
  }
  return true;
}

int launch_fused_small(const Plan& P, const FusedSmall& f, const float* params, const float* x, float* y, float* raw1,
                       float* raw2, float* partial, float sigma, uint64_t seed, uint64_t first_sample, hipStream_t s) {
  SmallArgs a{};
  a.x = x; a.params = params; a.y = y; a.raw1 = raw1; a.raw2 = raw2;
  a.part1 = partial; a.part2 = partial + (int64_t)P.batch * 2 * f.c1;
  a.B = P.batch; a.c0 = P.c0; a.h = P.h0; a.w = P.w0;
  a.c1 = f.c1; a.c2 = f.c2; a.n = f.n; a.cr = f.cr; a.c3 = f.c3; a.c4 = f.c4;
  a.w1 = f.w1; a.b1 = f.b1; a.bn1 = f.bn1; a.w2 = f.w2; a.b2 = f.b2; a.bn2 = f.bn2;
  a.wf1 = f.wf1; a.bf1 = f.bf1; a.wf2 = f.wf2; a.bf2 = f.bf2; a.w3 = f.w3; a.b3 = f.b3; a.w4 = f.w4; a.b4 = f.b4;
  a.sigma = sigma; a.seed = seed; a.first_sample = first_sample;
  hipLaunchKernelGGL(k_small_conv1, dim3(P.batch), dim3(NT_MAX), lds1(a), s, a);
  hipLaunchKernelGGL(k_small_conv2, dim3(P.batch, f.c2 / COB), dim3(NT_CONV2), lds2(a), s, a);
  hipLaunchKernelGGL(k_small_tail, dim3(P.batch), dim3(NT_MAX), lds3(a), s, a);
  return launch_status("fused_small");
}

}  // namespace ae
