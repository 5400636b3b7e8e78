// ae_conv_direct.hip — general-shape convolution kernels on the vector ALUs.
// They serve every layer shape the MFMA implicit-GEMM kernels do not take
// (channel counts that are not a multiple of the MFMA K-slab, e.g. the 1- or
// 3-channel first layer and the 1- or 3-channel last layer) and are the only
// weight-gradient kernels for those shapes.
//
// Activations are [n][H][W][C]; packed weights are [C_out][k][k][C_in].
// If `up` is set the input tensor is stored at half resolution and read through a
// nearest-neighbour x2 upsample: source pixel = (h >> 1, w >> 1).
#include "ae_device.h"
#include "ae_internal.h"

namespace ae {
namespace {

constexpr int NT = 256;

// one thread per output element, output channel fastest
template <typename T>
__global__ void k_conv_direct(const T* __restrict__ x, const T* __restrict__ wp, const float* __restrict__ bias,
                              T* __restrict__ y, float* __restrict__ y_aux, int64_t total, int Hc, int Wc, int Cin,
                              int Cout, int k, int up, int act) {
  const int p = (k - 1) >> 1;
  const int Hin = Hc >> up, Win = Wc >> up;
  for (int64_t idx = (int64_t)blockIdx.x * NT + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * NT) {
    const int co = (int)(idx % Cout);
    int64_t pix = idx / Cout;
    const int w = (int)(pix % Wc); pix /= Wc;
    const int h = (int)(pix % Hc);
    const int64_t n = pix / Hc;
    float acc = bias ? bias[co] : 0.0f;
    for (int r = 0; r < k; ++r) {
      const int hh = h + r - p;
      if (hh < 0 || hh >= Hc) continue;
      for (int s = 0; s < k; ++s) {
        const int ww = w + s - p;
        if (ww < 0 || ww >= Wc) continue;
        const T* xs = x + ((n * Hin + (hh >> up)) * Win + (ww >> up)) * Cin;
        const T* ws = wp + ((int64_t)(co * k + r) * k + s) * Cin;
        for (int ci = 0; ci < Cin; ++ci) acc = fmaf(Store<T>::ld(xs + ci), Store<T>::ld(ws + ci), acc);
      }
    }
    // the conv result is a stored tensor of the format: round it before the activation
    const float a = apply_act(round_to_storage<T>(acc), act);
    Store<T>::st(y + idx, a);
    if (y_aux) y_aux[idx] = a;
  }
}

// Weight gradient.  grid.x covers the weights (ci fastest so that x reads coalesce), grid.y splits the
// pixels into chunks; chunk c leaves its sums in partial[c][widx] and k_wgrad_direct_reduce adds the
// chunks in index order into the canonical layout dW[co][ci][r][s] (fp32): no atomics, the same bits every run.
// With a single chunk the kernel writes dW itself (partial = null).
template <typename T>
__global__ void k_wgrad_direct(const T* __restrict__ x, const T* __restrict__ dy, float* __restrict__ dw,
                               float* __restrict__ partial, int64_t rows, int rows_per_block, int Hc, int Wc, int Cin,
                               int Cout, int k, int up) {
  const int p = (k - 1) >> 1;
  const int Hin = Hc >> up, Win = Wc >> up;
  const int64_t nweights = (int64_t)Cout * k * k * Cin;
  const int64_t widx = (int64_t)blockIdx.x * NT + threadIdx.x;
  if (widx >= nweights) return;
  const int ci = (int)(widx % Cin);
  int64_t t = widx / Cin;
  const int s = (int)(t % k); t /= k;
  const int r = (int)(t % k);
  const int co = (int)(t / k);
  const int64_t m0 = (int64_t)blockIdx.y * rows_per_block;
  const int64_t m1 = m0 + rows_per_block < rows ? m0 + rows_per_block : rows;
  float acc = 0.0f;
  for (int64_t m = m0; m < m1; ++m) {
    const int w = (int)(m % Wc);
    const int h = (int)((m / Wc) % Hc);
    const int64_t n = m / ((int64_t)Wc * Hc);
    const int hh = h + r - p, ww = w + s - p;
    if (hh < 0 || hh >= Hc || ww < 0 || ww >= Wc) continue;
    const float xv = Store<T>::ld(x + ((n * Hin + (hh >> up)) * Win + (ww >> up)) * Cin + ci);
    acc = fmaf(Store<T>::ld(dy + m * Cout + co), xv, acc);
  }
  if (partial) partial[(int64_t)blockIdx.y * nweights + widx] = acc;
  else dw[(((int64_t)co * Cin + ci) * k + r) * k + s] = acc;
}

__global__ void k_wgrad_direct_reduce(const float* __restrict__ partial, int chunks, int64_t nweights, int Cin, int k,
                                      float* __restrict__ dw) {
  const int64_t widx = (int64_t)blockIdx.x * NT + threadIdx.x;
  if (widx >= nweights) return;
  float acc = 0.0f;
  for (int c = 0; c < chunks; ++c) acc += partial[(int64_t)c * nweights + widx];
  const int ci = (int)(widx % Cin);
  int64_t t = widx / Cin;
  const int s = (int)(t % k); t /= k;
  const int r = (int)(t % k);
  const int64_t co = t / k;
  dw[((co * Cin + ci) * k + r) * k + s] = acc;
}

}  // namespace

int launch_conv_direct(const ConvArgs& a, hipStream_t s) {
  const int64_t total = (int64_t)a.n * a.hc * a.wc * a.cout;
  int64_t g = (total + NT - 1) / NT;
  if (g > (1 << 22)) g = 1 << 22;
  if (a.dtype == AE_BF16)
    hipLaunchKernelGGL((k_conv_direct<bf16_t>), dim3((unsigned)g), dim3(NT), 0, s, (const bf16_t*)a.x,
                       (const bf16_t*)a.w, a.bias, (bf16_t*)a.y, a.y_aux, total, a.hc, a.wc, a.cin, a.cout, a.k, a.up, a.act);
  else
    hipLaunchKernelGGL((k_conv_direct<float>), dim3((unsigned)g), dim3(NT), 0, s, (const float*)a.x, (const float*)a.w,
                       a.bias, (float*)a.y, a.y_aux, total, a.hc, a.wc, a.cin, a.cout, a.k, a.up, a.act);
  return launch_status("conv_direct");
}

// pixel chunks of the fallback weight gradient: enough to fill the machine, at least 512 rows each, at most 16
static int64_t wgrad_direct_chunks(const WgradArgs& a) {
  const int64_t rows = (int64_t)a.n * a.hc * a.wc;
  const int64_t nweights = (int64_t)a.cout * a.k * a.k * a.cin;
  const int64_t gx = (nweights + NT - 1) / NT;
  int64_t chunks = (4096 + gx - 1) / gx;
  const int64_t max_chunks = (rows + 511) / 512;
  if (chunks > max_chunks) chunks = max_chunks;
  if (chunks > 16) chunks = 16;
  return chunks < 1 ? 1 : chunks;
}

// scratch (floats) launch_wgrad_direct wants for its chunk sums; with less it uses fewer chunks
int64_t wgrad_direct_workspace_floats(const WgradArgs& a) {
  const int64_t chunks = wgrad_direct_chunks(a);
  return chunks > 1 ? chunks * a.cout * a.k * a.k * a.cin : 0;
}

int launch_wgrad_direct(const WgradArgs& a, float* workspace, int64_t workspace_floats, hipStream_t s) {
  const int64_t rows = (int64_t)a.n * a.hc * a.wc;
  const int64_t nweights = (int64_t)a.cout * a.k * a.k * a.cin;
  const int64_t gx = (nweights + NT - 1) / NT;
  int64_t chunks = wgrad_direct_chunks(a);
  if (!workspace) workspace_floats = 0;
  if (chunks * nweights > workspace_floats) chunks = workspace_floats / nweights;
  if (chunks < 1) chunks = 1;
  const int rpb = (int)((rows + chunks - 1) / chunks);
  chunks = (rows + rpb - 1) / rpb;
  float* partial = chunks > 1 ? workspace : nullptr;
  dim3 grid((unsigned)gx, (unsigned)chunks);
  if (a.dtype == AE_BF16)
    hipLaunchKernelGGL((k_wgrad_direct<bf16_t>), grid, dim3(NT), 0, s, (const bf16_t*)a.x, (const bf16_t*)a.dy,
                       a.dw_canonical, partial, rows, rpb, a.hc, a.wc, a.cin, a.cout, a.k, a.up);
  else
    hipLaunchKernelGGL((k_wgrad_direct<float>), grid, dim3(NT), 0, s, (const float*)a.x, (const float*)a.dy,
                       a.dw_canonical, partial, rows, rpb, a.hc, a.wc, a.cin, a.cout, a.k, a.up);
  AE_TRY(launch_status("wgrad_direct"));
  if (chunks > 1) {
    hipLaunchKernelGGL(k_wgrad_direct_reduce, dim3((unsigned)gx), dim3(NT), 0, s, partial, (int)chunks, nweights, a.cin, a.k,
                       a.dw_canonical);
    return launch_status("wgrad_direct_reduce");
  }
  return AE_OK;
}

}  // namespace ae
