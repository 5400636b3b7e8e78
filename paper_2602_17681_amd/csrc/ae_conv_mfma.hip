// ae_conv_mfma.hip — convolution / fully-connected layers as implicit GEMM on the
// CDNA4 matrix cores.
//
//   C[M][N] = A[M][K] * B[N][K]^T,  M = batch*H*W output pixels, N = C_out,
//   K = k*k*C_in ordered (r, s, ci).
// A is never materialised: row m is pixel (n,h,w) and the K-slab [kt*BK, kt*BK+BK)
// lies inside one filter tap (r,s) because C_in is a multiple of BK, so the slab is
// BK contiguous channels of input pixel (h+r-p, w+s-p) (zero outside the image; read
// through a x2 nearest upsample when `up`).  B is the packed weight [C_out][k][k][C_in].
//
// One workgroup of 256 threads (4 wavefronts, 2x2) computes a BM x BN tile with
// v_mfma_f32_32x32x16_bf16 (bf16) or v_mfma_f32_32x32x2_f32 (fp32); A and B slabs are
// staged through LDS, double buffered, one barrier per slab.  The epilogue adds the
// bias, rounds to the storage type, optionally reduces per-channel sum / sum of squares
// of the tile (batch-norm statistics), applies the activation and stores [M][N].
#include "ae_device.h"
#include "ae_internal.h"

namespace ae {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

struct IgemmParams {
  const void* x; const void* w; const float* bias; void* y; float* y_aux; float* partial;
  int64_t M;
  int N, K;             // C_out, k*k*C_in
  int Hc, Wc, Cin, ksz, up;
  int act;
  int tiles_n;
};

// ---------------------------------------------------------------------------
// bf16: BK = 32 elements (64 bytes per row per slab); LDS rows padded to 80 bytes so
// that the eight rows a ds_read_b128 serves per cycle fall into distinct banks.
// ---------------------------------------------------------------------------
template <int BM, int BN>
__global__ __launch_bounds__(256) void k_igemm_bf16(IgemmParams p) {
  constexpr int BK = 32;
  constexpr int LDS = 40;                       // row stride in elements (80 bytes)
  constexpr int WM = BM / 2, WN = BN / 2;       // wave tile
  constexpr int MI = WM / 32, NJ = WN / 32;     // 32x32 MFMA tiles per wave
  constexpr int A_CHUNKS = BM * 4 / 256;        // 16-byte chunks per thread per slab
  constexpr int B_CHUNKS = BN * 4 / 256;
  __shared__ __attribute__((aligned(16))) bf16_t sA[2][BM * LDS];
  __shared__ __attribute__((aligned(16))) bf16_t sB[2][BN * LDS];
  __shared__ float sRed[2][2][BN];              // [wave row][sum | sumsq][column]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int tile_n = blockIdx.x % p.tiles_n;
  const int64_t tile_m = blockIdx.x / p.tiles_n;
  const int64_t m0 = tile_m * BM;
  const int n0 = tile_n * BN;
  const bf16_t* __restrict__ X = (const bf16_t*)p.x;
  const bf16_t* __restrict__ W = (const bf16_t*)p.w;
  const int pad = (p.ksz - 1) >> 1;
  const int Hin = p.Hc >> p.up, Win = p.Wc >> p.up;

  // --- loader bookkeeping: this thread's rows of the A and B slabs
  const int chunk = tid & 3;                    // which 16 bytes of the 64-byte row
  int a_h[A_CHUNKS], a_w[A_CHUNKS];
  int64_t a_img[A_CHUNKS];                      // element offset of the sample's image, -1 if the row is past M
#pragma unroll
  for (int i = 0; i < A_CHUNKS; ++i) {
    const int row = (tid >> 2) + i * 64;
    const int64_t m = m0 + row;
    if (m < p.M) {
      const int w = (int)(m % p.Wc);
      const int64_t t = m / p.Wc;
      a_h[i] = (int)(t % p.Hc);
      a_w[i] = w;
      a_img[i] = (t / p.Hc) * (int64_t)Hin * Win * p.Cin;
    } else {
      a_h[i] = 0; a_w[i] = 0; a_img[i] = -1;
    }
  }
  const bf16_t* b_ptr[B_CHUNKS];
#pragma unroll
  for (int i = 0; i < B_CHUNKS; ++i) {
    const int row = (tid >> 2) + i * 64;
    b_ptr[i] = (n0 + row < p.N) ? W + (int64_t)(n0 + row) * p.K + chunk * 8 : nullptr;
  }

  uint4 ra[A_CHUNKS], rb[B_CHUNKS];
  const uint4 zero4 = make_uint4(0u, 0u, 0u, 0u);
  int rs = 0, ci0 = 0;                          // filter tap and first channel of the slab being loaded
  auto load_slab = [&](int kt) {
    const int r = rs / p.ksz, s = rs - r * p.ksz;
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i) {
      const int hh = a_h[i] + r - pad, ww = a_w[i] + s - pad;
      const bool ok = a_img[i] >= 0 && hh >= 0 && hh < p.Hc && ww >= 0 && ww < p.Wc;
      ra[i] = ok ? *reinterpret_cast<const uint4*>(X + a_img[i] + ((int64_t)(hh >> p.up) * Win + (ww >> p.up)) * p.Cin +
                                                   ci0 + chunk * 8)
                 : zero4;
    }
#pragma unroll
    for (int i = 0; i < B_CHUNKS; ++i)
      rb[i] = b_ptr[i] ? *reinterpret_cast<const uint4*>(b_ptr[i] + (int64_t)kt * BK) : zero4;
    ci0 += BK;
    if (ci0 == p.Cin) { ci0 = 0; ++rs; }
  };
  auto store_slab = [&](int buf) {
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i)
      *reinterpret_cast<uint4*>(&sA[buf][((tid >> 2) + i * 64) * LDS + chunk * 8]) = ra[i];
#pragma unroll
    for (int i = 0; i < B_CHUNKS; ++i)
      *reinterpret_cast<uint4*>(&sB[buf][((tid >> 2) + i * 64) * LDS + chunk * 8]) = rb[i];
  };

  floatx16 acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  const int KT = p.K / BK;
  load_slab(0);
  store_slab(0);
  __syncthreads();
  const int frag_row = lane & 31, frag_k = (lane >> 5) * 8;
  for (int kt = 0; kt < KT; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < KT) load_slab(kt + 1);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 a[MI], b[NJ];
#pragma unroll
      for (int i = 0; i < MI; ++i)
        a[i] = *reinterpret_cast<const bf16x8*>(&sA[buf][(wm * WM + i * 32 + frag_row) * LDS + ks * 16 + frag_k]);
#pragma unroll
      for (int j = 0; j < NJ; ++j)
        b[j] = *reinterpret_cast<const bf16x8*>(&sB[buf][(wn * WN + j * 32 + frag_row) * LDS + ks * 16 + frag_k]);
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < KT) store_slab(buf ^ 1);
    __syncthreads();
  }

  // --- epilogue.  Accumulator element e of lane l in tile (i,j):
  //     row = wm*WM + i*32 + (e/4)*8 + (l/32)*4 + e%4,  column = wn*WN + j*32 + l%32
  bf16_t* __restrict__ Y = (bf16_t*)p.y;
  const int col_lane = lane & 31, row_lane = (lane >> 5) * 4;
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int col = n0 + wn * WN + j * 32 + col_lane;
    const bool col_ok = col < p.N;
    const float bias = (p.bias && col_ok) ? p.bias[col] : 0.0f;
    float s1 = 0.0f, s2 = 0.0f;
#pragma unroll
    for (int i = 0; i < MI; ++i) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int64_t m = m0 + wm * WM + i * 32 + (e >> 2) * 8 + row_lane + (e & 3);
        if (m < p.M && col_ok) {
          const float v = bf16_to_f32(f32_to_bf16(acc[i][j][e] + bias));   // the stored conv result
          s1 += v;
          s2 = fmaf(v, v, s2);
          const float a = apply_act(v, p.act);
          Y[m * p.N + col] = f32_to_bf16(a);
          if (p.y_aux) p.y_aux[m * p.N + col] = a;
        }
      }
    }
    if (p.partial) {
      s1 += __shfl_xor(s1, 32, 64);
      s2 += __shfl_xor(s2, 32, 64);
      if (lane < 32) {
        sRed[wm][0][wn * WN + j * 32 + col_lane] = s1;
        sRed[wm][1][wn * WN + j * 32 + col_lane] = s2;
      }
    }
  }
  if (p.partial) {
    __syncthreads();
    for (int i = tid; i < 2 * BN; i += 256) {
      const int q = i / BN, c = i - q * BN;
      if (n0 + c < p.N) p.partial[(tile_m * 2 + q) * p.N + n0 + c] = sRed[0][q][c] + sRed[1][q][c];
    }
  }
}

int tile_n_for(int cout) { return cout > 64 ? 128 : 64; }

}  // namespace

bool conv_mfma_supported(const ConvArgs& a) {
  if (a.dtype != AE_BF16) return false;
  if (a.cin % 32 != 0 || a.cout < 32) return false;
  const int64_t M = (int64_t)a.n * a.hc * a.wc;
  const int64_t tiles = ((M + 127) / 128) * ((a.cout + tile_n_for(a.cout) - 1) / tile_n_for(a.cout));
  return tiles < 0x7FFFFFFF;
}

int conv_partial_rows(const ConvArgs&, bool mfma) { return mfma ? 128 : kReduceRows; }

int launch_conv_mfma(const ConvArgs& a, hipStream_t s) {
  if (!conv_mfma_supported(a)) return fail(AE_EINVAL, "conv_mfma: shape not supported");
  IgemmParams p;
  p.x = a.x; p.w = a.w; p.bias = a.bias; p.y = a.y; p.y_aux = a.y_aux; p.partial = a.partial;
  p.M = (int64_t)a.n * a.hc * a.wc;
  p.N = a.cout; p.K = a.k * a.k * a.cin;
  p.Hc = a.hc; p.Wc = a.wc; p.Cin = a.cin; p.ksz = a.k; p.up = a.up; p.act = a.act;
  const int bn = tile_n_for(a.cout);
  p.tiles_n = (a.cout + bn - 1) / bn;
  const int64_t tiles_m = (p.M + 127) / 128;
  dim3 grid((unsigned)(tiles_m * p.tiles_n));
  if (bn == 128) hipLaunchKernelGGL((k_igemm_bf16<128, 128>), grid, dim3(256), 0, s, p);
  else hipLaunchKernelGGL((k_igemm_bf16<128, 64>), grid, dim3(256), 0, s, p);
  return launch_status("conv_mfma");
}

}  // namespace ae
