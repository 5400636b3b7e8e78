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
// One workgroup of 256 threads (4 wavefronts) computes a BM x BN tile with
// v_mfma_f32_32x32x16_bf16 (bf16) or v_mfma_f32_32x32x2_f32 (fp32).  Kernels in this file:
//   k_conv3_patch  3x3 convolutions of 16/32/64-wide images (wider ones by column strips): the input patch
//                  of a tile lives in LDS and all nine taps are read from it (one global read per input
//                  element); the weights, packed in MFMA fragment order, go straight into registers
//   k_igemm        every other shape: per-tap slabs through a three-stage global-to-LDS ring,
//                  optionally split over K; also the two cheaper forms of a 3x3 convolution behind
//                  a x2 upsample (four 2x2 phase convolutions forward, one 4x4 stride-2
//                  convolution for the input gradient; see IgemmParams)
//   k_wgrad_row3   weight gradient, three taps per workgroup from one input patch (bf16)
//   k_wgrad_rows, k_wgrad   weight gradient, one tap per workgroup (fp32, 1x1, odd shapes)
// The shared epilogue adds the bias, rounds to the storage type, optionally reduces per-channel
// sum / sum of squares of the tile (batch-norm statistics), applies the activation and stores [M][N].
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
  unsigned x_bytes, w_bytes;   // sizes of the two operand tensors (buffer range checks)
  // split-K (layers with too few output tiles to fill the chip): workgroup (split, tile) works on
  // K slabs [split*slabs_per_split, ...) and writes its fp32 tile to split_out[split][M][N];
  // k_splitk_finish sums the splits and applies bias / rounding / activation
  int tiles_mn, slabs_per_split;
  float* split_out;
  // Source geometry.  GEMM row m is pixel (n, i, j) of an Hc x Wc grid; tap (r, s) of that row
  // reads source position (i*stride + r - pad_h, j*stride + s - pad_w) of an Hv x Wv image
  // (stored at (Hv>>up) x (Wv>>up): nearest-neighbour upsampling folded into the read), zero
  // outside.  Plain convolution: Hv = Hc, Wv = Wc, stride 1, pad = (ksz-1)/2.
  int Hv, Wv, stride, pad;
  // phases = 4: the convolution behind a x2 upsample, written as four 2x2 convolutions of the
  // stored input (one per output parity (a, b) = (phase>>1, phase&1), pads 1-a and 1-b, weights
  // w + phase*N*K); row (n, i, j) of phase (a, b) is output pixel (2i+a, 2j+b) of a 2Hc x 2Wc image
  int phases;
  // epilogue variants of the dense-GEMM use (EPI template parameter of k_igemm):
  //   1: the stored output is MX block-quantised (blocks of mx_block output columns: a power of two from one 16-byte
  //      chunk up to the 64 columns of a wave tile; FP4 E2M1 elements);
  //   2: nothing is stored; the epilogue forms resid[m][n] - (acc + bias) and leaves per-tile column sums of it
  //      and of its square in `partial` (resid: [M][N] in the storage type)
  const void* resid;
  int mx_block, mx_elem;       // block size and element format (MX_FP4 / MX_INT4 / MX_FP8) of epilogue 1
  // Square dense products (M = N = K) with triangular operands: K range per tile, and tiles nobody wants skipped.
  //   1: x[m][k] = 0 for k > m and w[n][k] = 0 for k > n (lower times upper): K ends at min(last row, last column) + 1
  //   2: x[m][k] = 0 for k < m, wanted outputs n >= m: K starts at the tile's first row; tiles below the diagonal return
  //   3: w[n][k] = 0 for k < n, wanted outputs n < m: K starts at the tile's first column; tiles above the diagonal return
  //   4: x[m][k] = 0 for k < m and w[n][k] = 0 for k < n (upper times lower): K starts at max(first row, first column)
  // Blocked triangular inverse, all pairs of neighbouring tri_b x tri_b diagonal blocks in one launch (tile sizes divide
  // tri_b): only the tiles of one off-diagonal block per pair are computed, over the K range of one block:
  //   8: tile rows in an even block r, columns in block r+1, K = block r;
  //   9: tile rows in an odd block r, columns in block r-1, K = block r
  // tri_d > 0 (modes 8, 9): the matrices are an identity block beyond row and column tri_d; tiles of the odd block that
  // lie wholly beyond it return (their outputs are zero and stay unwritten) and K ranges over the odd block end at tri_d.
  int tri, tri_b, tri_d;
  // k_conv3_patch on images wider than its tile: a tile is TH rows x Wt columns of one of `strips` column strips
  // of the image (Wt = Wc / strips, TH = 256 / Wt); GEMM row m = tile * 256 + th * Wt + tw then is pixel
  // (row block * TH + th, strip * Wt + tw) of its image.  1: a tile spans the image width and rows are pixels in order.
  int strips = 1;
  int log_wt = 6;              // log2 of the strip width Wc / strips
  int log_w = -1, log_h = -1;  // log2 of Wc and Hc when both are powers of two (the four-phase output mapping), else -1
  // Companion tensor of the output's shape and layout (interior tiles only): the saved activation a of the layer whose
  // output gradient this launch computes.  With dyv = (a > 0 ? value : 0) per stored value:
  //   1: dyv is stored instead of the value (ReLU backward); partial receives per-tile column sums of dyv (the bias gradient);
  //   2: the value is stored unchanged; partial receives per-tile column sums of dyv and of dyv * xhat, with
  //      xhat = a * invstd/scale - (shift/scale + mean) * invstd from comp_bn = [scale | shift | mean | invstd] (the sums
  //      of a batch-norm backward behind ReLU and max-pooling; columns with scale = 0 get a zero second sum).
  const void* comp = nullptr;
  int comp_mode = 0;
  const float* comp_bn = nullptr;
};

// output row (pixel index in y) of GEMM row m.  Column strips: the part that depends on the 256-row tile alone
// (image, row block, strip) is igemm_strip_base, taken once per tile by the caller; the strip width is a power of two.
__device__ __forceinline__ int64_t igemm_strip_base(const IgemmParams& p, int64_t m_tile) {
  const unsigned tile = (unsigned)(m_tile >> 8), wt = 1u << p.log_wt, th_n = 256u >> p.log_wt;
  const unsigned strip = tile % (unsigned)p.strips, t2 = tile / (unsigned)p.strips;
  const unsigned blocks = (unsigned)p.Hc / th_n;
  const unsigned rb = t2 % blocks, img = t2 / blocks;
  return ((int64_t)img * p.Hc + rb * th_n) * p.Wc + strip * wt;
}
__device__ __forceinline__ int64_t igemm_out_row(const IgemmParams& p, int64_t m, int phase, int64_t strip_base) {
  if (p.strips > 1) {
    const unsigned ml = (unsigned)m & 255u;
    return strip_base + (int64_t)((ml >> p.log_wt) * (unsigned)p.Wc + (ml & ((1u << p.log_wt) - 1u)));
  }
  if (p.phases == 1) return m;
  const unsigned mu = (unsigned)m;
  unsigned j, i, n;
  if (p.log_w >= 0) {        // power-of-two images: no divisions
    j = mu & ((unsigned)p.Wc - 1u);
    const unsigned t = mu >> p.log_w;
    i = t & ((unsigned)p.Hc - 1u); n = t >> p.log_h;
  } else {
    j = mu % (unsigned)p.Wc;
    const unsigned t = mu / (unsigned)p.Wc;
    i = t % (unsigned)p.Hc; n = t / (unsigned)p.Hc;
  }
  return ((int64_t)n * (2 * p.Hc) + 2 * i + (phase >> 1)) * (2 * p.Wc) + 2 * j + (phase & 1);
}

// ---------------------------------------------------------------------------
// The kernel, for T = bf16 (v_mfma_f32_32x32x16_bf16) or T = float (v_mfma_f32_32x32x2_f32).
// A slab row is BKB = 64 or 128 bytes of K = CPR 16-byte chunks.  LDS rows are not
// padded; chunk c of row r is stored in slot c ^ f(r) with f(r) = (r>>2)&3 (64-byte rows)
// or (r>>1)&7 (128-byte rows): the LDS has 64 banks and serves 16 lanes of a 16-byte
// access per pass, and with this swizzle the 16 rows of a pass fall into 16 different
// 16-byte columns for the loader's stores and for the MFMA fragment reads alike.
// A fragment read fetches 16 bytes per lane: lanes 0-31 chunk 2*ks, lanes 32-63 chunk
// 2*ks+1 of their row.  For bf16 that is exactly the operand of one K=16 MFMA; for fp32
// the four floats feed four K=2 MFMAs (component j of the low lanes is paired with
// component j of the high lanes — any pairing works as long as A and B use the same).
// Global loads are buffer loads: the hardware range check returns zero for the offsets
// that the loader marks invalid (zero padding of the image, rows past M or N), so no
// select or clamp is needed, and addresses are 32-bit byte offsets that only change when
// the filter tap changes.
// ---------------------------------------------------------------------------
typedef unsigned uint4v __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));
constexpr unsigned kOob = 0x80000000u;         // beyond any tensor (tensors are < 2 GiB): reads as zero

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

// Workgroups are handed to the 8 accelerator dies (XCDs, each with its own L2) round-robin by
// workgroup id.  This maps the hardware id to a logical one such that each XCD works on one
// contiguous range of logical ids, so that workgroups which share operand rows (neighbouring
// tiles, the taps of one tile) hit in the same L2.
__device__ __forceinline__ int xcd_logical_block(int b, int nb) {
  const int per = nb >> 3;                       // full rounds of 8
  return b < (per << 3) ? (b & 7) * per + (b >> 3) : b;
}

template <typename T> __device__ __forceinline__ void mma_step(const uint4v& a, const uint4v& b, floatx16& c);
template <> __device__ __forceinline__ void mma_step<bf16_t>(const uint4v& a, const uint4v& b, floatx16& c) {
  c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
template <> __device__ __forceinline__ void mma_step<float>(const uint4v& a, const uint4v& b, floatx16& c) {
  const float4v fa = __builtin_bit_cast(float4v, a), fb = __builtin_bit_cast(float4v, b);
  c = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[0], fb[0], c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[1], fb[1], c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[2], fb[2], c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[3], fb[3], c, 0, 0, 0);
}

// Epilogue of a tile that lies wholly inside the output (no bounds checks): bias, rounding to the
// storage type, optional column statistics of the stored value, optional ReLU, then 16-byte
// row stores staged through this wave's LDS area.
// the 16/sizeof(T) values of a 16-byte chunk held in registers
template <typename T> __device__ __forceinline__ void unpack_chunk(const uint4v& w, float (&v)[16 / (int)sizeof(T)]);
template <> __device__ __forceinline__ void unpack_chunk<bf16_t>(const uint4v& w, float (&v)[8]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    v[2 * i] = __uint_as_float((uint32_t)w[i] << 16);
    v[2 * i + 1] = __uint_as_float((uint32_t)w[i] & 0xFFFF0000u);
  }
}
template <> __device__ __forceinline__ void unpack_chunk<float>(const uint4v& w, float (&v)[4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) v[i] = __uint_as_float((uint32_t)w[i]);
}

// Per-lane state of the companion-tensor epilogues (IgemmParams::comp): a lane stores the same 16-byte column chunk of
// every row it handles, so it keeps that chunk's column sums (and the two coefficients of xhat per column).
template <int EPC> struct CompSums { float s1[EPC], s2[EPC], p1[EPC], p0[EPC]; };

template <typename T, int MI, int NJ, int WN, int SW, bool STATS, bool RELU, bool MXQ = false, int COMP = 0>
__device__ __forceinline__ void igemm_store_interior(const floatx16 (&acc)[MI][NJ], const float (&bias)[NJ], T* stage,
                                                     T* yrow, int N, int lane, float (&s1)[NJ], float (&s2)[NJ],
                                                     const IgemmParams& p, int64_t mrow0, int phase, T* ycol,
                                                     CompSums<16 / (int)sizeof(T)>* cs = nullptr) {
  constexpr int ES = (int)sizeof(T);
  constexpr int EPC = 16 / ES;               // elements per 16-byte chunk
  constexpr int CPRO = WN / EPC;             // chunks per staged row
  const int col_lane = lane & 31, row_lane = (lane >> 5) * 4;
  const int64_t sbase = p.strips > 1 ? igemm_strip_base(p, mrow0) : 0;   // (a wave's rows lie in one 256-row tile)
  // companion tensor: all of this wave's chunks are requested before the first row is staged, so that their
  // latency runs behind the conversion and the stores of the rows before them
  constexpr int NCH = (32 * CPRO) / 64;
  uint4v cmp[COMP != 0 ? MI : 1][COMP != 0 ? NCH : 1];
  if constexpr (COMP != 0) {
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int c = 0; c < NCH; ++c) {
        const int idx = c * 64 + lane;
        const int lr = idx / CPRO, ch = idx % CPRO;
        const T* dst = (p.phases == 1 && p.strips == 1) ? yrow + (int64_t)(i * 32 + lr) * N + ch * EPC
                                                        : ycol + igemm_out_row(p, mrow0 + i * 32 + lr, phase, sbase) * N + ch * EPC;
        cmp[i][c] = *reinterpret_cast<const uint4v*>(reinterpret_cast<const T*>(p.comp) + (dst - reinterpret_cast<T*>(p.y)));
      }
  }
#pragma unroll
  for (int i = 0; i < MI; ++i) {
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int lr = (e >> 2) * 8 + row_lane + (e & 3);
        float v = acc[i][j][e] + bias[j];
        if (STATS) {   // statistics of the stored value, taken about the channel's bias (see k_bn_finalize)
          v = round_to_storage<T>(v);
          const float d = v - bias[j];
          s1[j] += d;
          s2[j] = fmaf(d, d, s2[j]);
        }
        if (RELU) v = fmaxf(v, 0.0f);          // rounding is monotonic and keeps 0: same as ReLU of the rounded value
        Store<T>::st(&stage[lr * SW + j * 32 + col_lane], v);
      }
    }
#pragma unroll
    for (int c = 0; c < (32 * CPRO) / 64; ++c) {
      const int idx = c * 64 + lane;
      const int lr = idx / CPRO, ch = idx % CPRO;
      T* dst = (p.phases == 1 && p.strips == 1) ? yrow + (int64_t)(i * 32 + lr) * N + ch * EPC
                                                : ycol + igemm_out_row(p, mrow0 + i * 32 + lr, phase, sbase) * N + ch * EPC;
      if constexpr (MXQ) {
        // MX block quantisation of the stored row: a block of mx_block columns is mx_block/EPC neighbouring lanes of this
        // pass (a staged row is CPRO >= mx_block/EPC consecutive lanes, blocks do not straddle rows)
        float f[EPC];
        Store<T>::ldv(&stage[lr * SW + ch * EPC], f);
        float amax = 0.0f;
#pragma unroll
        for (int t = 0; t < EPC; ++t) amax = fmaxf(amax, fabsf(f[t]));
        for (int off = 1; off < p.mx_block / EPC; off <<= 1) amax = fmaxf(amax, __shfl_xor(amax, off, 64));
        if (amax > 0.0f) {
          const int k = mx_scale_exp(amax, p.mx_elem == MX_FP8 ? 8 : (p.mx_elem == MX_INT4 ? 0 : 2));
          const float sc = ldexpf(1.0f, k), inv_sc = ldexpf(1.0f, -k);
#pragma unroll
          for (int t = 0; t < EPC; ++t)
            f[t] = p.mx_elem == MX_FP8 ? MxFormat<MX_FP8>::quant(f[t], inv_sc, sc)
                                       : (p.mx_elem == MX_INT4 ? MxFormat<MX_INT4>::quant(f[t], inv_sc, sc) : mx_quant_e2m1(f[t], inv_sc, sc));
        }
        Store<T>::stv(dst, f);
      } else if constexpr (COMP != 0) {
        float f[EPC], a[EPC];
        Store<T>::ldv(&stage[lr * SW + ch * EPC], f);
        unpack_chunk<T>(cmp[i][c], a);
#pragma unroll
        for (int t = 0; t < EPC; ++t) {
          const float dyv = a[t] > 0.0f ? f[t] : 0.0f;
          cs->s1[t] += dyv;
          if (COMP == 2) cs->s2[t] = fmaf(dyv, fmaf(a[t], cs->p1[t], cs->p0[t]), cs->s2[t]);
          else f[t] = dyv;
        }
        if (COMP == 1) Store<T>::stv(dst, f);
        else *reinterpret_cast<uint4v*>(dst) = *reinterpret_cast<const uint4v*>(&stage[lr * SW + ch * EPC]);
      } else {
        *reinterpret_cast<uint4v*>(dst) = *reinterpret_cast<const uint4v*>(&stage[lr * SW + ch * EPC]);
      }
    }
  }
}

// Epilogue variant 2: column sums of resid - (acc + bias) and of its square over the tile's rows; nothing stored.
template <typename T, int MI, int NJ>
__device__ __forceinline__ void igemm_resid_stats(const floatx16 (&acc)[MI][NJ], const float (&bias)[NJ], const T* rrow, int N,
                                                  int lane, float (&s1)[NJ], float (&s2)[NJ]) {
  const int col_lane = lane & 31, row_lane = (lane >> 5) * 4;
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int lr = (e >> 2) * 8 + row_lane + (e & 3);
        const float dv = Store<T>::ld(rrow + (int64_t)(i * 32 + lr) * N + j * 32 + col_lane) - (acc[i][j][e] + bias[j]);
        s1[j] += dv;
        s2[j] = fmaf(dv, dv, s2[j]);
      }
}

// Epilogue shared by the implicit-GEMM kernels.  Accumulator element e of lane l in tile (i,j):
//     row = wm*WM + i*32 + (e/4)*8 + (l/32)*4 + e%4,  column = wn*WN + j*32 + l%32
// Results go through a wave-private LDS staging area (the operand buffers are free: the K loop
// ended on a barrier) so that global stores are 16 bytes wide and each instruction covers
// whole row segments.  smem: at least 4*32*(WN + 16/sizeof(T))*sizeof(T) bytes; sRed: [WGM][2][BN].
template <typename T, int BM, int BN, int WGM, int WGN, bool INTERIOR, int EPI = 0>
__device__ __forceinline__ void igemm_epilogue(floatx16 (&acc)[BM / WGM / 32][BN / WGN / 32], const IgemmParams& p,
                                               char* smem, float (*sRed)[2][BN], int64_t m0, int n0, int64_t tile_m,
                                               int phase = 0) {
  constexpr int ES = (int)sizeof(T);
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int MI = WM / 32, NJ = WN / 32;
  constexpr int SW = WN + 16 / ES;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  T* __restrict__ Y = (T*)p.y;
  const int col_lane = lane & 31, row_lane = (lane >> 5) * 4;
  const bool wide_store = ((p.N * ES) % 16 == 0) && !p.y_aux;
  T* stage = reinterpret_cast<T*>(smem) + wave * (32 * SW);
  float s1[NJ], s2[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) { s1[j] = 0.0f; s2[j] = 0.0f; }
  if constexpr (INTERIOR) {
    float bias[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) bias[j] = p.bias ? p.bias[n0 + wn * WN + j * 32 + col_lane] : 0.0f;
    T* yrow = Y + (m0 + wm * WM) * p.N + n0 + wn * WN;
    T* ycol = Y + n0 + wn * WN;
    const int64_t mrow0 = m0 + wm * WM;
    if constexpr (EPI == 1)
      igemm_store_interior<T, MI, NJ, WN, SW, false, false, true>(acc, bias, stage, yrow, p.N, lane, s1, s2, p, mrow0, phase, ycol);
    else if constexpr (EPI == 2)
      igemm_resid_stats<T, MI, NJ>(acc, bias, (const T*)p.resid + (m0 + wm * WM) * p.N + n0 + wn * WN, p.N, lane, s1, s2);
    else if constexpr (EPI == 3 || EPI == 4) {
      // companion-tensor sums (EPI 3: IgemmParams::comp_mode 1, EPI 4: comp_mode 2): this lane's chunk of columns is the same in every row it stores (CPRO divides 64)
      constexpr int EPC = 16 / ES, CPRO = WN / EPC;
      static_assert(64 % CPRO == 0, "a lane keeps one column chunk");
      CompSums<EPC> cs;
      const int colc = n0 + wn * WN + (lane % CPRO) * EPC;
#pragma unroll
      for (int t = 0; t < EPC; ++t) {
        cs.s1[t] = 0.0f; cs.s2[t] = 0.0f; cs.p1[t] = 0.0f; cs.p0[t] = 0.0f;
        if (EPI == 4) {
          const float sc = p.comp_bn[colc + t], sh = p.comp_bn[p.N + colc + t];
          const float mu = p.comp_bn[2 * p.N + colc + t], is = p.comp_bn[3 * p.N + colc + t];
          if (sc != 0.0f) {
            const float inv = 1.0f / sc;
            cs.p1[t] = is * inv;
            cs.p0[t] = -(sh * inv + mu) * is;
          }
        }
      }
      igemm_store_interior<T, MI, NJ, WN, SW, false, false, false, EPI - 2>(acc, bias, stage, yrow, p.N, lane, s1, s2, p, mrow0, phase, ycol, &cs);
#pragma unroll
      for (int t = 0; t < EPC; ++t) {
        for (int off = CPRO; off < 64; off <<= 1) {
          cs.s1[t] += __shfl_xor(cs.s1[t], off, 64);
          cs.s2[t] += __shfl_xor(cs.s2[t], off, 64);
        }
        if (lane < CPRO) {
          sRed[wm][0][wn * WN + lane * EPC + t] = cs.s1[t];
          sRed[wm][1][wn * WN + lane * EPC + t] = cs.s2[t];
        }
      }
    }
    else if (p.partial) igemm_store_interior<T, MI, NJ, WN, SW, true, false>(acc, bias, stage, yrow, p.N, lane, s1, s2, p, mrow0, phase, ycol);
    else if (p.act == ACT_RELU) igemm_store_interior<T, MI, NJ, WN, SW, false, true>(acc, bias, stage, yrow, p.N, lane, s1, s2, p, mrow0, phase, ycol);
    else igemm_store_interior<T, MI, NJ, WN, SW, false, false>(acc, bias, stage, yrow, p.N, lane, s1, s2, p, mrow0, phase, ycol);
  } else {
#pragma unroll
    for (int i = 0; i < MI; ++i) {
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const int col = n0 + wn * WN + j * 32 + col_lane;
        const bool col_ok = col < p.N;
        const float bias = (p.bias && col_ok) ? p.bias[col] : 0.0f;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int lr = (e >> 2) * 8 + row_lane + (e & 3);
          const int64_t m = m0 + wm * WM + i * 32 + lr;
          const float v = round_to_storage<T>(acc[i][j][e] + bias);   // the stored conv result
          if (p.partial && m < p.M && col_ok) { const float d = v - bias; s1[j] += d; s2[j] = fmaf(d, d, s2[j]); }
          const float a = apply_act(v, p.act);
          if (wide_store) {
            Store<T>::st(&stage[lr * SW + j * 32 + col_lane], a);
          } else if (m < p.M && col_ok) {
            Store<T>::st(&Y[m * p.N + col], a);
            if (p.y_aux) p.y_aux[m * p.N + col] = a;
          }
        }
      }
      if (wide_store) {
        constexpr int EPC = 16 / ES;               // elements per 16-byte chunk
        constexpr int CPRO = WN / EPC;             // chunks per staged row
#pragma unroll
        for (int c = 0; c < (32 * CPRO) / 64; ++c) {
          const int idx = c * 64 + lane;
          const int lr = idx / CPRO, ch = idx % CPRO;
          const int64_t m = m0 + wm * WM + i * 32 + lr;
          const int col0 = n0 + wn * WN + ch * EPC;
          if (m < p.M && col0 < p.N)
            *reinterpret_cast<uint4v*>(Y + m * p.N + col0) = *reinterpret_cast<const uint4v*>(&stage[lr * SW + ch * EPC]);
        }
      }
    }
  }
  if (p.partial && EPI != 3 && EPI != 4) {
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      float t1 = s1[j] + __shfl_xor(s1[j], 32, 64);
      float t2 = s2[j] + __shfl_xor(s2[j], 32, 64);
      if (lane < 32) {
        sRed[wm][0][wn * WN + j * 32 + col_lane] = t1;
        sRed[wm][1][wn * WN + j * 32 + col_lane] = t2;
      }
    }
  }
  if (p.partial) {
    __syncthreads();
    for (int i = tid; i < 2 * BN; i += WGM * WGN * 64) {
      const int q = i / BN, c = i - q * BN;
      float t = 0.0f;
#pragma unroll
      for (int g = 0; g < WGM; ++g) t += sRed[g][q][c];
      if (n0 + c < p.N) p.partial[(tile_m * 2 + q) * p.N + n0 + c] = t;
    }
  }
}

// ---- hand-scheduled LDS fragment reads of the DMA pipeline -------------------------------
// The compiler orders an LDS read after EVERY outstanding global-to-LDS load (it cannot tell
// the stages apart), which would serialise the pipeline; these reads are therefore issued as
// inline assembly, and the waits on them (lgkmcnt) are placed by hand: LDS reads of a wave
// return in order, so "at most n outstanding" identifies which fragments have arrived.  An
// empty asm with the fragment as in/out operand keeps the MFMAs after the wait.
typedef __attribute__((address_space(3))) char lds_char;
typedef __attribute__((address_space(3))) void lds_void_t;
// 16 bytes per lane from a buffer straight into LDS: lane l writes lds_wave_base + 16*l
// (offsets past the buffer's range deliver zeros like any buffer load)
__device__ __forceinline__ void dma_load16(__amdgpu_buffer_rsrc_t rsrc, char* lds_wave_base, unsigned voffset) {
  typedef __attribute__((address_space(3))) void lds_void;
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void*)lds_wave_base, 16, voffset, 0, 0, 0);
}
// the same with a scalar (uniform) byte offset added to every lane's offset
__device__ __forceinline__ void dma_load16s(__amdgpu_buffer_rsrc_t rsrc, char* lds_wave_base, unsigned voffset, unsigned soffset) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void_t*)lds_wave_base, 16, voffset, soffset, 0, 0);
}
template <int I, int N, int STRIDE>
struct LdsReadFrags {
  static __device__ __forceinline__ void run(uint4v (&f)[N], unsigned addr) {
#if defined(__HIP_DEVICE_COMPILE__)             // the host pass only needs the kernel's stub
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(f[I]) : "v"(addr), "n"(I * STRIDE));
#endif
    LdsReadFrags<I + 1, N, STRIDE>::run(f, addr);
  }
};
template <int N, int STRIDE>
struct LdsReadFrags<N, N, STRIDE> {
  static __device__ __forceinline__ void run(uint4v (&)[N], unsigned) {}
};
template <int I, int N>
struct TieFrags {
  static __device__ __forceinline__ void run(uint4v (&f)[N]) {
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("" : "+v"(f[I]));
#endif
    TieFrags<I + 1, N>::run(f);
  }
};
template <int N>
struct TieFrags<N, N> {
  static __device__ __forceinline__ void run(uint4v (&)[N]) {}
};
// MFMAs of K-steps K .. KS-1 of one slab; fragments of step k arrived once at most
// (KS-1-k)*(MI+NJ) reads are outstanding
template <typename T, int KS, int K, int MI, int NJ>
struct SlabSteps {
  static __device__ __forceinline__ void run(uint4v (&a)[KS][MI], uint4v (&b)[KS][NJ], floatx16 (&acc)[MI][NJ]) {
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"((KS - 1 - K) * (MI + NJ)));
#endif
    TieFrags<0, MI>::run(a[K]);
    TieFrags<0, NJ>::run(b[K]);
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NJ; ++j) mma_step<T>(a[K][i], b[K][j], acc[i][j]);
    __builtin_amdgcn_sched_barrier(0);           // keep these MFMAs ahead of the next step's wait
    SlabSteps<T, KS, K + 1, MI, NJ>::run(a, b, acc);
  }
};
template <typename T, int KS, int MI, int NJ>
struct SlabSteps<T, KS, KS, MI, NJ> {
  static __device__ __forceinline__ void run(uint4v (&)[KS][MI], uint4v (&)[KS][NJ], floatx16 (&)[MI][NJ]) {}
};
template <int K, int KS, int MI, int NJ, int BKB>
struct SlabReads {
  static __device__ __forceinline__ void run(uint4v (&a)[KS][MI], uint4v (&b)[KS][NJ], unsigned addr_a, unsigned addr_b,
                                             const int (&lane_off)[KS]) {
    LdsReadFrags<0, NJ, 32 * BKB>::run(b[K], addr_b + (unsigned)lane_off[K]);
    LdsReadFrags<0, MI, 32 * BKB>::run(a[K], addr_a + (unsigned)lane_off[K]);
    SlabReads<K + 1, KS, MI, NJ, BKB>::run(a, b, addr_a, addr_b, lane_off);
  }
};
template <int KS, int MI, int NJ, int BKB>
struct SlabReads<KS, KS, MI, NJ, BKB> {
  static __device__ __forceinline__ void run(uint4v (&)[KS][MI], uint4v (&)[KS][NJ], unsigned, unsigned, const int (&)[KS]) {}
};

// INTERIOR: the host guarantees M % BM == 0, N % BN == 0, 16-byte aligned rows, no sigmoid, no
// auxiliary copy and no activation together with statistics, so the epilogue needs no checks.
// DMA: the slabs go from global memory straight into LDS (buffer loads with the LDS
// destination: lane l of a wave writes 16 bytes at base + 16*l, which is exactly the loader's
// linear slot order), three stages deep, so loads run two slabs ahead without holding
// registers.  A wave waits for its own loads of the slab it is about to read (vmcnt), then
// the workgroup barrier makes every wave's loads visible and also guarantees that the stage
// about to be refilled has been read by everybody.
template <typename T, int BM, int BN, int WGM, int WGN, int BKB, bool INTERIOR, bool DMA, int EPI = 0>
__global__ __launch_bounds__(WGM * WGN * 64) __attribute__((amdgpu_waves_per_eu(2))) void k_igemm(IgemmParams p) {
  static_assert(EPI == 0 || INTERIOR, "the special epilogues exist for check-free tiles only");
  static_assert(WGM * WGN == 4 || WGM * WGN == 8, "four or eight wavefronts per workgroup");
  constexpr int NT = WGM * WGN * 64;            // threads: all of them load, each wavefront owns a WM x WN part of the tile
  static_assert(BKB == 64 || BKB == 128, "slab row bytes");
  constexpr int ES = (int)sizeof(T);
  constexpr int BK = BKB / ES;                  // K elements per slab
  constexpr int CPR = BKB / 16;                 // 16-byte chunks per slab row
  constexpr int RSTEP = NT / CPR;               // rows covered by one pass of the loader threads
  constexpr int WM = BM / WGM, WN = BN / WGN;   // wave tile
  constexpr int MI = WM / 32, NJ = WN / 32;     // 32x32 MFMA tiles per wave
  constexpr int A_CHUNKS = BM / RSTEP, B_CHUNKS = BN / RSTEP;
  constexpr int SW = WN + 16 / ES;              // staging row stride of the epilogue (elements): +16 bytes
  constexpr int NSTAGE = DMA ? (NT == 512 ? 4 : 3) : 2;   // eight wavefronts: one workgroup per compute unit, LDS for a fourth stage
  constexpr int SLAB_BYTES = NSTAGE * (BM + BN) * BKB;
  constexpr int STAGE_BYTES = (NT / 64) * 32 * SW * ES;
  __shared__ __attribute__((aligned(16))) char smem[SLAB_BYTES > STAGE_BYTES ? SLAB_BYTES : STAGE_BYTES];
  char* const sA = smem;                        // [NSTAGE][BM*BKB]
  char* const sB = smem + NSTAGE * BM * BKB;    // [NSTAGE][BN*BKB]
  __shared__ float sRed[WGM][2][BN];            // [wave row][sum | sumsq][column]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  int lb0 = xcd_logical_block((int)blockIdx.x, (int)gridDim.x);
  // triangular products: tile rows differ in work by an order of magnitude, so neighbouring tiles go to different
  // XCDs (the hardware's own round-robin) instead of one contiguous range per XCD, the longest K ranges first
  if (p.tri != 0 && p.tri < 8) lb0 = p.tri == 1 ? (int)gridDim.x - 1 - (int)blockIdx.x : (int)blockIdx.x;
  if (p.tri == 4 && (gridDim.x & 63) == 0) {    // runs of eight consecutive tiles per XCD (they share an operand panel in its L2), runs interleaved
    const int i = (int)blockIdx.x >> 3, x = (int)blockIdx.x & 7;
    lb0 = ((((i >> 3) << 3) + x) << 3) + (i & 7);
  }
  int phase = 0;
  if (p.phases == 4) { phase = lb0 & 3; lb0 >>= 2; }   // the four phases of a tile run side by side: they read the same input
  const int split = INTERIOR ? 0 : lb0 / p.tiles_mn;
  const int lb = INTERIOR ? lb0 : lb0 - split * p.tiles_mn;
  // tile order: groups of kGroupM tile rows are walked column by column, so the workgroups in flight on an XCD
  // cover a squarish patch of the output (few distinct operand rows per K slab in its L2) instead of a wide strip
  constexpr int kGroupM = 4;
  const int gsz = kGroupM * p.tiles_n, grp = lb / gsz, in_grp = lb - grp * gsz;
  const int gm = min(p.tiles_mn / p.tiles_n - grp * kGroupM, kGroupM);
  int tile_n = in_grp / gm;
  int64_t tile_m = grp * kGroupM + in_grp % gm;
  if (p.tri == 3) {                             // K range [column, K): walk column by column, the longest first
    const int tiles_m = p.tiles_mn / p.tiles_n;
    tile_n = lb / tiles_m;
    tile_m = lb - tile_n * tiles_m;
  }
  if (p.tri == 4 && p.tiles_mn == p.tiles_n * p.tiles_n) {
    // K range [max(row, column), K): on a square tile grid walk the L-shaped shells max(tile row, tile column) = 0, 1, ...
    // so that the workgroups are dispatched longest first and the hardware's in-order dispatch balances the rest
    int sh = (int)sqrtf((float)lb);
    while (sh * sh > lb) --sh;
    while ((sh + 1) * (sh + 1) <= lb) ++sh;
    const int r = lb - sh * sh;                 // 0 .. 2 sh
    tile_m = r <= sh ? r : sh;
    tile_n = r <= sh ? sh : r - sh - 1;
  }
  if (p.tri >= 8) {                             // only the tiles of one off-diagonal block per pair are launched
    const int tbm = p.tri_b / BM, tbn = p.tri_b / BN, per_pair = tbm * tbn;
    const int pair = lb / per_pair, in_pair = lb - pair * per_pair;
    const int tr = in_pair / tbn, tc = in_pair - tr * tbn;
    tile_m = (2 * pair + (p.tri == 9 ? 1 : 0)) * tbm + tr;
    tile_n = (2 * pair + (p.tri == 9 ? 0 : 1)) * tbn + tc;
  }
  const int64_t m0 = tile_m * BM;
  const int n0 = tile_n * BN;
  const int pad_h = p.pad - (phase >> 1), pad_w = p.pad - (phase & 1);
  const int Hin = p.Hv >> p.up, Win = p.Wv >> p.up;
  const __amdgpu_buffer_rsrc_t rX = make_rsrc(p.x, p.x_bytes);
  const __amdgpu_buffer_rsrc_t rW = make_rsrc(p.w, p.w_bytes);

  // --- loader bookkeeping: thread t moves rows (t / CPR) + RSTEP*i, LDS slot t % CPR of each
  const int slot = tid % CPR;
  const int lrow = tid / CPR;
  const int fsw = BKB == 64 ? ((lrow >> 2) & 3) : ((lrow >> 1) & 7);   // RSTEP*i does not touch these bits
  const int gchunk = slot ^ fsw;
  int a_h[A_CHUNKS], a_w[A_CHUNKS];
  unsigned a_img[A_CHUNKS];                     // byte offset of the sample's image, kOob if the row is past M
  unsigned a_off[A_CHUNKS];                     // byte offset of the current tap's pixel (+ chunk), kOob if padding
#pragma unroll
  for (int i = 0; i < A_CHUNKS; ++i) {
    const int64_t m = m0 + lrow + i * RSTEP;
    const bool ok = m < p.M;
    const unsigned mu = ok ? (unsigned)m : 0u;
    a_w[i] = (int)(mu % (unsigned)p.Wc);
    const unsigned t = mu / (unsigned)p.Wc;
    a_h[i] = (int)(t % (unsigned)p.Hc);
    a_img[i] = ok ? (t / (unsigned)p.Hc) * (unsigned)(Hin * Win) * (unsigned)p.Cin * (unsigned)ES : kOob;
  }
  unsigned b_off[B_CHUNKS];
#pragma unroll
  for (int i = 0; i < B_CHUNKS; ++i) {
    const int row = n0 + lrow + i * RSTEP;
    b_off[i] = row < p.N ? (unsigned)(phase * p.N + row) * (unsigned)p.K * (unsigned)ES + (unsigned)gchunk * 16u : kOob;
  }

  int k_lo = 0, k_hi = p.K;                                             // triangular operands: see IgemmParams::tri
  if (p.tri == 1) k_hi = (int)min((int64_t)p.K, min(m0 + BM, (int64_t)n0 + BN));
  else if (p.tri == 2) { if ((int64_t)n0 + BN <= m0) return; k_lo = (int)m0; }
  else if (p.tri == 3) { if ((int64_t)n0 >= m0 + BM) return; k_lo = n0; }
  else if (p.tri == 4) k_lo = (int)max(m0, (int64_t)n0);
  else if (p.tri >= 8) {
    const int rb = (int)(m0 / p.tri_b), cb = n0 / p.tri_b;
    if (p.tri == 9 ? !((rb & 1) == 1 && cb == rb - 1) : !((rb & 1) == 0 && cb == rb + 1)) return;
    k_lo = rb * p.tri_b;
    k_hi = k_lo + p.tri_b;
    if (p.tri_d > 0) {
      if ((p.tri == 9 ? m0 : (int64_t)n0) >= p.tri_d) return;
      if (p.tri == 9) k_hi = min(k_hi, p.tri_d);
    }
  }
  const int kt_lo = k_lo / BK, kt_hi = (k_hi + BK - 1) / BK;
  const int kt0 = INTERIOR ? kt_lo : max(kt_lo, split * p.slabs_per_split);   // first K slab of this workgroup
  int rs = (kt0 * BK) / p.Cin, ci0 = (kt0 * BK) % p.Cin;                // filter tap and first channel of the next slab to load
  unsigned kbyte = (unsigned)(kt0 * BKB);       // byte offset of the next slab inside a weight row
#define IGEMM_TAP()                                                                                          \
  {                                                                                                          \
    const int r_ = rs / p.ksz, s_ = rs - r_ * p.ksz;                                                         \
    _Pragma("unroll") for (int i = 0; i < A_CHUNKS; ++i) {                                                   \
      const int hh = a_h[i] * p.stride + r_ - pad_h, ww = a_w[i] * p.stride + s_ - pad_w;                    \
      const bool ok = a_img[i] != kOob && hh >= 0 && hh < p.Hv && ww >= 0 && ww < p.Wv;                      \
      const unsigned pix = (unsigned)((hh >> p.up) * Win + (ww >> p.up));                                    \
      a_off[i] = ok ? a_img[i] + pix * (unsigned)p.Cin * (unsigned)ES + (unsigned)gchunk * 16u : kOob;       \
    }                                                                                                        \
  }
#define IGEMM_LOAD(RA, RB)                                                                                   \
  {                                                                                                          \
    if (ci0 == 0) IGEMM_TAP();                                                                               \
    _Pragma("unroll") for (int i = 0; i < A_CHUNKS; ++i)                                                     \
        RA[i] = __builtin_amdgcn_raw_buffer_load_b128(rX, a_off[i] + (unsigned)ci0 * (unsigned)ES, 0, 0);    \
    _Pragma("unroll") for (int i = 0; i < B_CHUNKS; ++i)                                                     \
        RB[i] = __builtin_amdgcn_raw_buffer_load_b128(rW, b_off[i] + kbyte, 0, 0);                           \
    ci0 += BK;                                                                                               \
    kbyte += BKB;                                                                                            \
    if (ci0 == p.Cin) { ci0 = 0; ++rs; }                                                                     \
  }
  const int st_off = lrow * BKB + slot * 16;    // this thread's byte offset inside a slab buffer (+ i*RSTEP*BKB)
#define IGEMM_STORE(BUF, RA, RB)                                                                             \
  {                                                                                                          \
    _Pragma("unroll") for (int i = 0; i < A_CHUNKS; ++i)                                                     \
        *reinterpret_cast<uint4v*>(sA + (BUF) * BM * BKB + st_off + i * RSTEP * BKB) = RA[i];                \
    _Pragma("unroll") for (int i = 0; i < B_CHUNKS; ++i)                                                     \
        *reinterpret_cast<uint4v*>(sB + (BUF) * BN * BKB + st_off + i * RSTEP * BKB) = RB[i];                \
  }
  // fragment reads: lane l wants row (l%32) of a 32-row MFMA tile, chunk 2*ks + l/32;
  // the lane-dependent part of the address is the same for A and B and for every tile
  const int frag_row = lane & 31, frag_c = lane >> 5;
  const int ffr = BKB == 64 ? ((frag_row >> 2) & 3) : ((frag_row >> 1) & 7);
  int lane_off[BKB / 32];
#pragma unroll
  for (int ks = 0; ks < BKB / 32; ++ks) lane_off[ks] = frag_row * BKB + (((ks * 2 + frag_c) ^ ffr) * 16);
#define IGEMM_COMPUTE(BUF)                                                                                   \
  {                                                                                                          \
    _Pragma("unroll") for (int ks = 0; ks < BKB / 32; ++ks) {                                                \
      uint4v a[MI], b[NJ];                                                                                   \
      _Pragma("unroll") for (int i = 0; i < MI; ++i)                                                         \
          a[i] = *reinterpret_cast<const uint4v*>(sA + (BUF) * BM * BKB + (wm * WM + i * 32) * BKB + lane_off[ks]); \
      _Pragma("unroll") for (int j = 0; j < NJ; ++j)                                                         \
          b[j] = *reinterpret_cast<const uint4v*>(sB + (BUF) * BN * BKB + (wn * WN + j * 32) * BKB + lane_off[ks]); \
      _Pragma("unroll") for (int i = 0; i < MI; ++i)                                                         \
        _Pragma("unroll") for (int j = 0; j < NJ; ++j) mma_step<T>(a[i], b[j], acc[i][j]);                   \
    }                                                                                                        \
  }

  floatx16 acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  const int KT = INTERIOR ? kt_hi - kt0 : min(kt_hi - kt0, p.slabs_per_split);   // (tri launches have one split)
  if (ci0 != 0) IGEMM_TAP();                     // a split that starts inside a tap (the loaders compute a tap's offsets at its first slab)
  if constexpr (DMA) {
    constexpr int L = A_CHUNKS + B_CHUNKS;       // loads per thread and slab
    static_assert(RSTEP * BKB == NT * 16, "one pass of the loader covers 16 bytes per thread");
#define IGEMM_DMA(STG)                                                                                       \
  {                                                                                                          \
    if (ci0 == 0) IGEMM_TAP();                                                                               \
    char* const da = sA + (STG) * BM * BKB + wave * 1024;                                                    \
    char* const db = sB + (STG) * BN * BKB + wave * 1024;                                                    \
    _Pragma("unroll") for (int i = 0; i < A_CHUNKS; ++i)                                                     \
        dma_load16(rX, da + i * (NT * 16), a_off[i] + (unsigned)ci0 * (unsigned)ES);                         \
    _Pragma("unroll") for (int i = 0; i < B_CHUNKS; ++i)                                                     \
        dma_load16(rW, db + i * (NT * 16), b_off[i] + kbyte);                                                \
    ci0 += BK;                                                                                               \
    kbyte += BKB;                                                                                            \
    if (ci0 == p.Cin) { ci0 = 0; ++rs; }                                                                     \
  }
    constexpr int KS = BKB / 32;
    const unsigned lds_a = (unsigned)(size_t)(lds_char*)sA + (unsigned)(wm * WM * BKB);
    const unsigned lds_b = (unsigned)(size_t)(lds_char*)sB + (unsigned)(wn * WN * BKB);
    IGEMM_DMA(0);
    if (KT > 1) IGEMM_DMA(1);
    if constexpr (NSTAGE == 4) { if (KT > 2) IGEMM_DMA(2); }
    int cur = 0, nxt = NSTAGE - 1;
    for (int kt = 0; kt < KT; ++kt) {
      // vmcnt(n): at most n of this wave's loads outstanding (they complete in order): the slabs issued after slab kt;
      // the other counters are left alone (expcnt 7, lgkmcnt 15)
      if (NSTAGE == 4 && kt + 2 < KT) __builtin_amdgcn_s_waitcnt(((2 * L) & 15) | (((2 * L) >> 4) << 14) | 0x0F70);
      else if (kt + 1 < KT) __builtin_amdgcn_s_waitcnt((L & 15) | ((L >> 4) << 14) | 0x0F70);
      else __builtin_amdgcn_s_waitcnt(0x0F70);
      __builtin_amdgcn_s_barrier();
      uint4v fa[KS][MI], fb[KS][NJ];
      SlabReads<0, KS, MI, NJ, BKB>::run(fa, fb, lds_a + (unsigned)(cur * BM * BKB), lds_b + (unsigned)(cur * BN * BKB), lane_off);
      if (kt + NSTAGE - 1 < KT) IGEMM_DMA(nxt);
      SlabSteps<T, KS, 0, MI, NJ>::run(fa, fb, acc);
      cur = cur == NSTAGE - 1 ? 0 : cur + 1;
      nxt = nxt == NSTAGE - 1 ? 0 : nxt + 1;
    }
#undef IGEMM_DMA
    __syncthreads();                             // every wave is done with the slabs: the epilogue reuses the memory
  } else {
  uint4v ra0[A_CHUNKS], rb0[B_CHUNKS], ra1[A_CHUNKS], rb1[B_CHUNKS];
  IGEMM_LOAD(ra0, rb0);
  if (KT > 1) IGEMM_LOAD(ra1, rb1);
  IGEMM_STORE(0, ra0, rb0);
  __syncthreads();
  for (int kt = 0; kt < KT; kt += 2) {
    // even slab: LDS buffer 0; register set 1 holds slab kt+1; set 0 is free
    if (kt + 2 < KT) IGEMM_LOAD(ra0, rb0);
    IGEMM_COMPUTE(0);
    if (kt + 1 < KT) IGEMM_STORE(1, ra1, rb1);
    __syncthreads();
    if (kt + 1 >= KT) break;
    // odd slab: LDS buffer 1; register set 0 holds slab kt+2; set 1 is free
    if (kt + 3 < KT) IGEMM_LOAD(ra1, rb1);
    IGEMM_COMPUTE(1);
    if (kt + 2 < KT) IGEMM_STORE(0, ra0, rb0);
    __syncthreads();
  }
  }
#undef IGEMM_TAP
#undef IGEMM_LOAD
#undef IGEMM_STORE
#undef IGEMM_COMPUTE

  if constexpr (!INTERIOR) {
    if (p.split_out) {
      float* __restrict__ P = p.split_out + (int64_t)split * p.M * p.N;
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
          const int col = n0 + wn * WN + j * 32 + (lane & 31);
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int64_t m = m0 + wm * WM + i * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
            if (m < p.M && col < p.N) P[m * p.N + col] = acc[i][j][e];
          }
        }
      return;
    }
  }
  igemm_epilogue<T, BM, BN, WGM, WGN, INTERIOR, EPI>(acc, p, smem, sRed, m0, n0, tile_m, phase);
}

// y = act(round(sum over splits of partial[split] + bias)) for split-K launches
template <typename T>
__global__ void k_splitk_finish(const float* __restrict__ partial, int splits, int64_t M, int N, const float* __restrict__ bias,
                                int act, T* __restrict__ y, float* __restrict__ y_aux) {
  const int64_t total = M * N;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    float acc = 0.0f;
#pragma unroll 8
    for (int sp = 0; sp < splits; ++sp) acc += partial[(int64_t)sp * total + i];
    if (bias) acc += bias[(int)(i % N)];
    const float a = apply_act(round_to_storage<T>(acc), act);
    Store<T>::st(y + i, a);
    if (y_aux) y_aux[i] = a;
  }
}

// wait until at most N LDS reads are outstanding, then hand the fragments to the compiler
template <int N, int MI>
__device__ __forceinline__ void lds_wait_tie_a(uint4v (&a)[MI]) {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N));
#endif
  TieFrags<0, MI>::run(a);
}
template <typename T, int MI, int NJ>
__device__ __forceinline__ void mma_group(const uint4v (&a)[MI], const uint4v (&b)[NJ], floatx16 (&acc)[MI][NJ]) {
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j) mma_step<T>(a[i], b[j], acc[i][j]);
}

// A-fragment reads of the patch kernel: one address per 32-pixel tile, K-step selected by ^ 32
template <int I, int N>
struct Conv3Reads {
  static __device__ __forceinline__ void run(uint4v (&f)[N], const unsigned (&addr)[N], unsigned kxor) {
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("ds_read_b128 %0, %1" : "=v"(f[I]) : "v"(addr[I] ^ kxor));
#endif
    Conv3Reads<I + 1, N>::run(f, addr, kxor);
  }
};
template <int N>
struct Conv3Reads<N, N> {
  static __device__ __forceinline__ void run(uint4v (&)[N], const unsigned (&)[N], unsigned) {}
};

// ---------------------------------------------------------------------------
// 3x3 convolution with the input patch resident in LDS and the weights straight in registers.
//
// The per-tap kernel above fetches every input pixel nine times (once per filter tap) through
// the vector cache, whose 64 bytes per clock and compute unit then bound the MFMA rate.  Here a
// workgroup owns TH = 256/W whole image rows (W = image width, a template parameter) and, for
// each slab of 64 bytes of input channels, loads the (TH+2) x (W+2) patch of pixels around its
// rows ONCE — zero padding included, delivered by the buffer range check — and forms all nine
// taps from it: tap (r,s) of pixel (th,tw) is patch cell (th+r, tw+s).
//
// LDS: the patch is double buffered, cells of 64 bytes stored linearly (the global-to-LDS load
// writes lane l at base + 16*l), chunk c of cell q in slot c ^ ((q>>2)&3), so that the 16 cells
// a fragment read touches per pass fall into 16 different 16-byte columns for any tap shift.
//
// Weights never enter LDS (two wavefronts at most share a column, and the LDS port is what
// the patch fragments need): they are packed in fragment order (ConvArgs::w_frag) — the 32
// rows x 32 K-bytes block (nb, kb) is one KiB at (nb * K-bytes/32 + kb) KiB, lane l's MFMA
// operand at byte 16 l of it — and a wave loads the operands of its own WN columns into
// registers two steps ahead (ring of three stages; nine taps, so a tap always uses stage
// tap % 3).  The K loop runs channel slab outer, tap inner (nine steps, fully unrolled); a
// share of the next slab's patch loads is issued at taps 0..6.  The workgroup needs two
// barriers per channel slab: before tap 8, when every wave's share of the next patch has
// landed (tap 8 reads that patch's first fragments), and before tap 0, when every wave has
// read its last fragments of the patch buffer that the loads issued from then on overwrite.
// ---------------------------------------------------------------------------
constexpr int patch_passes(int w) { return (((256 / w + 2) * (w + 2)) * 4 + 255) / 256; }
// patch passes of the next channel slab issued at tap `tap` (spread over taps 0..6)
constexpr int passes_at(int passes, int tap) { return tap < 7 ? passes / 7 + (tap < passes % 7 ? 1 : 0) : 0; }
constexpr int passes_before(int passes, int tap) {
  int n = 0;
  for (int t = 0; t < tap; ++t) n += passes_at(passes, t);
  return n;
}
constexpr int vm_imm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0F70; }   // s_waitcnt vmcnt(n) only

template <typename T, int BN, int WGM, int WGN, int W, bool INTERIOR, int EPI = 0>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void k_conv3_patch(IgemmParams p) {
  static_assert(WGM * WGN == 4, "four wavefronts per workgroup");
  constexpr int ES = (int)sizeof(T);
  constexpr int BM = 256, BKB = 64;
  constexpr int TH = BM / W, PW = W + 2, PC = (TH + 2) * PW;
  constexpr int PASSES = patch_passes(W);
  constexpr int PATCH_BYTES = PASSES * 4096;
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int MI = WM / 32, NJ = WN / 32;
  constexpr int SW = WN + 16 / ES;
  constexpr int OPER_BYTES = 2 * PATCH_BYTES;
  constexpr int EPI_BYTES = 4 * 32 * SW * ES + WGM * 2 * BN * 4;
  __shared__ __attribute__((aligned(64))) char smem[OPER_BYTES > EPI_BYTES ? OPER_BYTES : EPI_BYTES];
  char* const sP = smem;                        // [2][PATCH_BYTES]
  float (*sRed)[2][BN] = reinterpret_cast<float (*)[2][BN]>(smem + 4 * 32 * SW * ES);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int lb = xcd_logical_block((int)blockIdx.x, (int)gridDim.x);
  const int tile_n = lb % p.tiles_n;
  const int tile_m = lb / p.tiles_n;
  const int64_t m0 = (int64_t)tile_m * BM;
  const int n0 = tile_n * BN;
  const int tiles_per_img = p.Hc / TH;
  const int strip = tile_m % p.strips, row_tile = tile_m / p.strips;   // (strips = 1: the tile spans the image width)
  const int img = row_tile / tiles_per_img;
  const int h0 = (row_tile - img * tiles_per_img) * TH;
  const int w0 = strip * W;
  const int Hin = p.Hc >> p.up, Win = p.Wc >> p.up;
  const __amdgpu_buffer_rsrc_t rX = make_rsrc(p.x, p.x_bytes);
  const __amdgpu_buffer_rsrc_t rW = make_rsrc(p.w, p.w_bytes);

  // patch loader: slot q = pass*256 + tid of the linear patch buffer
  unsigned a_off[PASSES];
#pragma unroll
  for (int i = 0; i < PASSES; ++i) {
    const int q = i * 256 + tid;
    const int cell = q >> 2;
    const int chunk = (q & 3) ^ ((cell >> 2) & 3);
    const int pr = cell / PW, pc = cell - pr * PW;
    const int hh = h0 - 1 + pr, ww = w0 + pc - 1;
    const bool ok = cell < PC && hh >= 0 && hh < p.Hc && ww >= 0 && ww < p.Wc;
    const unsigned pix = ((unsigned)img * (unsigned)Hin + (unsigned)(hh >> p.up)) * (unsigned)Win + (unsigned)(ww >> p.up);
    a_off[i] = ok ? pix * (unsigned)(p.Cin * ES) + (unsigned)chunk * 16u : kOob;
  }
  // weight operands: one KiB block per 32 columns and K-step, this lane's 16 bytes of it
  const unsigned kb32 = (unsigned)(p.K * ES) >> 5;
  unsigned wv[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) wv[j] = ((((unsigned)(n0 + wn * WN)) >> 5) + (unsigned)j) * kb32 * 1024u + (unsigned)lane * 16u;
  // fragment geometry
  const int frag_row = lane & 31, fc = lane >> 5;
  unsigned cell0[MI];                           // patch cell of this lane's pixel for tap (0,0)
#pragma unroll
  for (int i = 0; i < MI; ++i) {
    const int ml = wm * WM + i * 32 + frag_row;
    cell0[i] = (unsigned)((ml / W) * PW + (ml % W));
  }
  const unsigned lds_p = (unsigned)(size_t)(lds_char*)sP;

  floatx16 acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  const int NC = (p.Cin * ES) / BKB;            // channel slabs
  const unsigned tap_bytes = (unsigned)(p.Cin * ES);
#define PATCH_DMA(BUF, PASS, CBYTE) dma_load16(rX, sP + (BUF) * PATCH_BYTES + (PASS) * 4096 + wave * 1024, a_off[PASS] + (CBYTE))
#define WFRAG_LOAD(STG, KBYTE)                                                                               \
  {                                                                                                          \
    const unsigned so = ((KBYTE) >> 5) << 10;                                                                \
    _Pragma("unroll") for (int j = 0; j < NJ; ++j) {                                                         \
      bq[STG][0][j] = __builtin_amdgcn_raw_buffer_load_b128(rW, wv[j], so, 0);                               \
      bq[STG][1][j] = __builtin_amdgcn_raw_buffer_load_b128(rW, wv[j], so + 1024u, 0);                       \
    }                                                                                                        \
  }
  // Patch fragment registers: set 0 holds K-step 0 of the current tap (read during the previous step), set 1
  // K-step 1 (read at the start of the step, behind the MFMAs of K-step 0); while the MFMAs of K-step 1 run,
  // set 0 is refilled for the next tap.  The waits for the weight registers are the compiler's.
  uint4v f0a[MI], f1a[MI];
  uint4v bq[3][2][NJ];
#define CONV3_ADDR(AA, CELLS, TAPV)                                                                          \
  _Pragma("unroll") for (int i = 0; i < MI; ++i) {                                                           \
    const unsigned cell = CELLS[i] + (unsigned)(((TAPV) / 3) * PW + (TAPV) % 3);                             \
    AA[i] = lds_p + (cell << 6) + ((((unsigned)fc) ^ ((cell >> 2) & 3u)) << 4);                              \
  }
  // prologue: the first patch, the weights of steps 0 and 1; fragments of (slab 0, tap 0, K-step 0)
#pragma unroll
  for (int i = 0; i < PASSES; ++i) PATCH_DMA(0, i, 0u);
  WFRAG_LOAD(0, 0u);
  WFRAG_LOAD(1, tap_bytes);
  __builtin_amdgcn_s_waitcnt(vm_imm(0));
  __builtin_amdgcn_s_barrier();
  {
    unsigned aa[MI];
    CONV3_ADDR(aa, cell0, 0)
    Conv3Reads<0, MI>::run(f0a, aa, 0u);
  }

  // One step: tap TAP of channel slab c.  `last` = this is the last channel slab.
#define CONV3_STEP(TAP)                                                                                      \
  {                                                                                                          \
    if ((TAP) == 8 && !last) {                                                                               \
      __builtin_amdgcn_s_waitcnt(vm_imm(2 * NJ));   /* (only the weights tap 7 asked for may be outstanding) */ \
      __builtin_amdgcn_s_barrier();                                                                          \
    }                                                                                                        \
    if ((TAP) == 0 && c > 0) __builtin_amdgcn_s_barrier();                                                   \
    if (!last) {                                                                                             \
      _Pragma("unroll") for (int q = 0; q < passes_at(PASSES, (TAP)); ++q)                                   \
          PATCH_DMA(nbuf, passes_before(PASSES, (TAP)) + q, cbyte + (unsigned)BKB);                          \
    }                                                                                                        \
    if (!last || (TAP) < 7)                                                                                  \
      WFRAG_LOAD(((TAP) + 2) % 3, (unsigned)(((TAP) + 2) % 9) * tap_bytes + cbyte + ((TAP) >= 7 ? (unsigned)BKB : 0u)) \
    {                                                                                                        \
      unsigned aa[MI];                                                                                       \
      CONV3_ADDR(aa, cellb, (TAP))                                                                           \
      Conv3Reads<0, MI>::run(f1a, aa, 32u);                                                                  \
    }                                                                                                        \
    lds_wait_tie_a<MI, MI>(f0a);                                                                             \
    mma_group<T, MI, NJ>(f0a, bq[(TAP) % 3][0], acc);                                                        \
    __builtin_amdgcn_sched_barrier(0);                                                                       \
    lds_wait_tie_a<0, MI>(f1a);                                                                              \
    if (!(last && (TAP) == 8)) {                                                                             \
      unsigned aa[MI];                                                                                       \
      if ((TAP) == 8) { CONV3_ADDR(aa, celln, 0) } else { CONV3_ADDR(aa, cellb, ((TAP) + 1) % 9) }           \
      Conv3Reads<0, MI>::run(f0a, aa, 0u);                                                                   \
    }                                                                                                        \
    __builtin_amdgcn_sched_barrier(0);                                                                       \
    mma_group<T, MI, NJ>(f1a, bq[(TAP) % 3][1], acc);                                                        \
    __builtin_amdgcn_sched_barrier(0);                                                                       \
  }
  // (the last slab is a copy of its own with `last` a constant: where one body served both, the compiler's wait
  // for a weight register had to assume the fewer loads in flight of the last slab, and stalled every other slab's
  // taps 7 and 8 on loads issued a moment before)
#define CONV3_SLAB(LASTV)                                                                                    \
  {                                                                                                          \
    constexpr bool last = LASTV;                                                                             \
    const int nbuf = (c + 1) & 1;                                                                            \
    unsigned cellb[MI], celln[MI];               /* (the buffer offset is a multiple of 4 cells: same swizzle bits) */ \
    _Pragma("unroll") for (int i = 0; i < MI; ++i) {                                                         \
      cellb[i] = cell0[i] + (unsigned)((c & 1) * (PATCH_BYTES / 64));                                        \
      celln[i] = cell0[i] + (unsigned)(nbuf * (PATCH_BYTES / 64));                                           \
    }                                                                                                        \
    const unsigned cbyte = (unsigned)(c * BKB);                                                              \
    CONV3_STEP(0) CONV3_STEP(1) CONV3_STEP(2) CONV3_STEP(3) CONV3_STEP(4)                                    \
    CONV3_STEP(5) CONV3_STEP(6) CONV3_STEP(7) CONV3_STEP(8)                                                  \
  }
  int c = 0;
  for (; c + 1 < NC; ++c) CONV3_SLAB(false)
  CONV3_SLAB(true)
#undef CONV3_SLAB
#undef CONV3_STEP
#undef CONV3_ADDR
#undef WFRAG_LOAD
#undef PATCH_DMA
  __syncthreads();                               // every wave is done with the operands: the epilogue reuses the memory
  igemm_epilogue<T, BM, BN, WGM, WGN, INTERIOR, EPI>(acc, p, smem, sRed, m0, n0, (int64_t)tile_m);
}

struct IgemmTile { int bm, bn, bkb; };

// Largest tile that still gives every compute unit about two workgroups.
IgemmTile pick_tile(int64_t M, int cout, int cin, int es, bool wide = true, int min_wide_tiles = 256) {
  // large dense bf16 products whose 256 x 256 tiles all lie inside the output and still fill the chip: eight
  // wavefronts per workgroup, a third fewer operand bytes through LDS per multiply-add than 256 x 128
  if (wide && es == 2 && cout % 256 == 0 && M % 256 == 0 && (M / 256) * (cout / 256) >= min_wide_tiles) return IgemmTile{256, 256, 64};
  const int bn = cout > 64 ? 128 : 64;
  const int64_t tiles_n = (cout + bn - 1) / bn;
  int bm = es == 2 ? 256 : 128;                 // 256-row tiles: bf16 only (register budget)
  if (((M + 255) / 256) * tiles_n < 512) bm = 128;
  (void)cin;
  const int bkb = 64;                           // three LDS stages of 64-byte slabs: 2-3 workgroups per compute unit
  return IgemmTile{bm, bn, bkb};
}

}  // namespace

// The GEMM behind the two forms of an upsampled convolution: rows are pixels of the STORED
// (half-size) grid, 2x2 taps per phase or 4x4 taps with stride 2.
static ConvArgs conv_effective(const ConvArgs& a) {
  ConvArgs e = a;
  if (a.geom == CONV_PLAIN) return e;
  e.hc = a.hc / 2; e.wc = a.wc / 2; e.up = 0;
  e.k = a.geom == CONV_UP_PHASES ? 2 : 4;
  e.geom = CONV_PLAIN;                      // (applying this twice must not halve twice)
  return e;
}

bool conv_mfma_supported(const ConvArgs& a0) {
  const ConvArgs a = conv_effective(a0);
  const int es = (int)dtype_size(a.dtype);
  if ((a.cin * es) % 64 != 0 || a.cout < 32) return false;
  const int64_t M = (int64_t)a.n * a.hc * a.wc;
  const int64_t x_bytes = a0.geom == CONV_UP_DGRAD ? (int64_t)a0.n * a0.hc * a0.wc * a.cin * es
                                                   : (int64_t)a.n * (a.hc >> a.up) * (a.wc >> a.up) * a.cin * es;
  const int64_t w_bytes = (int64_t)a.cout * a.k * a.k * a.cin * es * (a0.geom == CONV_UP_PHASES ? 4 : 1);
  if (x_bytes >= 0x7FFFFFFF || w_bytes >= 0x7FFFFFFF) return false;   // 32-bit buffer offsets
  return M * ((a.cout + 63) / 64) / 128 < 0x7FFFFFFF && M < 0x7FFFFFFF;
}

// The patch kernel takes 3x3 convolutions whose image width is 16..128 (a power of two), whose
// tiles of 256/W rows divide the image height, with enough tiles to fill the chip, and whose
// epilogue needs no run-time checks.
// column width of the patch kernel's tiles
static int conv3_patch_bn(const ConvArgs& a) { return a.cout % 128 == 0 ? 128 : 64; }
static bool conv3_patch_usable(const ConvArgs& a) {
  if (a.geom != CONV_PLAIN || a.k != 3 || !conv_mfma_supported(a)) return false;
  // (a 128-pixel-wide tile would need 96 KB of LDS, one workgroup per compute unit: wider images are cut into column
  // strips of 64 pixels instead, whose halo columns come from the neighbouring strip)
  if (a.wc != 16 && a.wc != 32 && a.wc != 64 && a.wc != 128 && a.wc != 256) return false;
  // (measured on the 128 x 128 layers of the largest workload against the per-tap kernel: 93 against 109 us with four
  // channel slabs, 109 against 131 us with two)
  const int th = 256 / (a.wc > 64 ? 64 : a.wc);
  if (a.hc % th != 0 || a.cout % 64 != 0) return false;
  const int bn = conv3_patch_bn(a);
  const int64_t tiles = ((int64_t)a.n * a.hc * a.wc / 256) * (a.cout / bn);
  if (tiles < 256) return false;
  return !a.y_aux && a.act != ACT_SIGMOID && !(a.partial && a.act != ACT_NONE);
}

int conv_partial_rows(const ConvArgs& a, bool mfma) {
  if (!mfma) return kReduceRows;
  if (conv3_patch_usable(a)) return 256;
  return pick_tile((int64_t)a.n * a.hc * a.wc, a.cout, a.cin, (int)dtype_size(a.dtype)).bm;
}

// Split-K: layers with fewer than 128 output tiles (small batch x fully-connected) and a long K.
static int conv_mfma_splits(const ConvArgs& a0) {
  if (a0.partial || a0.epi != CONV_EPI_NONE || a0.geom == CONV_UP_PHASES || !conv_mfma_supported(a0) || conv3_patch_usable(a0)) return 1;
  const ConvArgs a = conv_effective(a0);
  const int es = (int)dtype_size(a.dtype);
  const int64_t M = (int64_t)a.n * a.hc * a.wc;
  const IgemmTile t = pick_tile(M, a.cout, a.cin, es, a0.tri == 0);
  const int64_t tiles = ((M + t.bm - 1) / t.bm) * ((a.cout + t.bn - 1) / t.bn);
  const int64_t KT = (int64_t)a.k * a.k * a.cin * es / t.bkb;
  if (tiles >= 256 || KT < 16) return 1;          // one workgroup per compute unit or more: no split
  int64_t splits = (512 + tiles - 1) / tiles;
  if (splits > KT / 4) splits = KT / 4;
  return splits < 1 ? 1 : (int)splits;
}

int64_t conv_mfma_splitk_floats(const ConvArgs& a0) {
  const int splits = conv_mfma_splits(a0);
  const ConvArgs a = conv_effective(a0);
  return splits > 1 ? (int64_t)splits * a.n * a.hc * a.wc * a.cout : 0;
}

// Four 2x2 phase convolutions: the kernel's epilogue without run-time checks only, and
// enough workgroups without splitting K.
bool conv_up_phases_usable(const ConvArgs& a0) {
  if (a0.up != 1 || a0.k != 3 || (a0.hc & 1) || (a0.wc & 1)) return false;
  ConvArgs a = a0;
  a.geom = CONV_UP_PHASES;
  if (!conv_mfma_supported(a)) return false;
  if (a.partial || a.y_aux || a.act == ACT_SIGMOID) return false;
  const ConvArgs e = conv_effective(a);
  const int64_t M = (int64_t)e.n * e.hc * e.wc;
  const IgemmTile t = pick_tile(M, e.cout, e.cin, (int)dtype_size(e.dtype));
  if (M % t.bm != 0 || e.cout % t.bn != 0) return false;
  return (M / t.bm) * (e.cout / t.bn) * 4 >= 256;
}

// The special epilogues: 1x1 layers, check-free tiles of the shapes they are instantiated for, no split-K.
bool conv_epi_usable(const ConvArgs& a) {
  if (a.epi == CONV_EPI_NONE) return true;
  if (a.geom != CONV_PLAIN || a.k != 1 || a.up != 0 || a.hc != 1 || a.wc != 1 || !conv_mfma_supported(a)) return false;
  if (a.y_aux || a.act != ACT_NONE || a.cout % 128 != 0) return false;
  if (a.epi == CONV_EPI_RESID && (!a.partial || !a.resid)) return false;
  if (a.epi == CONV_EPI_MXQ && a.partial) return false;
  if (a.epi == CONV_EPI_MXQ) {
    const int epc = 16 / (int)dtype_size(a.dtype);
    if (a.mx_block < epc || a.mx_block > 64 || (a.mx_block & (a.mx_block - 1)) != 0) return false;
    if (a.mx_elem != MX_FP4 && a.mx_elem != MX_INT4 && a.mx_elem != MX_FP8) return false;
  }
  const IgemmTile t = pick_tile(a.n, a.cout, a.cin, (int)dtype_size(a.dtype));
  return (t.bn == 128 || t.bn == 256) && a.n % t.bm == 0;
}

bool conv_up_dgrad_usable(const ConvArgs& a0) {
  if (a0.k != 3 || a0.up != 0 || (a0.hc & 1) || (a0.wc & 1) || a0.partial || a0.y_aux || a0.bias || a0.act != ACT_NONE) return false;
  ConvArgs a = a0;
  a.geom = CONV_UP_DGRAD;
  return conv_mfma_supported(a);
}

// Number of row blocks whose column sums a launch with a companion tensor (ConvArgs::comp) leaves in `partial`, or 0
// if this launch cannot take one: the epilogue exists for bfloat16 launches whose tiles all lie inside the output,
// without split-K and without an epilogue variant of their own.
int conv_comp_blocks(const ConvArgs& a0) {
  if (a0.dtype != AE_BF16 || !conv_mfma_supported(a0) || a0.epi != CONV_EPI_NONE || a0.tri != 0 || a0.geom == CONV_UP_PHASES ||
      a0.y_aux || a0.act != ACT_NONE || a0.bias)
    return 0;
  const ConvArgs a = conv_effective(a0);
  const int64_t M = (int64_t)a.n * a.hc * a.wc;
  if (conv3_patch_usable(a0)) return (int)(M / 256);
  const IgemmTile t = pick_tile(M, a.cout, a.cin, 2, a0.geom == CONV_PLAIN, 256);
  if (t.bn == 256 || M % t.bm != 0 || a.cout % t.bn != 0) return 0;
  ConvArgs probe = a0;
  probe.partial = reinterpret_cast<float*>(1);     // only null / non-null matters: statistics keep K in one piece
  if (conv_mfma_splits(probe) != 1) return 0;
  return (int)(M / t.bm);
}

bool conv_weights_frag_order(const ConvArgs& a) { return conv3_patch_usable(a); }

int launch_conv_mfma(const ConvArgs& a0, hipStream_t s) {
  if (!conv_mfma_supported(a0)) return fail(AE_EINVAL, "conv_mfma: shape not supported");
  if (a0.w_frag != conv3_patch_usable(a0)) return fail(AE_EINVAL, "conv_mfma: the order of the packed weights does not fit the kernel of this launch (conv_weights_frag_order)");
  if (a0.geom == CONV_UP_PHASES && !conv_up_phases_usable(a0)) return fail(AE_EINVAL, "conv_mfma: phase form not usable here");
  if (!conv_epi_usable(a0)) return fail(AE_EINVAL, "conv_mfma: epilogue variant not usable for this shape");
  const ConvArgs a = conv_effective(a0);
  const int es = (int)dtype_size(a.dtype);
  IgemmParams p;
  p.x = a.x; p.w = a.w; p.bias = a.bias; p.y = a.y; p.y_aux = a.y_aux; p.partial = a.partial;
  p.M = (int64_t)a.n * a.hc * a.wc;
  p.N = a.cout; p.K = a.k * a.k * a.cin;
  p.Hc = a.hc; p.Wc = a.wc; p.Cin = a.cin; p.ksz = a.k; p.up = a.up; p.act = a.act;
  p.Hv = a.hc; p.Wv = a.wc; p.stride = 1; p.pad = (a.k - 1) >> 1; p.phases = 1;
  if ((a.hc & (a.hc - 1)) == 0 && (a.wc & (a.wc - 1)) == 0) {
    p.log_w = p.log_h = 0;
    while ((1 << p.log_w) < a.wc) ++p.log_w;
    while ((1 << p.log_h) < a.hc) ++p.log_h;
  }
  p.resid = a0.resid;
  p.comp = a0.comp; p.comp_mode = a0.comp_mode; p.comp_bn = a0.comp_bn;
  if (a0.comp_mode != 0) {
    if (a0.comp_mode < 1 || a0.comp_mode > 2 || !a0.comp || !a0.partial || (a0.comp_mode == 2 && !a0.comp_bn) ||
        conv_comp_blocks(a0) == 0)
      return fail(AE_EINVAL, "conv_mfma: companion-tensor epilogue not usable for this launch");
  }
  p.mx_block = a0.mx_block;
  p.mx_elem = a0.mx_elem;
  p.tri = a0.tri;
  p.tri_b = a0.tri_b;
  p.tri_d = a0.tri >= 8 ? a0.tri_d : 0;
  if (a0.tri >= 8 && (a0.tri > 9 || a.dtype != AE_F32 || a0.tri_b < 128 || a0.tri_b % 128 != 0 || a.n % (2 * a0.tri_b) != 0 ||
                      a0.tri_d < 0 || a0.tri_d > a.n || a0.tri_d % 128 != 0))
    return fail(AE_EINVAL, "conv_mfma: bad block size for the blocked triangular inverse");
  if (a0.tri != 0 && (a0.tri < 0 || (a0.tri > 4 && a0.tri < 8) || a0.tri > 9 || a.k != 1 || a.hc != 1 || a.wc != 1 || a.up != 0 || a.n != a.cout || a.cin != a.cout ||
                      a0.epi != CONV_EPI_NONE || a.partial))
    return fail(AE_EINVAL, "conv_mfma: triangular K ranges are for square dense products only");
  p.x_bytes = (unsigned)((int64_t)a.n * (a.hc >> a.up) * (a.wc >> a.up) * a.cin * es);
  p.w_bytes = (unsigned)((int64_t)a.cout * a.k * a.k * a.cin * es);
  if (a0.geom == CONV_UP_PHASES) {
    p.pad = 1; p.phases = 4;
    p.w_bytes *= 4u;
  } else if (a0.geom == CONV_UP_DGRAD) {
    p.Hv = a0.hc; p.Wv = a0.wc; p.stride = 2; p.pad = 1;
    p.x_bytes = (unsigned)((int64_t)a0.n * a0.hc * a0.wc * a.cin * es);
  }
  if (conv3_patch_usable(a0)) {
    const int bn = conv3_patch_bn(a);
    p.tiles_n = a.cout / bn;
    p.strips = a.wc > 64 ? a.wc / 64 : 1;
    p.log_wt = 6;                                // strips of 64 pixels
    dim3 pgrid((unsigned)((p.M / 256) * p.tiles_n));
#define PATCH_LAUNCH_E(T, WV, E)                                                                             \
  do {                                                                                                      \
    if (bn == 128) hipLaunchKernelGGL((k_conv3_patch<T, 128, 2, 2, WV, true, E>), pgrid, dim3(256), 0, s, p); \
    else hipLaunchKernelGGL((k_conv3_patch<T, 64, 4, 1, WV, true, E>), pgrid, dim3(256), 0, s, p);           \
  } while (0)
#define PATCH_LAUNCH_W(T, WV) PATCH_LAUNCH_E(T, WV, 0)
    if (a0.comp_mode != 0) {            // (conv_comp_blocks: bfloat16 only)
      if (a0.comp_mode == 1) { if (a.wc == 16) PATCH_LAUNCH_E(bf16_t, 16, 3); else if (a.wc == 32) PATCH_LAUNCH_E(bf16_t, 32, 3); else PATCH_LAUNCH_E(bf16_t, 64, 3); }
      else { if (a.wc == 16) PATCH_LAUNCH_E(bf16_t, 16, 4); else if (a.wc == 32) PATCH_LAUNCH_E(bf16_t, 32, 4); else PATCH_LAUNCH_E(bf16_t, 64, 4); }
      return launch_status("conv3_patch");
    }
#define PATCH_LAUNCH(T)                                     \
  do {                                                      \
    if (a.wc == 16) PATCH_LAUNCH_W(T, 16);                  \
    else if (a.wc == 32) PATCH_LAUNCH_W(T, 32);             \
    else PATCH_LAUNCH_W(T, 64);                             \
  } while (0)
    if (a.dtype == AE_BF16) PATCH_LAUNCH(bf16_t);
    else PATCH_LAUNCH(float);
#undef PATCH_LAUNCH
#undef PATCH_LAUNCH_W
#undef PATCH_LAUNCH_E
    return launch_status("conv3_patch");
  }
  // the wide tile exists without run-time checks only; tiles of very different K lengths (the triangular modes 1-3)
  // balance better when smaller unless there are at least four per compute unit (measured: d = 8192, not 4096)
  const bool wide_ok = (a0.tri == 0 || a0.tri <= 3) && !a.y_aux && a.act != ACT_SIGMOID && !(a.partial && a.act != ACT_NONE) && a0.geom == CONV_PLAIN;
  const IgemmTile t = pick_tile(p.M, a.cout, a.cin, es, wide_ok, a0.tri == 0 ? 256 : 1024);
  p.tiles_n = (a.cout + t.bn - 1) / t.bn;
  const int64_t tiles_m = (p.M + t.bm - 1) / t.bm;
  const int KT = (int)((int64_t)p.K * es / t.bkb);
  int splits = conv_mfma_splits(a0);
  if (splits > 1 && (!a.splitk_ws || (int64_t)splits * p.M * p.N > a.splitk_floats)) splits = 1;
  if (a0.tri != 0) splits = 1;
  p.tiles_mn = (int)(tiles_m * p.tiles_n);
  p.slabs_per_split = (KT + splits - 1) / splits;
  splits = (KT + p.slabs_per_split - 1) / p.slabs_per_split;
  p.split_out = splits > 1 ? a.splitk_ws : nullptr;
  dim3 grid((unsigned)(tiles_m * p.tiles_n * splits * p.phases));
  if (a0.tri >= 8) {
    const int64_t all_pairs = p.M / (2 * a0.tri_b);
    const int64_t pairs = a0.tri_pairs > 0 && a0.tri_pairs < all_pairs ? a0.tri_pairs : all_pairs;
    grid = dim3((unsigned)(pairs * (a0.tri_b / t.bm) * (a0.tri_b / t.bn)));
  }
  const bool interior = splits == 1 && p.M % t.bm == 0 && p.N % t.bn == 0 && !a.y_aux && a.act != ACT_SIGMOID &&
                        !(a.partial && a.act != ACT_NONE);
#define IGEMM_LAUNCH_K(T, BMV, BNV, GM, GN, KB)                                                        \
  do {                                                                                                 \
    if (interior) hipLaunchKernelGGL((k_igemm<T, BMV, BNV, GM, GN, KB, true, true>), grid, dim3(256), 0, s, p); \
    else hipLaunchKernelGGL((k_igemm<T, BMV, BNV, GM, GN, KB, false, true>), grid, dim3(256), 0, s, p); \
  } while (0)
#define IGEMM_LAUNCH_T(T, BMV, BNV, GM, GN) IGEMM_LAUNCH_K(T, BMV, BNV, GM, GN, 64)   /* pick_tile: 64-byte slabs only */
#define IGEMM_LAUNCH(BMV, BNV, GM, GN)                                         \
  do {                                                                         \
    if (a.dtype == AE_BF16) IGEMM_LAUNCH_T(bf16_t, BMV, BNV, GM, GN);          \
    else IGEMM_LAUNCH_T(float, BMV, BNV, GM, GN);                              \
  } while (0)
  if (a0.comp_mode != 0) {
    // (conv_comp_blocks: bfloat16, interior tiles, no split, not the eight-wavefront tile)
#define IGEMM_LAUNCH_COMP(BMV, BNV, GM, GN)                                                                           \
  do {                                                                                                                \
    if (a0.comp_mode == 1) hipLaunchKernelGGL((k_igemm<bf16_t, BMV, BNV, GM, GN, 64, true, true, 3>), grid, dim3(256), 0, s, p); \
    else hipLaunchKernelGGL((k_igemm<bf16_t, BMV, BNV, GM, GN, 64, true, true, 4>), grid, dim3(256), 0, s, p);         \
  } while (0)
    if (t.bm == 256 && t.bn == 128) IGEMM_LAUNCH_COMP(256, 128, 2, 2);
    else if (t.bm == 256) IGEMM_LAUNCH_COMP(256, 64, 4, 1);
    else if (t.bn == 128) IGEMM_LAUNCH_COMP(128, 128, 2, 2);
    else IGEMM_LAUNCH_COMP(128, 64, 2, 2);
#undef IGEMM_LAUNCH_COMP
    return launch_status("conv_mfma_comp");
  }
  if (a0.epi != CONV_EPI_NONE) {
    // (conv_epi_usable: interior tiles, BN = 128, no split)
#define IGEMM_LAUNCH_EPI(T, BMV, E) hipLaunchKernelGGL((k_igemm<T, BMV, 128, 2, 2, 64, true, true, E>), grid, dim3(256), 0, s, p)
    if (t.bn == 256) {
      if (a0.epi == CONV_EPI_MXQ) hipLaunchKernelGGL((k_igemm<bf16_t, 256, 256, 2, 4, 64, true, true, 1>), grid, dim3(512), 0, s, p);
      else hipLaunchKernelGGL((k_igemm<bf16_t, 256, 256, 2, 4, 64, true, true, 2>), grid, dim3(512), 0, s, p);
    } else if (a.dtype == AE_BF16) {
      if (t.bm == 256) { if (a0.epi == CONV_EPI_MXQ) IGEMM_LAUNCH_EPI(bf16_t, 256, 1); else IGEMM_LAUNCH_EPI(bf16_t, 256, 2); }
      else { if (a0.epi == CONV_EPI_MXQ) IGEMM_LAUNCH_EPI(bf16_t, 128, 1); else IGEMM_LAUNCH_EPI(bf16_t, 128, 2); }
    } else {
      if (a0.epi == CONV_EPI_MXQ) IGEMM_LAUNCH_EPI(float, 128, 1); else IGEMM_LAUNCH_EPI(float, 128, 2);
    }
#undef IGEMM_LAUNCH_EPI
    return launch_status("conv_mfma_epi");
  }
  if (t.bn == 256) hipLaunchKernelGGL((k_igemm<bf16_t, 256, 256, 2, 4, 64, true, true>), grid, dim3(512), 0, s, p);   // (pick_tile: interior only)
  else if (t.bm == 256 && t.bn == 128) IGEMM_LAUNCH_K(bf16_t, 256, 128, 2, 2, 64);
  else if (t.bm == 256) IGEMM_LAUNCH_K(bf16_t, 256, 64, 4, 1, 64);
  else if (t.bn == 128) IGEMM_LAUNCH(128, 128, 2, 2);
  else IGEMM_LAUNCH(128, 64, 2, 2);
#undef IGEMM_LAUNCH_K
#undef IGEMM_LAUNCH
#undef IGEMM_LAUNCH_T
  AE_TRY(launch_status("conv_mfma"));
  if (splits > 1) {
    int64_t g = (p.M * p.N + 255) / 256;
    if (g > 8192) g = 8192;
    if (a.dtype == AE_BF16)
      hipLaunchKernelGGL((k_splitk_finish<bf16_t>), dim3((unsigned)g), dim3(256), 0, s, a.splitk_ws, splits, p.M, p.N, a.bias,
                         a.act, (bf16_t*)a.y, a.y_aux);
    else
      hipLaunchKernelGGL((k_splitk_finish<float>), dim3((unsigned)g), dim3(256), 0, s, a.splitk_ws, splits, p.M, p.N, a.bias,
                         a.act, (float*)a.y, a.y_aux);
    return launch_status("splitk_finish");
  }
  return AE_OK;
}

}  // namespace ae

// ===========================================================================
// Weight gradient on the matrix cores (bf16).
//
//   dW[co][(r,s,ci)] = sum over pixels m of dY[m][co] * Xg[m][(r,s,ci)]
// where Xg is the gathered input of tap (r,s).  Both operands are stored with the
// reduction index (the pixel) outermost, so the MFMA operands (8 consecutive pixels
// of one channel per lane) are transposes of what memory holds.  The slabs go to
// LDS exactly as loaded, [pixel][channel], and are read back with the gfx950 LDS
// transpose load (ds_read_b64_tr_b16): within a group of 16 lanes, the lane with
// local index 4*j+q supplies the address of 4 channels (4q..4q+3) of pixel j, and
// lane i receives channel i of pixels 0..3.
//
// A workgroup owns one output tile (BM output channels x BN input channels of one
// tap) and one contiguous range of pixels; partial tiles go to a workspace
// [split][C_out][k*k*C_in] (fp32) that a second kernel sums in a fixed order and
// writes in the canonical [C_out][C_in][k][k] layout, so the result is deterministic.
// ===========================================================================
namespace ae {
namespace {

typedef short short4v __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) short4v lds_short4v;

struct WgradParams {
  const void* x; const void* dy; float* partial;
  int64_t M;            // pixels
  int Cout, Cin, Hc, Wc, ksz, up;
  int tiles_m, tiles_n; // tiles over C_out and over C_in
  int rows_per_split;   // multiple of 32
  int K;                // k*k*C_in
  int log_w, log_h;     // log2 of Wc / Hc when both are powers of two (POW2 kernels)
  unsigned x_bytes, dy_bytes;
};

__device__ __forceinline__ bf16x8 lds_tr_frag(const bf16_t* base0, const bf16_t* base1) {
  // two transposing 64-bit loads: pixels p..p+3 and p+4..p+7 of this lane's channel
  short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4v*)base0);
  short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4v*)base1);
  union { short s[8]; bf16x8 v; } u;
  u.s[0] = lo[0]; u.s[1] = lo[1]; u.s[2] = lo[2]; u.s[3] = lo[3];
  u.s[4] = hi[0]; u.s[5] = hi[1]; u.s[6] = hi[2]; u.s[7] = hi[3];
  return u.v;
}

// One slab of MFMAs of the weight-gradient kernel.  sa / sb point at the wave's first
// channel of the [pixel][channel] slabs.
template <typename T, int MI, int NJ, int BK, int LA, int LB>
__device__ __forceinline__ void wgrad_compute(const T* sa, const T* sb, int lane, floatx16 (&acc)[MI][NJ]) {
  if constexpr (sizeof(T) == 2) {
    // transposing-load geometry of this lane: 16-lane group G covers channels 16*(G&1).. of
    // the 32-channel MFMA tile and pixels 8*(G>>1)..; local lane sl addresses pixel sl/4,
    // channels 4*(sl%4)..
    const int grp = lane >> 4, sl = lane & 15;
    const int t_pix = 8 * (grp >> 1) + (sl >> 2);
    const int t_ch = 16 * (grp & 1) + 4 * (sl & 3);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 a[MI], bb[NJ];
#pragma unroll
      for (int i = 0; i < MI; ++i) {
        const bf16_t* q = &sa[(ks * 16 + t_pix) * LA + i * 32 + t_ch];
        a[i] = lds_tr_frag(q, q + 4 * LA);
      }
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const bf16_t* q = &sb[(ks * 16 + t_pix) * LB + j * 32 + t_ch];
        bb[j] = lds_tr_frag(q, q + 4 * LB);
      }
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], bb[j], acc[i][j], 0, 0, 0);
    }
  } else {
    // fp32: lane l supplies channel l%32 of pixel 2*st + l/32 — a plain 4-byte read
    const int ch = lane & 31, half = lane >> 5;
#pragma unroll
    for (int st = 0; st < BK / 2; ++st) {
      float a[MI], bb[NJ];
#pragma unroll
      for (int i = 0; i < MI; ++i) a[i] = sa[(2 * st + half) * LA + i * 32 + ch];
#pragma unroll
      for (int j = 0; j < NJ; ++j) bb[j] = sb[(2 * st + half) * LB + j * 32 + ch];
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], bb[j], acc[i][j], 0, 0, 0);
    }
  }
}

template <typename T, int BM, int BN, bool POW2>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void k_wgrad(WgradParams p) {
  constexpr int ES = (int)sizeof(T);
  constexpr int EPC = 16 / ES;                   // elements per 16-byte chunk
  constexpr int BK = ES == 2 ? 32 : 16;          // pixels per slab
  // LDS row strides in elements (64 banks).  bf16: +64 bytes: 32 lanes of a transposing
  // load touch 4 pixel rows x 64 bytes, which then tile the 256-byte bank space; fp32:
  // +128 bytes, so that the two pixel rows a 64-lane 4-byte read touches are 32 banks apart.
  constexpr int LPAD = 32;
  constexpr int LA = BM + LPAD, LB = BN + LPAD;
  constexpr int WM = BM / 2, WN = BN / 2;
  constexpr int MI = WM / 32, NJ = WN / 32;
  constexpr int A_TPR = BM / EPC, B_TPR = BN / EPC;  // 16-byte chunks per pixel row
  constexpr int A_CHUNKS = BK * A_TPR / 256, B_CHUNKS = BK * B_TPR / 256;
  __shared__ __attribute__((aligned(16))) T sA[2][BK * LA];
  __shared__ __attribute__((aligned(16))) T sB[2][BK * LB];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  // block -> (split, tile_m, tile_n, tap): the tap varies fastest so that the blocks
  // sharing a dY slab and overlapping x slabs run at the same time
  const int taps = p.ksz * p.ksz;
  int b = xcd_logical_block((int)blockIdx.x, (int)gridDim.x);
  const int tap = b % taps; b /= taps;
  const int tn = b % p.tiles_n; b /= p.tiles_n;
  const int tm = b % p.tiles_m;
  const int split = b / p.tiles_m;
  const int r = tap / p.ksz, s = tap - r * p.ksz;
  const int pad = (p.ksz - 1) >> 1;
  const int co0 = tm * BM, ci0 = tn * BN;
  const int Hin = p.Hc >> p.up, Win = p.Wc >> p.up;
  const int64_t m_begin = (int64_t)split * p.rows_per_split;
  const int64_t m_end = (m_begin + p.rows_per_split < p.M) ? m_begin + p.rows_per_split : p.M;
  const int KT = (int)((m_end - m_begin + BK - 1) / BK);

  // Buffer loads: rows past the split's end and taps that fall into the zero padding get an
  // offset beyond the tensor and read as zero.  Pixel coordinates come from shifts when the
  // image sides are powers of two (POW2), from divisions otherwise.
  const __amdgpu_buffer_rsrc_t rX = make_rsrc(p.x, p.x_bytes);
  const __amdgpu_buffer_rsrc_t rDY = make_rsrc(p.dy, p.dy_bytes);
  const unsigned a_col = (unsigned)(co0 * ES);   // + chunk below
  const unsigned b_col = (unsigned)(ci0 * ES);
  int kload = 0;
#define WGRAD_LOAD(RA, RB)                                                                                   \
  {                                                                                                          \
    const int64_t mb = m_begin + (int64_t)kload * BK;                                                        \
    _Pragma("unroll") for (int i = 0; i < A_CHUNKS; ++i) {                                                   \
      const int id = tid + i * 256;                                                                          \
      const int64_t m = mb + id / A_TPR;                                                                     \
      const unsigned off = m < m_end ? (unsigned)m * (unsigned)(p.Cout * ES) + a_col + (unsigned)(id % A_TPR) * 16u : kOob; \
      RA[i] = __builtin_amdgcn_raw_buffer_load_b128(rDY, off, 0, 0);                                         \
    }                                                                                                        \
    _Pragma("unroll") for (int i = 0; i < B_CHUNKS; ++i) {                                                   \
      const int id = tid + i * 256;                                                                          \
      const int64_t m = mb + id / B_TPR;                                                                     \
      const unsigned mm = (unsigned)m;                                                                       \
      unsigned w, h, n;                                                                                      \
      if (POW2) {                                                                                            \
        w = mm & (unsigned)(p.Wc - 1); h = (mm >> p.log_w) & (unsigned)(p.Hc - 1); n = mm >> (p.log_w + p.log_h); \
      } else {                                                                                               \
        w = mm % (unsigned)p.Wc; const unsigned t = mm / (unsigned)p.Wc;                                     \
        h = t % (unsigned)p.Hc; n = t / (unsigned)p.Hc;                                                      \
      }                                                                                                      \
      const int hh = (int)h + r - pad, ww = (int)w + s - pad;                                                \
      const bool ok = m < m_end && hh >= 0 && hh < p.Hc && ww >= 0 && ww < p.Wc;                             \
      const unsigned pix = (n * (unsigned)Hin + (unsigned)(hh >> p.up)) * (unsigned)Win + (unsigned)(ww >> p.up); \
      const unsigned off = ok ? pix * (unsigned)(p.Cin * ES) + b_col + (unsigned)(id % B_TPR) * 16u : kOob;  \
      RB[i] = __builtin_amdgcn_raw_buffer_load_b128(rX, off, 0, 0);                                          \
    }                                                                                                        \
    ++kload;                                                                                                 \
  }
#define WGRAD_STORE(BUF, RA, RB)                                                                             \
  {                                                                                                          \
    _Pragma("unroll") for (int i = 0; i < A_CHUNKS; ++i) {                                                   \
      const int id = tid + i * 256;                                                                          \
      *reinterpret_cast<uint4v*>(&sA[BUF][(id / A_TPR) * LA + (id % A_TPR) * EPC]) = RA[i];                  \
    }                                                                                                        \
    _Pragma("unroll") for (int i = 0; i < B_CHUNKS; ++i) {                                                   \
      const int id = tid + i * 256;                                                                          \
      *reinterpret_cast<uint4v*>(&sB[BUF][(id / B_TPR) * LB + (id % B_TPR) * EPC]) = RB[i];                  \
    }                                                                                                        \
  }
#define WGRAD_COMPUTE(BUF) wgrad_compute<T, MI, NJ, BK, LA, LB>(&sA[BUF][wm * WM], &sB[BUF][wn * WN], lane, acc)

  floatx16 acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  // KT >= 1: every split owns at least one pixel (the host sizes the splits that way)
  uint4v ra0[A_CHUNKS], rb0[B_CHUNKS], ra1[A_CHUNKS], rb1[B_CHUNKS];
  WGRAD_LOAD(ra0, rb0);
  if (KT > 1) WGRAD_LOAD(ra1, rb1);
  WGRAD_STORE(0, ra0, rb0);
  __syncthreads();
  for (int kt = 0; kt < KT; kt += 2) {
    if (kt + 2 < KT) WGRAD_LOAD(ra0, rb0);
    WGRAD_COMPUTE(0);
    if (kt + 1 < KT) WGRAD_STORE(1, ra1, rb1);
    __syncthreads();
    if (kt + 1 >= KT) break;
    if (kt + 3 < KT) WGRAD_LOAD(ra1, rb1);
    WGRAD_COMPUTE(1);
    if (kt + 2 < KT) WGRAD_STORE(0, ra0, rb0);
    __syncthreads();
  }
#undef WGRAD_LOAD
#undef WGRAD_STORE
#undef WGRAD_COMPUTE

  // partial[split][co][tap*Cin + ci]
  float* __restrict__ P = p.partial + (int64_t)split * p.Cout * p.K;
  const int col_lane = lane & 31, row_lane = (lane >> 5) * 4;
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int ci = ci0 + wn * WN + j * 32 + col_lane;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int co = co0 + wm * WM + i * 32 + (e >> 2) * 8 + row_lane + (e & 3);
        if (co < p.Cout && ci < p.Cin) P[(int64_t)co * p.K + tap * p.Cin + ci] = acc[i][j][e];
      }
    }
}

// The same kernel for images whose width is a multiple of the slab depth BK: a slab is then BK
// consecutive pixels of ONE image row, so the sample, the row and the row's validity for the
// block's tap are uniform (scalar registers, advanced incrementally) and a thread's share of the
// address arithmetic is one add, one compare and one select per 16-byte load.  The output
// gradient advances through the scalar offset of the buffer load.  Every slab is full (the
// host makes the splits multiples of BK).
template <typename T, int BM, int BN, int BK>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void k_wgrad_rows(WgradParams p) {
  constexpr int ES = (int)sizeof(T);
  constexpr int EPC = 16 / ES;
  constexpr int LPAD = 32;
  constexpr int LA = BM + LPAD, LB = BN + LPAD;
  constexpr int WM = BM / 2, WN = BN / 2;
  constexpr int MI = WM / 32, NJ = WN / 32;
  constexpr int A_TPR = BM / EPC, B_TPR = BN / EPC;
  constexpr int A_CHUNKS = BK * A_TPR / 256, B_CHUNKS = BK * B_TPR / 256;
  static_assert(A_CHUNKS >= 1 && B_CHUNKS >= 1, "slab too small for 256 loader threads");
  __shared__ __attribute__((aligned(16))) T sA[2][BK * LA];
  __shared__ __attribute__((aligned(16))) T sB[2][BK * LB];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int taps = p.ksz * p.ksz;
  int b = xcd_logical_block((int)blockIdx.x, (int)gridDim.x);
  const int tap = b % taps; b /= taps;
  const int tn = b % p.tiles_n; b /= p.tiles_n;
  const int tm = b % p.tiles_m;
  const int split = b / p.tiles_m;
  const int r = tap / p.ksz, s = tap - r * p.ksz;
  const int pad = (p.ksz - 1) >> 1;
  const int co0 = tm * BM, ci0 = tn * BN;
  const int Hin = p.Hc >> p.up, Win = p.Wc >> p.up;
  const int64_t m_begin = (int64_t)split * p.rows_per_split;
  const int64_t m_end = (m_begin + p.rows_per_split < p.M) ? m_begin + p.rows_per_split : p.M;
  const int KT = (int)((m_end - m_begin) / BK);

  const __amdgpu_buffer_rsrc_t rX = make_rsrc(p.x, p.x_bytes);
  const __amdgpu_buffer_rsrc_t rDY = make_rsrc(p.dy, p.dy_bytes);
  unsigned a_voff[A_CHUNKS], b_voff[B_CHUNKS];
  int b_pw[B_CHUNKS];
#pragma unroll
  for (int i = 0; i < A_CHUNKS; ++i) {
    const int id = tid + i * 256;
    a_voff[i] = (unsigned)(id / A_TPR) * (unsigned)(p.Cout * ES) + (unsigned)(co0 * ES) + (unsigned)(id % A_TPR) * 16u;
  }
#pragma unroll
  for (int i = 0; i < B_CHUNKS; ++i) {
    const int id = tid + i * 256;
    b_pw[i] = id / B_TPR + s - pad;
    b_voff[i] = (unsigned)(ci0 * ES) + (unsigned)(id % B_TPR) * 16u;
  }
  // coordinates of the next slab to load (uniform)
  unsigned a_soff = (unsigned)m_begin * (unsigned)(p.Cout * ES);
  int w0 = (int)((unsigned)m_begin % (unsigned)p.Wc);
  int h = (int)(((unsigned)m_begin / (unsigned)p.Wc) % (unsigned)p.Hc);
  int n = (int)((unsigned)m_begin / ((unsigned)p.Wc * (unsigned)p.Hc));
  const unsigned cin_bytes = (unsigned)(p.Cin * ES);
#define WGRAD_LOAD(RA, RB)                                                                                   \
  {                                                                                                          \
    _Pragma("unroll") for (int i = 0; i < A_CHUNKS; ++i)                                                     \
        RA[i] = __builtin_amdgcn_raw_buffer_load_b128(rDY, a_voff[i], a_soff, 0);                            \
    const int hh = h + r - pad;                                                                              \
    const bool row_ok = hh >= 0 && hh < p.Hc;                                                                \
    const unsigned row_base = ((unsigned)n * (unsigned)Hin + (unsigned)((row_ok ? hh : 0) >> p.up)) * (unsigned)Win * cin_bytes; \
    _Pragma("unroll") for (int i = 0; i < B_CHUNKS; ++i) {                                                   \
      const int ww = w0 + b_pw[i];                                                                           \
      const bool ok = row_ok && (unsigned)ww < (unsigned)p.Wc;                                               \
      const unsigned off = ok ? row_base + (unsigned)(ww >> p.up) * cin_bytes + b_voff[i] : kOob;            \
      RB[i] = __builtin_amdgcn_raw_buffer_load_b128(rX, off, 0, 0);                                          \
    }                                                                                                        \
    a_soff += (unsigned)(BK * p.Cout * ES);                                                                  \
    w0 += BK;                                                                                                \
    if (w0 == p.Wc) { w0 = 0; if (++h == p.Hc) { h = 0; ++n; } }                                             \
  }
#define WGRAD_STORE(BUF, RA, RB)                                                                             \
  {                                                                                                          \
    _Pragma("unroll") for (int i = 0; i < A_CHUNKS; ++i) {                                                   \
      const int id = tid + i * 256;                                                                          \
      *reinterpret_cast<uint4v*>(&sA[BUF][(id / A_TPR) * LA + (id % A_TPR) * EPC]) = RA[i];                  \
    }                                                                                                        \
    _Pragma("unroll") for (int i = 0; i < B_CHUNKS; ++i) {                                                   \
      const int id = tid + i * 256;                                                                          \
      *reinterpret_cast<uint4v*>(&sB[BUF][(id / B_TPR) * LB + (id % B_TPR) * EPC]) = RB[i];                  \
    }                                                                                                        \
  }
#define WGRAD_COMPUTE(BUF) wgrad_compute<T, MI, NJ, BK, LA, LB>(&sA[BUF][wm * WM], &sB[BUF][wn * WN], lane, acc)

  floatx16 acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  uint4v ra0[A_CHUNKS], rb0[B_CHUNKS], ra1[A_CHUNKS], rb1[B_CHUNKS];
  WGRAD_LOAD(ra0, rb0);
  if (KT > 1) WGRAD_LOAD(ra1, rb1);
  WGRAD_STORE(0, ra0, rb0);
  __syncthreads();
  for (int kt = 0; kt < KT; kt += 2) {
    if (kt + 2 < KT) WGRAD_LOAD(ra0, rb0);
    WGRAD_COMPUTE(0);
    if (kt + 1 < KT) WGRAD_STORE(1, ra1, rb1);
    __syncthreads();
    if (kt + 1 >= KT) break;
    if (kt + 3 < KT) WGRAD_LOAD(ra1, rb1);
    WGRAD_COMPUTE(1);
    if (kt + 2 < KT) WGRAD_STORE(0, ra0, rb0);
    __syncthreads();
  }
#undef WGRAD_LOAD
#undef WGRAD_STORE
#undef WGRAD_COMPUTE

  float* __restrict__ P = p.partial + (int64_t)split * p.Cout * p.K;
  const int col_lane = lane & 31, row_lane = (lane >> 5) * 4;
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int ci = ci0 + wn * WN + j * 32 + col_lane;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int co = co0 + wm * WM + i * 32 + (e >> 2) * 8 + row_lane + (e & 3);
        P[(int64_t)co * p.K + tap * p.Cin + ci] = acc[i][j][e];   // tiles divide C_out and C_in exactly
      }
    }
}

// ---------------------------------------------------------------------------
// Weight gradient of a 3x3 convolution, three taps (one filter row r) per workgroup (bf16).
//
// With one tap per workgroup the slabs of dY and of the shifted input stream through the vector
// cache once per tap, and its 64 bytes per clock bound the kernel at about half the MFMA rate.
// Here a workgroup owns BM output channels x 64 input channels x the three taps (r, s = 0..2): per
// slab of 64 consecutive pixels it loads the dY slab once and ONE input patch — the slab's pixels
// of row h + r - 1 plus one pixel of halo on each side — from which the three taps are shifted
// views.  Slabs never straddle image rows (the host checks W % 64 == 0 or 64 % W == 0); a slab of
// a narrow image (W = SW < 64) is 64/SW whole rows, each with its own halo.
// LDS (three stages, filled by global-to-LDS loads): dY slab [64 px][BM] and patch
// [64/SW segments][SW + 4 cells][64 ci]; cell 1 of a segment is the left halo, cells 2..SW+1 the
// slab's pixels, cell SW+2 the right halo.  The 64-byte columns of a row are XOR-swizzled with
// the pixel / cell index such that the transposing reads (8 pixels x 64 bytes per instruction)
// spread evenly over the banks; for every fragment the swizzle is a per-lane constant, so all
// reads are base + immediate.  Schedule per slab: wait for the next slab's loads, barrier, issue
// the loads of the slab after that, then four K-steps of 16 pixels with the fragments of the
// next K-step (the first of the next slab included) in flight behind the MFMAs.
// ---------------------------------------------------------------------------
typedef unsigned uint2v __attribute__((ext_vector_type(2)));
struct TrFrag { uint2v lo, hi; };               // pixels 0..3 and 4..7 of a lane's channel

template <int OFF>
__device__ __forceinline__ void tr_read(TrFrag& f, unsigned addr, int row_bytes4 /* = 4 pixel rows */) {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(f.lo) : "v"(addr), "n"(OFF));
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(f.hi) : "v"(addr + (unsigned)row_bytes4), "n"(OFF));
#endif
}
// The patch operand of a K-step for all taps of a filter row at once: pixels 0..11 of a lane's channel, from the
// lane's cell on.  Tap s of pixel j reads cell j + s, so the operand of tap s is pixels s .. s+7 of this run: the taps
// are cut out of one 12-pixel read in registers (funnel shifts for the odd tap) instead of being read from LDS once
// each — three 8-byte reads per K-step instead of six, on the port that bounds this kernel.
struct TrRun { uint2v lo, hi, ex; };            // pixels 0..3, 4..7, 8..11
template <int OFF>
__device__ __forceinline__ void tr_read_run(TrRun& f, unsigned addr) {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(f.lo) : "v"(addr), "n"(OFF));
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(f.hi) : "v"(addr + 4u * 128u), "n"(OFF));
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(f.ex) : "v"(addr + 8u * 128u), "n"(OFF));
#endif
}
template <int NTAP>
__device__ __forceinline__ void tr_run_taps(TrRun& f, bf16x8 (&bv)[NTAP]) {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("" : "+v"(f.lo), "+v"(f.hi), "+v"(f.ex));
#endif
  const unsigned d0 = f.lo[0], d1 = f.lo[1], d2 = f.hi[0], d3 = f.hi[1], d4 = f.ex[0];
  union { unsigned w[4]; bf16x8 v; } u;
  u.w[0] = d0; u.w[1] = d1; u.w[2] = d2; u.w[3] = d3;
  bv[0] = u.v;
  if (NTAP > 1) {
    u.w[0] = __builtin_amdgcn_alignbit(d1, d0, 16); u.w[1] = __builtin_amdgcn_alignbit(d2, d1, 16);
    u.w[2] = __builtin_amdgcn_alignbit(d3, d2, 16); u.w[3] = __builtin_amdgcn_alignbit(d4, d3, 16);
    bv[1] = u.v;
  }
  if (NTAP > 2) {
    u.w[0] = d1; u.w[1] = d2; u.w[2] = d3; u.w[3] = d4;
    bv[NTAP > 2 ? 2 : 0] = u.v;
  }
}
__device__ __forceinline__ bf16x8 tr_value(TrFrag& f) {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("" : "+v"(f.lo), "+v"(f.hi));
#endif
  union { uint2v h[2]; bf16x8 v; } u;
  u.h[0] = f.lo; u.h[1] = f.hi;
  return u.v;
}

template <int BM, int SW>
struct Wgrad3 {
  static constexpr int BK = 64, SR = BK / SW, PCW = SW + 4, PCELLS = SR * PCW;
  static constexpr int RBA = BM * 2;            // bytes per pixel of the dY slab (256 or 128)
  static constexpr int A_BYTES = BK * RBA, A_PASSES = A_BYTES / 4096;
  static constexpr int X_UNITS = (PCELLS * 128 + 1023) / 1024;      // 1 KB = one wave-wide load
  static constexpr int XU = (X_UNITS + 3) / 4;   // units per wave
  static constexpr int STAGE = A_BYTES + X_UNITS * 1024;
  static constexpr int MI = BM / 64;            // 2x2 waves, wave tile (BM/2) x 32 per tap
  // K-step ks covers slab pixels 16*ks .. 16*ks+15: first cell (tap s = 0, before the +1+s) of the patch
  static constexpr int cell_base(int ks) { return ((ks * 16) / SW) * PCW + (ks * 16) % SW; }
};

// fragments of one K-step: MI of dY, the patch run that holds every tap (b_addr: the lane's address for tap 0)
template <int BM, int SW, int KS>
__device__ __forceinline__ void wgrad3_reads(TrFrag (&fa)[BM / 64], TrRun& fb, unsigned a_addr, unsigned b_addr) {
  typedef Wgrad3<BM, SW> G;
#pragma unroll
  for (int i = 0; i < G::MI; ++i) {
    // column i of the wave's co range: the swizzled column differs from a_addr's by (i << 6) XORed in
    if (i == 0) tr_read<KS * 16 * G::RBA>(fa[0], a_addr, 4 * G::RBA);
    else tr_read<KS * 16 * G::RBA>(fa[i], a_addr ^ 64u, 4 * G::RBA);
  }
  tr_read_run<G::cell_base(KS) * 128>(fb, b_addr);
}

// UP2: the convolution reads its input through a x2 nearest-neighbour upsample.  An output pixel (2i+a, 2j+b) then
// sees only 2 x 2 distinct stored pixels, (i + u - (1-a), j + v - (1-b)), u, v in {0,1}, and the nine taps fall onto
// them: r -> u = (a == 0 ? r > 0 : r > 1), s -> v likewise.  So the kernel forms, per output parity (a, b), the four
// correlations of that phase's quarter of dY with the shifted stored input — 16 tap matrices of a quarter of the
// pixels each, 4/9 of the multiply-adds — and k_wgrad_reduce_up2 adds, for every weight (r, s), the four phase
// matrices it belongs to (exact in real arithmetic; every product is of the same bf16 values as in the plain form).
// A workgroup owns (a, b, u) and the two taps v = 0, 1: a slab is 64 pixels of one phase (every other pixel of every
// other dY row, gathered by the global-to-LDS load), the patch is a row of the STORED image with its halo, and SW,
// Hc, Wc, M below are those of the stored image.
template <int BM, int SW, bool UP2>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void k_wgrad_row3(WgradParams p) {
  typedef Wgrad3<BM, SW> G;
  constexpr int MI = G::MI;
  constexpr int NTAP = UP2 ? 2 : 3;
  // (XOR address arithmetic below needs the alignment; 256 bytes of slack: the last pixels of a patch run may lie one
  // cell past the last stage's patch — they are read, never used)
  __shared__ __attribute__((aligned(1024))) char smem[3 * G::STAGE + 256];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  int b = xcd_logical_block((int)blockIdx.x, (int)gridDim.x);
  const int r = b % (UP2 ? 8 : 3); b /= (UP2 ? 8 : 3);      // UP2: r = (a, b, u) as three bits
  const int par_a = (r >> 2) & 1, par_b = (r >> 1) & 1, par_u = r & 1;
  const int tn = b % p.tiles_n; b /= p.tiles_n;
  const int tm = b % p.tiles_m;
  const int split = b / p.tiles_m;
  const int co0 = tm * BM, ci0 = tn * 64;
  const int Hin = UP2 ? p.Hc : (p.Hc >> p.up), Win = UP2 ? p.Wc : (p.Wc >> p.up);
  const int64_t m_begin = (int64_t)split * p.rows_per_split;
  const int64_t m_end = (m_begin + p.rows_per_split < p.M) ? m_begin + p.rows_per_split : p.M;
  const int KT = (int)((m_end - m_begin) / G::BK);
  const __amdgpu_buffer_rsrc_t rX = make_rsrc(p.x, p.x_bytes);
  const __amdgpu_buffer_rsrc_t rDY = make_rsrc(p.dy, p.dy_bytes);

  // ---- loaders.  dY: slot q = pass*256 + tid of the linear slab: pixel q / CPP, chunk q % CPP
  constexpr int CPP = G::RBA / 16;
  unsigned a_voff[G::A_PASSES];
#pragma unroll
  for (int i = 0; i < G::A_PASSES; ++i) {
    const int q = i * 256 + tid;
    const int px = q / CPP, chunk = q % CPP;
    const int sw = G::RBA == 256 ? (px & 3) : ((px >> 1) & 1);
    // UP2: slab pixel px = (segment row px / SW, column px % SW) of the stored image is dY pixel (2 row + a, 2 column + b)
    const unsigned dpx = UP2 ? (unsigned)((px / SW) * 2 * (2 * p.Wc) + (px % SW) * 2) : (unsigned)px;
    a_voff[i] = dpx * (unsigned)(p.Cout * 2) + (unsigned)(co0 * 2) + (unsigned)((chunk ^ (sw << 2)) * 16);
  }
  // patch: unit u = wave + 4*k of 1 KB: slot q = u*64 + lane: cell q / 8, chunk q % 8
  int x_seg[G::XU], x_pc[G::XU];
  unsigned x_chunk[G::XU];
  bool x_cell_ok[G::XU];
#pragma unroll
  for (int k = 0; k < G::XU; ++k) {
    const int q = (wave + 4 * k) * 64 + lane;
    const int cell = q >> 3;
    x_seg[k] = cell / G::PCW;
    x_pc[k] = cell - x_seg[k] * G::PCW;
    x_chunk[k] = (unsigned)(((q & 7) ^ (((cell >> 1) & 1) << 2)) * 16) + (unsigned)(ci0 * 2);
    x_cell_ok[k] = cell < G::PCELLS && x_pc[k] >= 1 && x_pc[k] <= SW + 2;
  }
  // coordinates of the next slab to load (uniform)
  unsigned a_soff = (unsigned)m_begin * (unsigned)(p.Cout * 2);     // (UP2: recomputed from (n, h, w0) per slab)
  int w0 = (int)((unsigned)m_begin % (unsigned)p.Wc);
  int h = (int)(((unsigned)m_begin / (unsigned)p.Wc) % (unsigned)p.Hc);
  int n = (int)((unsigned)m_begin / ((unsigned)p.Wc * (unsigned)p.Hc));
  const unsigned cin_bytes = (unsigned)(p.Cin * 2);
#define WGRAD3_DMA(STG)                                                                                      \
  {                                                                                                          \
    char* const da = smem + (STG) * G::STAGE + wave * 1024;                                                  \
    if (UP2) a_soff = (((unsigned)n * (unsigned)(2 * p.Hc) + (unsigned)(2 * h + par_a)) * (unsigned)(2 * p.Wc) + (unsigned)(2 * w0 + par_b)) * (unsigned)(p.Cout * 2); \
    _Pragma("unroll") for (int i = 0; i < G::A_PASSES; ++i)                                                  \
        dma_load16s(rDY, da + i * 4096, a_voff[i], a_soff);                                                  \
    _Pragma("unroll") for (int k = 0; k < G::XU; ++k) {                                                      \
      if (wave + 4 * k < G::X_UNITS) {                                                                       \
        const int row = h + x_seg[k] + (UP2 ? par_u + par_a - 1 : r - 1), col = w0 + x_pc[k] - 2;            \
        const bool ok = x_cell_ok[k] && row >= 0 && row < p.Hc && col >= 0 && col < p.Wc;                    \
        const unsigned pix = UP2 ? ((unsigned)n * (unsigned)Hin + (unsigned)row) * (unsigned)Win + (unsigned)col        \
                                 : ((unsigned)n * (unsigned)Hin + (unsigned)(row >> p.up)) * (unsigned)Win + (unsigned)(col >> p.up); \
        dma_load16(rX, smem + (STG) * G::STAGE + G::A_BYTES + (wave + 4 * k) * 1024, ok ? pix * cin_bytes + x_chunk[k] : kOob); \
      }                                                                                                      \
    }                                                                                                        \
    if (!UP2) a_soff += (unsigned)(G::BK * p.Cout * 2);                                                      \
    if (SW < 64) { h += G::SR; if (h == p.Hc) { h = 0; ++n; } }                                              \
    else { w0 += 64; if (w0 == p.Wc) { w0 = 0; if (++h == p.Hc) { h = 0; ++n; } } }                          \
  }

  // ---- fragment addresses (per-lane constants).  Transposing read: within 16 lanes, lane 4*j+q
  // addresses 4 channels (4q..) of pixel j; 16-lane group G: channels +16*(G&1), pixels +8*(G>>1)
  const int grp = lane >> 4, sl = lane & 15;
  const int lp = 8 * (grp >> 1) + (sl >> 2);
  const unsigned lds0 = (unsigned)(size_t)(lds_char*)smem;
  const int a_col = G::RBA == 256 ? (2 * wm) : wm;                       // 64-byte column of the wave's first 32 channels
  const int a_sw = G::RBA == 256 ? (lp & 3) : ((lp >> 1) & 1);
  const unsigned a_lane = (unsigned)(lp * G::RBA + ((a_col ^ a_sw) << 6) + 32 * (grp & 1) + 8 * (sl & 3));
  unsigned b_lane;                               // tap 0; tap s is s cells further (tr_run_taps)
  {
    // (UP2: tap v of column parity b reads stored column j + v - (1-b): the view shifted by b + v - 1)
    // (SW = 8: the 16 pixels of a K-step are two segment rows of the patch, PCW cells apart)
    const int lp_cell = SW >= 16 ? lp : (lp / SW) * G::PCW + lp % SW;
    const int cell = 1 + (UP2 ? par_b : 0) + lp_cell;   // + cell_base(ks) (a multiple of 4), + 4 and + 8 for the next pixels
    b_lane = (unsigned)(G::A_BYTES + cell * 128 + ((wn ^ ((cell >> 1) & 1)) << 6) + 32 * (grp & 1) + 8 * (sl & 3));
  }

  floatx16 acc[NTAP][MI];
#pragma unroll
  for (int s_ = 0; s_ < NTAP; ++s_)
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[s_][i][e] = 0.0f;

  [[maybe_unused]] TrFrag fa0[MI], fa1[MI];      // (used by the device pass only)
  [[maybe_unused]] TrRun fb0, fb1;
  [[maybe_unused]] constexpr int NR = 2 * MI + 3;                    // LDS reads per K-step
#define WGRAD3_MMA(FA, FB)                                                                                   \
  {                                                                                                          \
    bf16x8 av[MI], bv[NTAP];                                                                                 \
    _Pragma("unroll") for (int i = 0; i < MI; ++i) av[i] = tr_value(FA[i]);                                  \
    tr_run_taps<NTAP>(FB, bv);                                                                               \
    _Pragma("unroll") for (int s_ = 0; s_ < NTAP; ++s_) {                                                    \
      _Pragma("unroll") for (int i = 0; i < MI; ++i)                                                         \
          acc[s_][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[i], bv[s_], acc[s_][i], 0, 0, 0);          \
    }                                                                                                        \
    __builtin_amdgcn_sched_barrier(0);                                                                       \
  }
#define LGKM_WAIT(N) asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N))

  // prologue: slabs 0 and 1 in flight, fragments of (slab 0, K-step 0)
  WGRAD3_DMA(0);
  if (KT > 1) WGRAD3_DMA(1);
  __builtin_amdgcn_s_waitcnt(vm_imm(0));
  __builtin_amdgcn_s_barrier();
  wgrad3_reads<BM, SW, 0>(fa0, fb0, lds0 + a_lane, lds0 + b_lane);
  int cur = 0;
  for (int t = 0; t < KT; ++t) {
    // the loads of slab t+1 (issued one slab ago) are the only ones outstanding
    __builtin_amdgcn_s_waitcnt(vm_imm(0));
    __builtin_amdgcn_s_barrier();
    const int nxt = cur == 2 ? 0 : cur + 1;
    if (t + 2 < KT) { const int st2 = nxt == 2 ? 0 : nxt + 1; WGRAD3_DMA(st2); }
    [[maybe_unused]] const unsigned sa = lds0 + (unsigned)(cur * G::STAGE) + a_lane;
    [[maybe_unused]] const unsigned sb = lds0 + (unsigned)(cur * G::STAGE) + b_lane, nb = lds0 + (unsigned)(nxt * G::STAGE) + b_lane;
    [[maybe_unused]] const unsigned na = lds0 + (unsigned)(nxt * G::STAGE) + a_lane;
#if defined(__HIP_DEVICE_COMPILE__)
    wgrad3_reads<BM, SW, 1>(fa1, fb1, sa, sb);
    LGKM_WAIT(NR);
    WGRAD3_MMA(fa0, fb0)
    wgrad3_reads<BM, SW, 2>(fa0, fb0, sa, sb);
    LGKM_WAIT(NR);
    WGRAD3_MMA(fa1, fb1)
    wgrad3_reads<BM, SW, 3>(fa1, fb1, sa, sb);
    LGKM_WAIT(NR);
    WGRAD3_MMA(fa0, fb0)
    if (t + 1 < KT) {
      wgrad3_reads<BM, SW, 0>(fa0, fb0, na, nb);
      LGKM_WAIT(NR);
    } else {
      LGKM_WAIT(0);
    }
    WGRAD3_MMA(fa1, fb1)
#endif
    cur = nxt;
  }
#undef WGRAD3_DMA
#undef WGRAD3_MMA
#undef LGKM_WAIT

  // partial[split][co][(r*3 + s)*Cin + ci]   (UP2: [(r*2 + v)*Cin + ci] with r = (a, b, u), K = 16 Cin)
  float* __restrict__ P = p.partial + (int64_t)split * p.Cout * p.K;
  const int col_lane = lane & 31, row_lane = (lane >> 5) * 4;
  const int ci = ci0 + wn * 32 + col_lane;
#pragma unroll
  for (int s_ = 0; s_ < NTAP; ++s_)
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int co = co0 + wm * (BM / 2) + i * 32 + (e >> 2) * 8 + row_lane + (e & 3);
        P[(int64_t)co * p.K + (r * NTAP + s_) * p.Cin + ci] = acc[s_][i][e];
      }
}

// The same for the phase form of an upsampled convolution: dW[co][ci][r][s] = sum over splits and over the four output
// parities (a, b) of partial[split][co][((a, b, u_a(r)), v_b(s))][ci], u_0(r) = (r > 0), u_1(r) = (r > 1), v likewise.
__global__ __launch_bounds__(256) void k_wgrad_reduce_up2(const float* __restrict__ partial, int splits, int Cout, int Cin,
                                                          float* __restrict__ dw) {
  __shared__ float sm[4][64];
  const int64_t total = (int64_t)Cout * 9 * Cin;
  const int64_t stride = (int64_t)Cout * 16 * Cin;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t i = (int64_t)blockIdx.x * 64 + lane;
  float acc = 0.0f;
  int ci = 0, tap = 0, co = 0;
  if (i < total) {
    ci = (int)(i % Cin);
    const int64_t q = i / Cin;
    tap = (int)(q % 9);
    co = (int)(q / 9);
    const int r = tap / 3, s_ = tap % 3;
    for (int sp = wave; sp < splits; sp += 4) {
      const float* src = partial + (int64_t)sp * stride + (int64_t)co * 16 * Cin + ci;
      float t = 0.0f;
#pragma unroll
      for (int ab = 0; ab < 4; ++ab) {
        const int a = ab >> 1, b = ab & 1;
        const int u = a == 0 ? (r > 0) : (r > 1), v = b == 0 ? (s_ > 0) : (s_ > 1);
        t += src[((((a << 2) | (b << 1) | u) << 1) | v) * Cin];
      }
      acc += t;
    }
  }
  sm[wave][lane] = acc;
  __syncthreads();
  if (wave == 0 && i < total) dw[((int64_t)co * Cin + ci) * 9 + tap] = (sm[0][lane] + sm[1][lane]) + (sm[2][lane] + sm[3][lane]);
}

// dW[co][ci][r][s] = sum over splits of partial[split][co][(r,s,ci)].  A workgroup owns 64
// consecutive outputs; wave v sums splits v, v+4, ... (independent loads, several in flight),
// then the four waves are combined in a fixed order.
__global__ __launch_bounds__(256) void k_wgrad_reduce(const float* __restrict__ partial, int splits, int Cout, int Cin,
                                                      int taps, float* __restrict__ dw) {
  __shared__ float sm[4][64];
  const int64_t total = (int64_t)Cout * taps * Cin;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t i = (int64_t)blockIdx.x * 64 + lane;
  float acc = 0.0f;
  if (i < total) {
    const float* src = partial + i;
#pragma unroll 8
    for (int sp = wave; sp < splits; sp += 4) acc += src[(int64_t)sp * total];
  }
  sm[wave][lane] = acc;
  __syncthreads();
  if (wave == 0 && i < total) {
    const float t = (sm[0][lane] + sm[1][lane]) + (sm[2][lane] + sm[3][lane]);
    const int ci = (int)(i % Cin);
    const int64_t q = i / Cin;
    const int tap = (int)(q % taps);
    const int co = (int)(q / taps);
    dw[((int64_t)co * Cin + ci) * taps + tap] = t;
  }
}

struct WgradPlan { int bm, bn, bk, tiles_m, tiles_n, splits, rows_per_split, row3; };   // bk = 0: generic kernel; row3: three taps per workgroup

WgradPlan plan_wgrad(int cout, int cin, int k, int64_t rows, int wc, int es, int hc = 0, int up = 0) {
  WgradPlan w;
  w.row3 = 0;
  // an upsampled 3x3 layer in its phase form (row3 = 2): eight groups (a, b, u) of two taps over the stored image
  const int hs = hc >> 1, ws = wc >> 1;
  if (es == 2 && k == 3 && up == 1 && hc > 0 && !(hc & 1) && !(wc & 1) && (ws % 64 == 0 || (ws >= 8 && 64 % ws == 0)) &&
      ((int64_t)hs * ws) % 64 == 0) {
    w.row3 = 2;
    w.bm = cout % 128 == 0 ? 128 : 64;
    w.bn = 64;
    w.bk = 64;
    w.tiles_m = cout / w.bm;
    w.tiles_n = cin / 64;
    const int64_t prow = rows / 4;                       // pixels of one phase = pixels of the stored image
    const int64_t groups = (int64_t)w.tiles_m * w.tiles_n * 8;
    int64_t splits = (512 + groups - 1) / groups;
    const int64_t max_splits = (prow + 511) / 512;
    if (splits > max_splits) splits = max_splits;
    if (splits < 1) splits = 1;
    int64_t rps = (prow + splits - 1) / splits;
    rps = (rps + 63) / 64 * 64;
    w.rows_per_split = (int)rps;
    w.splits = (int)((prow + rps - 1) / rps);
    return w;
  }
  if (es == 2 && k == 3 && hc > 0 && (wc % 64 == 0 || (wc >= 16 && 64 % wc == 0)) && ((int64_t)hc * wc) % 64 == 0) {
    w.row3 = 1;
    w.bm = cout % 128 == 0 ? 128 : 64;
    w.bn = 64;
    w.bk = 64;
    w.tiles_m = cout / w.bm;
    w.tiles_n = cin / 64;
    const int64_t groups = (int64_t)w.tiles_m * w.tiles_n * 3;
    int64_t splits = (512 + groups - 1) / groups;       // two workgroups per compute unit fit: one round
    const int64_t max_splits = (rows + 511) / 512;
    if (splits > max_splits) splits = max_splits;
    if (splits < 1) splits = 1;
    int64_t rps = (rows + splits - 1) / splits;
    rps = (rps + 63) / 64 * 64;
    w.rows_per_split = (int)rps;
    w.splits = (int)((rows + rps - 1) / rps);
    return w;
  }
  w.bm = cout % 128 == 0 ? 128 : 64;
  w.bn = cin % 128 == 0 ? 128 : 64;
  if (w.bm == 64 && w.bn == 64) w.bn = 64;
  w.tiles_m = cout / w.bm;
  w.tiles_n = cin / w.bn;
  const int64_t tiles = (int64_t)w.tiles_m * w.tiles_n * k * k;
  int64_t splits = (1024 + tiles - 1) / tiles;          // about four workgroups per compute unit
  const int64_t max_splits = (rows + 511) / 512;        // at least 512 pixels per split
  if (splits > max_splits) splits = max_splits;
  if (splits < 1) splits = 1;
  // row-slab kernel: slabs of bk pixels that never straddle an image row
  const int bk_big = es == 2 ? 64 : 32;
  w.bk = wc % bk_big == 0 ? bk_big : (wc % (bk_big / 2) == 0 ? bk_big / 2 : 0);
  const int gran = w.bk ? w.bk : 32;
  int64_t rps = (rows + splits - 1) / splits;
  rps = (rps + gran - 1) / gran * gran;
  w.rows_per_split = (int)rps;
  w.splits = (int)((rows + rps - 1) / rps);
  return w;
}

}  // namespace

bool wgrad_mfma_supported(const WgradArgs& a) {
  if (a.cin % 64 != 0 || a.cout % 64 != 0) return false;
  const int64_t es = (int64_t)dtype_size(a.dtype);
  if ((int64_t)a.n * a.hc * a.wc * a.cout * es >= 0x7FFFFFFF) return false;                    // 32-bit buffer offsets
  if ((int64_t)a.n * (a.hc >> a.up) * (a.wc >> a.up) * a.cin * es >= 0x7FFFFFFF) return false;
  const int64_t rows = (int64_t)a.n * a.hc * a.wc;
  return rows < 0x7FFFFFFF;
}

// does launch_wgrad_mfma run this layer in the phase form of an upsampled convolution (4/9 of the multiply-adds)?
bool wgrad_mfma_up_phases(const WgradArgs& a) {
  if (!wgrad_mfma_supported(a)) return false;
  return plan_wgrad(a.cout, a.cin, a.k, (int64_t)a.n * a.hc * a.wc, a.wc, (int)dtype_size(a.dtype), a.hc, a.up).row3 == 2;
}

int64_t wgrad_mfma_workspace_floats(const WgradArgs& a) {
  const int64_t rows = (int64_t)a.n * a.hc * a.wc;
  const WgradPlan w = plan_wgrad(a.cout, a.cin, a.k, rows, a.wc, (int)dtype_size(a.dtype), a.hc, a.up);
  return (int64_t)w.splits * a.cout * a.cin * (w.row3 == 2 ? 16 : a.k * a.k);
}

int launch_wgrad_mfma(const WgradArgs& a, float* workspace, hipStream_t s) {
  if (!wgrad_mfma_supported(a)) return fail(AE_EINVAL, "wgrad_mfma: shape not supported");
  const int64_t rows = (int64_t)a.n * a.hc * a.wc;
  const WgradPlan w = plan_wgrad(a.cout, a.cin, a.k, rows, a.wc, (int)dtype_size(a.dtype), a.hc, a.up);
  WgradParams p;
  // a 1x1 layer that needs no split: the partial layout [co][ci] is the canonical one
  const bool direct = w.splits == 1 && a.k == 1;
  p.x = a.x; p.dy = a.dy; p.partial = direct ? a.dw_canonical : workspace;
  p.M = rows; p.Cout = a.cout; p.Cin = a.cin; p.Hc = a.hc; p.Wc = a.wc; p.ksz = a.k; p.up = a.up;
  p.tiles_m = w.tiles_m; p.tiles_n = w.tiles_n; p.rows_per_split = w.rows_per_split;
  p.K = a.k * a.k * a.cin;
  const int64_t es = (int64_t)dtype_size(a.dtype);
  p.dy_bytes = (unsigned)(rows * a.cout * es);
  p.x_bytes = (unsigned)((int64_t)a.n * (a.hc >> a.up) * (a.wc >> a.up) * a.cin * es);
  const bool pow2 = (a.hc & (a.hc - 1)) == 0 && (a.wc & (a.wc - 1)) == 0;
  p.log_w = p.log_h = 0;
  if (pow2) {
    while ((1 << p.log_w) < a.wc) ++p.log_w;
    while ((1 << p.log_h) < a.hc) ++p.log_h;
  }
  if (w.row3 == 2) {     // phase form: the kernel walks the stored image
    p.M = rows / 4; p.Hc = a.hc / 2; p.Wc = a.wc / 2; p.up = 0; p.K = 16 * a.cin;
  }
  const int64_t blocks = (int64_t)w.splits * w.tiles_m * w.tiles_n * (w.row3 == 2 ? 8 : w.row3 ? 3 : a.k * a.k);
  if (blocks > 0x7FFFFFFF) return fail(AE_EINVAL, "wgrad_mfma: grid too large");
  dim3 grid((unsigned)blocks);
#define WGRAD_LAUNCH_P(T, P2)                                                                           \
  do {                                                                                                  \
    if (w.bm == 128 && w.bn == 128) hipLaunchKernelGGL((k_wgrad<T, 128, 128, P2>), grid, dim3(256), 0, s, p); \
    else if (w.bm == 128) hipLaunchKernelGGL((k_wgrad<T, 128, 64, P2>), grid, dim3(256), 0, s, p);      \
    else if (w.bn == 128) hipLaunchKernelGGL((k_wgrad<T, 64, 128, P2>), grid, dim3(256), 0, s, p);      \
    else hipLaunchKernelGGL((k_wgrad<T, 64, 64, P2>), grid, dim3(256), 0, s, p);                        \
  } while (0)
#define WGRAD_LAUNCH(T)                      \
  do {                                       \
    if (pow2) WGRAD_LAUNCH_P(T, true);       \
    else WGRAD_LAUNCH_P(T, false);           \
  } while (0)
#define WGRAD_ROWS(T, BKV)                                                                              \
  do {                                                                                                  \
    if (w.bm == 128 && w.bn == 128) hipLaunchKernelGGL((k_wgrad_rows<T, 128, 128, BKV>), grid, dim3(256), 0, s, p); \
    else if (w.bm == 128) hipLaunchKernelGGL((k_wgrad_rows<T, 128, 64, BKV>), grid, dim3(256), 0, s, p); \
    else if (w.bn == 128) hipLaunchKernelGGL((k_wgrad_rows<T, 64, 128, BKV>), grid, dim3(256), 0, s, p); \
    else hipLaunchKernelGGL((k_wgrad_rows<T, 64, 64, BKV>), grid, dim3(256), 0, s, p);                  \
  } while (0)
  if (w.row3) {
    const int sw = p.Wc < 64 ? p.Wc : 64;
#define WGRAD_ROW3(BMV, UPV)                                                                            \
  do {                                                                                                  \
    if (sw == 64) hipLaunchKernelGGL((k_wgrad_row3<BMV, 64, UPV>), grid, dim3(256), 0, s, p);           \
    else if (sw == 32) hipLaunchKernelGGL((k_wgrad_row3<BMV, 32, UPV>), grid, dim3(256), 0, s, p);      \
    else hipLaunchKernelGGL((k_wgrad_row3<BMV, 16, UPV>), grid, dim3(256), 0, s, p);                    \
  } while (0)
    if (w.row3 == 2 && sw == 8) {      // stored images of 8 x 8: the phase form only
      if (w.bm == 128) hipLaunchKernelGGL((k_wgrad_row3<128, 8, true>), grid, dim3(256), 0, s, p);
      else hipLaunchKernelGGL((k_wgrad_row3<64, 8, true>), grid, dim3(256), 0, s, p);
    }
    else if (w.row3 == 2) { if (w.bm == 128) WGRAD_ROW3(128, true); else WGRAD_ROW3(64, true); }
    else { if (w.bm == 128) WGRAD_ROW3(128, false); else WGRAD_ROW3(64, false); }
#undef WGRAD_ROW3
  }
  else if (w.bk && a.dtype == AE_BF16) { if (w.bk == 64) WGRAD_ROWS(bf16_t, 64); else WGRAD_ROWS(bf16_t, 32); }
  else if (w.bk) { if (w.bk == 32) WGRAD_ROWS(float, 32); else WGRAD_ROWS(float, 16); }
  else if (a.dtype == AE_BF16) WGRAD_LAUNCH(bf16_t);
  else WGRAD_LAUNCH(float);
#undef WGRAD_ROWS
#undef WGRAD_LAUNCH_P
#undef WGRAD_LAUNCH
  AE_TRY(launch_status("wgrad_mfma"));
  if (direct) return AE_OK;
  const int64_t total = (int64_t)a.cout * a.cin * a.k * a.k;
  const int64_t g = (total + 63) / 64;
  if (w.row3 == 2)
    hipLaunchKernelGGL(k_wgrad_reduce_up2, dim3((unsigned)g), dim3(256), 0, s, workspace, w.splits, a.cout, a.cin, a.dw_canonical);
  else
    hipLaunchKernelGGL(k_wgrad_reduce, dim3((unsigned)g), dim3(256), 0, s, workspace, w.splits, a.cout, a.cin, a.k * a.k,
                       a.dw_canonical);
  return launch_status("wgrad_reduce");
}

}  // namespace ae
