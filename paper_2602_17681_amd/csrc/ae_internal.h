// ae_internal.h — declarations shared by the translation units of libaemodel.
// Host-side plan structures, error plumbing and the launcher prototypes of every
// kernel family.  Nothing here is visible across the C boundary.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "aemodel.h"

namespace ae {

// ---- error plumbing --------------------------------------------------------
int fail(int code, const char* fmt, ...);  // records the thread-local message, returns code
const char* last_error();
#define AE_HIP(expr)                                                                      \
  do {                                                                                    \
    hipError_t e_ = (expr);                                                               \
    if (e_ != hipSuccess) return ae::fail(AE_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)
#define AE_TRY(expr)          \
  do {                        \
    int rc_ = (expr);         \
    if (rc_ != AE_OK) return rc_; \
  } while (0)

inline int launch_status(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(AE_EHIP, "launch %s: %s", what, hipGetErrorString(e));
  return AE_OK;
}

inline size_t dtype_size(int dtype) { return dtype == AE_BF16 ? 2 : 4; }

// ---- plan ------------------------------------------------------------------
enum StepKind { ST_TRANSPOSE = 0, ST_CONV = 1, ST_CHANNEL = 2 };
enum Act { ACT_NONE = 0, ACT_RELU = 1, ACT_SIGMOID = 2 };

// One fused step of the pipeline.  Activations are stored [batch][H][W][C]
// (channels innermost) between steps; `flat` tensors (H = W = 1) coincide with
// the (c,h,w)-ordered vector the spec talks about.
struct Step {
  StepKind kind = ST_CONV;
  int last_token = -1;              // index of the last spec token folded into this step
  int cin = 0, hin = 0, win = 0;    // stored input tensor
  int cout = 0, hout = 0, wout = 0; // stored output tensor
  // ST_TRANSPOSE: per-sample [rows][cols] -> [cols][rows]
  int t_rows = 0, t_cols = 0;
  // ST_CONV (conv1 / conv3 / fc, optionally reading its input through a x2 nearest upsample)
  int k = 1, up = 0, has_bn = 0, act = ACT_NONE, pool = 0;
  int hc = 0, wc = 0;               // resolution the convolution runs at
  int64_t w_off = -1, b_off = -1, bn_off = -1;  // offsets into the parameter blob
  bool needs_dx = true;             // false for the first parametrised step
  // ST_CHANNEL (pnorm and/or awgn)
  int do_pnorm = 0, do_awgn = 0;
  // byte offsets into the model workspace (-1: not allocated), resolved to the pointers below at creation
  int64_t off_out = -1, off_raw = -1, off_wpack = -1, off_wpack_d = -1, off_bn = -1, off_aux = -1;
  // device workspace (owned by the model)
  void* out = nullptr;              // saved output (model dtype)
  void* raw = nullptr;              // conv output before bn/act/pool when those run as a second pass
  void* wpack = nullptr;            // weights repacked [C_out][k][k][C_in] in model dtype (null: use params directly)
  void* wpack_d = nullptr;          // weights repacked for the input-gradient conv [C_in][k][k][C_out], taps flipped
  float* bn_vec = nullptr;          // 6*C floats: scale, shift, mean, invstd, c1, c2
  float* aux = nullptr;             // binary32 copy of a sigmoid output produced in the conv epilogue (bf16 models):
                                    // y*(1-y) from a bf16-rounded y loses all accuracy where the sigmoid saturates
  bool mfma = false;                // forward uses the MFMA implicit-GEMM kernel
  bool up_phases = false;           // forward of an upsampled conv as four 2x2 phase convolutions (CONV_UP_PHASES)
  bool up_dgrad = false;            // its input gradient as one 4x4 stride-2 convolution (CONV_UP_DGRAD)
  bool wfrag = false, wfrag_d = false;   // packed weights of the forward / input-gradient conv in MFMA fragment order (conv_weights_frag_order)
  int thin = 0;                     // 1: thin-in kernels (input is the planar boundary tensor); 2: thin-out kernels
  bool recompute = false;           // thin-in + bn + relu + pool2: the conv output is recomputed by every pass that needs it, never stored
  bool out_planar = false;          // `out` is stored planar [n][C][H][W] (thin-out step)
};

struct Plan {
  int batch = 0, dtype = AE_F32, bn_mode = 0;
  int c0 = 0, h0 = 0, w0 = 0;       // boundary input (NCHW)
  int cl = 0, hl = 0, wl = 0;       // boundary output
  int64_t n_params = 0;
  int64_t latent_n = 0;
  std::vector<Step> steps;
  // workspace sizing (bytes)
  int64_t ws_bytes = 0;
  int64_t off_grad_a = 0, off_grad_b = 0, off_draw = 0, off_draw2 = 0, off_dfull = 0, off_partial = 0, off_wgrad = 0, off_wgrad_inorder = 0, off_splitk = 0;
  int64_t max_act_elems = 0;        // largest step output
  int64_t max_raw_elems = 0;        // largest conv-resolution tensor (raw / dRaw)
  int64_t max_full_elems = 0;       // largest conv-resolution input gradient of an upsampled conv
  int64_t max_partial_floats = 0;   // column-reduction partial buffer
  int64_t max_wgrad_floats = 0;     // split partial tiles of the MFMA weight-gradient kernel
  int64_t max_wgrad_inorder_floats = 0;   // the same for layers whose weight gradient runs in order on the caller's stream
  int64_t max_splitk_floats = 0;    // split-K partial tiles of the forward / input-gradient convolutions
};

int build_plan(const char* spec, int batch, int dtype, int bn_mode, Plan* plan);

// The three-launch forward path for small-image networks (ae_fused_small.hip): parameter offsets and channel
// counts of the matched plan.
struct FusedSmall {
  int64_t w1, b1, bn1, w2, b2, bn2, wf1, bf1, wf2, bf2, w3, b3, w4, b4;
  int c1, c2, n, cr, c3, c4;
};
bool fused_small_match(const Plan& P, FusedSmall* f);
int launch_fused_small(const Plan& P, const FusedSmall& f, const float* params, const float* x, float* y, float* raw1,
                       float* raw2, float* partial, float sigma, uint64_t seed, uint64_t first_sample, hipStream_t s);

// Rows of a column reduction handled by one block (partial-sum granularity): 256 for
// large tensors, fewer when that would leave the machine with too few blocks.
constexpr int kReduceRows = 256;
inline int reduce_rows_per_block(int64_t rows) {
  int rpb = kReduceRows;
  while (rpb > 16 && rows / rpb < 2048) rpb >>= 1;
  return rpb;
}
inline int reduce_blocks(int64_t rows) {
  const int rpb = reduce_rows_per_block(rows);
  return (int)((rows + rpb - 1) / rpb);
}

// ---- launchers (all asynchronous on `s`) -----------------------------------
// layout / dtype
int launch_transpose(const void* in, void* out, int64_t batch, int rows, int cols, int dtype, hipStream_t s);
int launch_to_f32_nchw(const void* in_nhwc, float* out_nchw, int64_t batch, int c, int hw, int dtype, hipStream_t s);

// weights
int launch_pack_weights(const float* w, void* wp, int cout, int cin, int k, int dtype, bool for_dgrad, hipStream_t s, bool frag = false);
// several layers in one launch
struct PackJob { const float* w; void* wp; int cout, cin, k, dgrad; int64_t first_block; int frag; };   // frag: rows in MFMA fragment order
constexpr int kMaxPackJobs = 32;
struct PackBatch { int n; PackJob job[kMaxPackJobs]; };
int launch_pack_weights_batch(PackBatch& pb, int dtype, hipStream_t s);
int launch_pack_weights_1x1(const float* w, void* wp, int cout, int cin, int dtype, bool for_dgrad, hipStream_t s);

// convolution family (direct kernels; see ae_conv.hip for the MFMA ones)
struct ConvArgs {
  const void* x; const void* w; const float* bias; void* y;
  int n, hc, wc, cin, cout, k, up, act, dtype;
  float* partial;  // nullable: per-row-block column sums / sums of squares of the fp32 result
  float* y_aux;    // nullable: binary32 copy of y (after the activation)
  float* splitk_ws = nullptr;      // scratch for split-K partial tiles (conv_mfma_splitk_floats), nullable: no split-K
  int64_t splitk_floats = 0;
  // A 3x3 convolution behind a x2 nearest-neighbour upsample (up = 1; hc, wc = its output size)
  // only ever sees four distinct inputs per output, so both directions have a cheaper form
  // (4/9 of the multiply-adds, exact in real arithmetic):
  //   CONV_UP_PHASES  forward: four 2x2 convolutions of the stored input, one per output parity,
  //                   with weights summed over the taps that read the same input
  //                   (w = [4][cout][2][2][cin], pack_weights_up);
  //   CONV_UP_DGRAD   input gradient: one 4x4 stride-2 convolution of the output gradient
  //                   (x = dY [n][hc][wc][cin], y = dX [n][hc/2][wc/2][cout], w = [cout][4][4][cin]),
  //                   which also replaces the 2x2 sum over each upsampled pixel.
  int geom = 0;
  // Companion tensor (see IgemmParams::comp in ae_conv_mfma.hip): the saved activation of the layer whose output
  // gradient this launch computes, same shape and layout as y.  comp_mode 1: y receives the ReLU-masked gradient and
  // partial its column sums; 2: y unchanged, partial receives the two sums of a batch-norm backward behind ReLU (+ pool),
  // comp_bn = [scale | shift | mean | invstd].  Usable where conv_comp_blocks() > 0 (= the row blocks written to partial).
  const void* comp = nullptr;
  int comp_mode = 0;
  const float* comp_bn = nullptr;
  // w is in MFMA fragment order (the packing kernels' `frag` form): the 32 rows x 32 K-bytes block (nb, kb) of the
  // [rows][K] matrix is one KiB at (nb * K-bytes/32 + kb) KiB, row r's bytes 16c..16c+15 of it at 16 (32 c + r).
  // Only where conv_weights_frag_order() says so (the kernel that loads its weights straight into registers).
  bool w_frag = false;
  // Dense-GEMM epilogues (k = 1 layers whose tiles all lie inside the output, no split-K):
  //   CONV_EPI_MXQ    the stored output is MX block-quantised (blocks of mx_block columns, a power of two between the
  //                   elements of 16 bytes and 64; FP4 E2M1 elements);
  //   CONV_EPI_RESID  nothing is stored: `partial` receives, per row tile, the column sums of
  //                   resid - (x w^T + bias) and of its square (resid: [rows][cout] in the storage type).
  int epi = 0;
  const void* resid = nullptr;
  int mx_block = 32;
  int mx_elem = 0;                 // element format of CONV_EPI_MXQ: 0 FP4 E2M1, 1 the 4-bit integer reading, 2 FP8 E4M3
  // Square dense products (n = cin = cout, k = 1) with triangular operands; the kernel then walks only the K range
  // that can hold non-zeros and returns at once in tiles that hold no wanted output (they are left unwritten):
  //   CONV_TRI_LOWER_UPPER  x lower triangular, w^T upper triangular (w[n][k] = 0 for k > n);
  //   CONV_TRI_UPPER_X      x upper triangular; wanted: the outputs on and above the diagonal;
  //   CONV_TRI_UPPER_W      w upper triangular (w[n][k] = 0 for k < n); wanted: the outputs below the diagonal.
  //   CONV_TRI_UPPER_LOWER  x upper triangular, w^T lower triangular (w[n][k] = 0 for k < n): every output wanted;
  //   CONV_TRI_PAIR_*       one level of a blocked triangular inverse: all pairs of neighbouring tri_b x tri_b diagonal
  //                         blocks (r even, r+1) in one launch; only the tiles of the named off-diagonal block of
  //                         each pair are computed, over the K range of the named block:
  //                           UPPER_K0: rows in block r, columns in block r+1, K = block r;
  //                           LOWER_K1: rows in block r+1, columns in block r, K = block r+1.
  //                         tri_pairs > 0 limits the launch to the first tri_pairs pairs (the rest keep their contents).
  int tri = 0;
  int tri_b = 0;
  //                         tri_d > 0 (a multiple of 128): the matrices are an identity block beyond row and column
  //                         tri_d; tiles and K ranges beyond it are skipped (outputs there are zero, left unwritten).
  int tri_pairs = 0;
  int tri_d = 0;
};
enum { CONV_TRI_NONE = 0, CONV_TRI_LOWER_UPPER = 1, CONV_TRI_UPPER_X = 2, CONV_TRI_UPPER_W = 3, CONV_TRI_UPPER_LOWER = 4,
       CONV_TRI_PAIR_UPPER_K0 = 8, CONV_TRI_PAIR_LOWER_K1 = 9 };
enum { CONV_PLAIN = 0, CONV_UP_PHASES = 1, CONV_UP_DGRAD = 2 };
enum { CONV_EPI_NONE = 0, CONV_EPI_MXQ = 1, CONV_EPI_RESID = 2 };
bool conv_epi_usable(const ConvArgs& a);         // can launch_conv_mfma run a.epi for this shape?
bool conv_up_phases_usable(const ConvArgs& a);   // a: the plain description (geom ignored)
int conv_comp_blocks(const ConvArgs& a);
bool conv_weights_frag_order(const ConvArgs& a);   // does this launch take its weights in fragment order (ConvArgs::w_frag)?
bool conv_up_dgrad_usable(const ConvArgs& a);    // a: the plain description of the input-gradient conv at conv resolution
// Summed weights of the two forms above from the canonical [cout][cin][3][3] fp32 weights.
int launch_pack_weights_up(const float* w, void* wp, int cout, int cin, int dtype, int geom, hipStream_t s);
int64_t conv_mfma_splitk_floats(const ConvArgs& a);   // 0: this layer runs without split-K
int launch_conv_direct(const ConvArgs& a, hipStream_t s);
bool conv_mfma_supported(const ConvArgs& a);
int launch_conv_mfma(const ConvArgs& a, hipStream_t s);
int conv_partial_rows(const ConvArgs& a, bool mfma);  // rows per partial-sum block of the kernel that will run

struct WgradArgs {
  const void* x; const void* dy; float* dw_canonical;  // dw is accumulated with atomics: must be zeroed first
  int n, hc, wc, cin, cout, k, up, dtype;
};
int64_t wgrad_direct_workspace_floats(const WgradArgs& a);   // scratch the fallback weight gradient wants (fewer chunks with less)
int launch_wgrad_direct(const WgradArgs& a, float* workspace, int64_t workspace_floats, hipStream_t s);
bool wgrad_mfma_supported(const WgradArgs& a);
bool wgrad_mfma_up_phases(const WgradArgs& a);   // will it run as the phase form of an upsampled conv (4/9 of the multiply-adds)?
int64_t wgrad_mfma_workspace_floats(const WgradArgs& a);
int launch_wgrad_mfma(const WgradArgs& a, float* workspace, hipStream_t s);  // overwrites dw (no zeroing needed)

// 3x3 convolutions with 1..4 channels on one side (first / last layer); see ae_conv_thin.hip
bool thin_in_supported(int ct, int cw, int k, int up);
bool thin_out_supported(int ct, int cw, int k, int dtype);
int thin_in_partial_rows();
int launch_thin_in_conv(const void* thin, const float* wcanon, const float* bias, void* out, float* partial, int n,
                        int h, int w, int ct, int cw, int flip, int act, int dtype, hipStream_t s);
int launch_thin_out_conv(const void* wide, const float* wcanon, const float* bias, void* out, float* out_f32, int n,
                         int hc, int wc, int ct, int cw, int up, int act, int dtype, hipStream_t s);
// bf16 matrix-core versions; see ae_conv_thin_mfma.hip
bool thin_in_mfma_supported(int ct, int cw, int k, int up, int dtype);
int thin_in_mfma_blocks(int n, int h, int w);   // = number of partial-sum blocks it writes
int64_t thin_wfrag_bytes(int cw);               // scratch for the repacked weights
int launch_thin_in_mfma(const void* thin, const float* wcanon, void* wfrag, const float* bias, void* out, float* partial,
                        int n, int h, int w, int ct, int cw, int flip, int act, int upsum, int dtype, hipStream_t s);
// first layer + batch-norm + ReLU + pool2 with the convolution output recomputed in every pass
bool thin_first_supported(int ct, int cw, int k, int up, int dtype, int h, int w);
int thin_first_blocks(int n, int h, int w, int cw, int pass);   // = partial blocks pass 0 / 2 write
int launch_thin_first(int pass, const void* thin, const float* wcanon, void* wfrag, const float* bias,
                      const float* bn_vec, const void* dout, void* out, float* partial, float* dw_canonical, int n, int h,
                      int w, int ct, int cw, hipStream_t s);
bool thin_out_mfma_supported(int ct, int cw, int k, int dtype);
int64_t thin_out_wz_bytes(int ct, int cw);
int launch_thin_out_mfma(const void* wide, const float* wcanon, void* wz, const float* bias, void* out, float* out_f32,
                         int n, int hc, int wc, int ct, int cw, int up, int act, int dtype, hipStream_t s);
bool thin_wgrad_mfma_supported(int ct, int cw, int wq, int dtype);
int64_t thin_wgrad_mfma_workspace_floats(int n, int hq, int wq, int cw);
int launch_thin_wgrad_mfma(const void* thin, const void* wide, float* workspace, float* dw_canonical, int n, int hq,
                           int wq, int ct, int cw, int mode, int up, int dtype, hipStream_t s);
int64_t thin_wgrad_workspace_floats(int64_t q_pixels, int ct, int cw);
int launch_thin_wgrad(const void* thin, const void* wide, float* workspace, float* dw_canonical, int n, int hq, int wq,
                      int ct, int cw, int mode, int up, int dtype, hipStream_t s);
int plane_sums_split(int64_t hw);   // pieces per plane = partial rows per sample
int launch_plane_sums(const void* x, int64_t n, int c, int64_t hw, int dtype, float* partial, hipStream_t s);

// per-channel reductions and the second pass after a conv
int launch_col_stats(const void* x, int64_t rows, int c, int dtype, float* partial, hipStream_t s);
// about: the per-channel constant the partial sums were taken about (the conv epilogues use the bias), or null
int launch_bn_finalize(const float* partial, int nblocks, int64_t rows, int c, const float* gamma_beta,
                       const float* stored_mean_var, const float* about, float* bn_vec, hipStream_t s);
int launch_post_forward(const void* raw, const float* bn_vec, void* out, int64_t n, int h, int w, int c, int act,
                        int pool, int dtype, hipStream_t s);
int launch_post_bwd_reduce(const void* raw, const void* dout, const void* out_act, const float* bn_vec, int64_t n, int h,
                           int w, int c, int act, int pool, int dtype, float* partial, hipStream_t s);
int launch_bn_bwd_finalize(const float* partial, int nblocks, int64_t rows, int c, float* dbias, float* bn_vec,
                           float* dgamma_dbeta, int batch_stats, hipStream_t s, const void* fix_raw = nullptr,
                           const void* fix_dout = nullptr, int64_t n = 0, int h = 0, int w = 0, int pool = 0);
int launch_act_bwd_colsum(const void* out, const float* out_f32, const void* dout, void* draw, int64_t rows, int c,
                          int act, int dtype, float* partial, hipStream_t s);
int launch_post_bwd_apply(const void* raw, const void* dout, const float* bn_vec, void* draw, int64_t n, int h, int w,
                          int c, int act, int pool, int has_bn, int dtype, hipStream_t s);
int launch_act_bwd(const void* out, const float* out_f32, const void* dout, void* draw, int64_t n_elem, int act,
                   int dtype, hipStream_t s);
int launch_colsum_finalize(const float* partial, int nblocks, int c, float* out, hipStream_t s);
int launch_upsum(const void* dfull, void* dx, int64_t n, int h, int w, int c, int dtype, hipStream_t s);
int launch_fill_zero(void* p, int64_t bytes, hipStream_t s);

// channel (power normalisation + noise), Monte-Carlo bookkeeping, loss
int launch_pnorm_awgn(const void* z, void* y, int64_t batch, int c, int hw, int dtype, int do_pnorm, int do_awgn,
                      float sigma, uint64_t seed, uint64_t first_sample, hipStream_t s);
int launch_pnorm_bwd(const void* z, const void* g, void* dz, int64_t batch, int64_t n, int dtype, hipStream_t s);
int launch_noise(uint64_t seed, uint64_t first_sample, int64_t batch, int64_t n, float* out, hipStream_t s);
int launch_gen_bits(uint64_t seed, uint64_t first_sample, int64_t batch, int k, float* x, hipStream_t s);
int launch_count_errors(const float* y, const float* x, int64_t batch, int k, uint64_t* bit_err, uint64_t* blk_err,
                        hipStream_t s);
int launch_mse(const void* y, const void* t, int64_t n, int dtype, float* loss, void* dy, hipStream_t s);

}  // namespace ae
