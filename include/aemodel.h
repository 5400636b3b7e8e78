/* aemodel.h — C boundary of the MI355X noisy-channel autoencoder library.
 *
 * The library runs the batched forward (and backward) pass of a learned
 * transmission pipeline: a conv / fully-connected encoder with batch-norm,
 * ReLU and 2x2 max-pooling, per-sample power normalisation, additive white
 * Gaussian noise from a Philox4x32-10 counter-based generator at a requested
 * SNR, and a nearest-upsampling conv / fc decoder, plus the MSE loss and the
 * Monte-Carlo bookkeeping (message bits, error counts) used for error-rate
 * estimation.  The pipeline and its five workloads are the ones the project's
 * contract states (the attached paper's text does not define them); each entry
 * point below therefore states the definition it implements in full.
 *
 * Conventions common to all calls
 *  - Every tensor pointer is a DEVICE pointer owned by the caller unless the
 *    argument is documented as host memory.  The library never frees or keeps a
 *    caller pointer beyond the call's enqueued work.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls only enqueue work; they do not synchronise.
 *  - Return value: AE_OK (0) or a negative ae_status.  No call aborts or throws;
 *    model_last_error() returns a thread-local message for the last failure.
 *  - dtype AE_F32: tensors are IEEE binary32.  dtype AE_BF16: x, y, dy, targets
 *    and every stored activation are bfloat16 (round-to-nearest-even), all
 *    accumulation / statistics / noise / loss arithmetic is binary32, and the
 *    parameter blob and the gradient blob are binary32 in both modes.
 *  - Image tensors at the boundary are NCHW, contiguous.
 *  - One model handle must not be used from two threads or two streams at once.
 */
#ifndef AEMODEL_H
#define AEMODEL_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ae_model ae_model; /* opaque, library-owned */

enum ae_status {
  AE_OK = 0,
  AE_EINVAL = -1, /* null pointer, bad size or bad enum value          */
  AE_ESPEC = -2,  /* layer spec does not parse or uses an unsupported sequence */
  AE_ESHAPE = -3, /* shapes in the spec do not fit together             */
  AE_ESTATE = -4, /* call order violated (backward before forward)      */
  AE_ENOMEM = -5, /* device allocation failed                           */
  AE_EHIP = -6    /* a HIP runtime call failed (no device, launch error) */
};

enum ae_dtype { AE_F32 = 0, AE_BF16 = 1 };

/* ---- layer spec ----------------------------------------------------------
 * Comma-separated tokens; the first is the per-sample input shape.
 *   in:CxHxW      input shape
 *   conv3:N       3x3 cross-correlation, stride 1, zero pad 1, N output channels, + bias
 *   conv1:N       1x1 convolution, + bias
 *   fc:N          fully connected layer on a flattened (Cx1x1) tensor, + bias
 *   bn            batch normalisation per channel over (batch, H, W), eps = 1e-5,
 *                 biased variance (bn_mode 0: batch statistics; 1: stored statistics)
 *   relu | sigmoid
 *   pool2         2x2 max-pool, stride 2 (H and W must be even)
 *   up2           nearest-neighbour upsampling x2 (must be followed by a conv)
 *   flatten       CxHxW -> (C*H*W)x1x1 in (c,h,w) order
 *   reshape:CxHxW inverse of flatten
 *   pnorm         scale each sample's whole tensor to unit mean power: x = z / sqrt(mean z^2)
 *                 (x = 0 when the sample is all zero)
 *   awgn          y = x + sigma * g, g ~ N(0,1) from Philox, sigma^2 = 10^(-snr_db/10)
 * Accepted sequences: [up2] conv|fc [bn] [relu|sigmoid] [pool2]; flatten; reshape;
 * pnorm; awgn; pnorm,awgn.  Anything else is AE_ESPEC.
 *
 * Parameter blob (binary32, caller-owned), in spec order:
 *   conv: W[C_out][C_in][k][k] then b[C_out];  fc: W[out][in] then b[out];
 *   bn: gamma[C], beta[C] (bn_mode 1: then mean[C], var[C]).
 * The gradient blob has the same layout (stored-statistics slots receive 0).
 */

/* Parse `layer_spec` and report sizes without touching the GPU (host-only).
 * Any output pointer may be NULL.  workspace_bytes is what model_create would
 * allocate on the device for this batch and dtype. */
int model_describe(const char* layer_spec, int batch, int dtype, int bn_mode, int64_t* n_params,
                   int64_t in_chw[3], int64_t out_chw[3], int64_t* latent_n, int64_t* workspace_bytes);

/* Build a model for a fixed batch size: parses the spec, infers shapes, chooses
 * a kernel per layer and allocates the model-owned device workspace (saved
 * activations, packed weights, batch-norm partial sums, gradient staging) on the
 * current device.  *out receives the handle; free it with model_destroy. */
int model_create(const char* layer_spec, int batch, int dtype, int bn_mode, ae_model** out);
void model_destroy(ae_model* m);

int model_param_count(const ae_model* m, int64_t* n_params);
int model_io_shape(const ae_model* m, int64_t in_chw[3], int64_t out_chw[3], int64_t* latent_n);

/* Global index of sample 0 of the next model_forward (default 0).  The noise of
 * a sample depends only on (seed, global sample index, element index), so a
 * Monte-Carlo run split into launches gives the same noise as one big launch. */
int model_set_sample_offset(ae_model* m, uint64_t first_sample);

/* Forward pass of the whole pipeline on one batch.
 *   params : device, binary32[n_params]          x : device, [batch][C][H][W] (model dtype)
 *   y      : device, [batch][C_out][H_out][W_out] (model dtype), written
 * Noise: element i (in (c,h,w) order) of the tensor entering `awgn`, sample with
 * global index g, receives sigma * N where sigma = (float)10^(-snr_db/20) and N is
 * deviate (i&1) of word pair (i&3)>>1 of Philox4x32-10(counter = (g_lo, g_hi, i>>2, 0),
 * key = (seed_lo, seed_hi)), mapped to a normal deviate by the fixed binary32
 * Box-Muller sequence documented with model_noise.  Activations are kept inside
 * the model for a following model_backward. */
int model_forward(ae_model* m, const void* params, const void* x, float snr_db, uint64_t seed, void* y,
                  void* stream);

/* Backward pass through the graph of the immediately preceding model_forward on
 * the same handle (AE_ESTATE otherwise), with the same params and x.
 *   dy    : device, gradient of a scalar loss w.r.t. y, same shape/dtype as y
 *   grads : device, binary32[n_params], overwritten with d loss / d params
 * Definitions: conv/fc adjoints; batch-norm with batch statistics
 * dx = gamma*invstd*(dy - mean(dy) - xhat*mean(dy*xhat)); max-pool routes to the
 * first maximum in scan order (0,0),(0,1),(1,0),(1,1); upsample sums its 2x2
 * copies; pnorm dz = (g - x*mean(g.x))/r; the noise is additive (identity);
 * ReLU derivative is 0 for inputs <= 0; sigmoid dy*y*(1-y). */
int model_backward(ae_model* m, const void* params, const void* x, const void* dy, void* grads, void* stream);

/* Mean squared error over all n_elem elements: *loss_dev = mean((y-t)^2) (device,
 * binary32, overwritten); if dy is non-NULL it receives 2*(y-t)/n_elem in `dtype`. */
int model_loss_mse(const void* y, const void* target, int64_t n_elem, int dtype, float* loss_dev, void* dy,
                   void* stream);

/* Standard-normal tensor out[batch][n] (device, binary32) exactly as the forward
 * pass draws it (before scaling by sigma).  Words (w0,w1) -> (g0,g1):
 *   u = fma(float(w0), 2^-32, 2^-33); ln u by range reduction to [sqrt(1/2), sqrt 2)
 *   and a fixed degree-8 polynomial; rho = sqrt(-2 ln u); the angle is the quadrant
 *   (top two bits of w1) plus a 24-bit fraction of a quarter turn, evaluated with
 *   fixed polynomials for sin and cos of (pi/2)*r on [0,1/2]; g0 = rho*cos, g1 = rho*sin.
 * Every step is one correctly rounded binary32 operation, so the tensor is
 * reproducible bit for bit on any IEEE machine. */
int model_noise(uint64_t seed, uint64_t first_sample, int64_t batch, int64_t n, float* out, void* stream);

/* Stand-alone fused power normalisation + AWGN on z[batch][n] (contiguous, `dtype`),
 * the same kernel the forward pass uses for a flattened latent.  y may alias z. */
int model_pnorm_awgn(const void* z, void* y, int64_t batch, int64_t n, int dtype, float snr_db, uint64_t seed,
                     uint64_t first_sample, void* stream);

/* Monte-Carlo message source: x_pm1[batch][k] (device, binary32) = +1 where bit j
 * of the sample's message is set, else -1.  Bit j of global sample g is bit (j&31)
 * of word (j>>5)&3 of Philox4x32-10(counter = (g_lo, g_hi, j>>7, 1), key = seed). */
int model_gen_bits(uint64_t seed, uint64_t first_sample, int64_t batch, int k, float* x_pm1, void* stream);

/* Hard decisions at 1/2 on y[batch][k] (device, binary32) against the sent symbols:
 * adds the number of wrong bits to *bit_err and the number of blocks with at least
 * one wrong bit to *blk_err (device, 64-bit counters the caller zeroes once). */
int model_count_errors(const float* y, const float* x_pm1, int64_t batch, int k, uint64_t* bit_err,
                       uint64_t* blk_err, void* stream);

/* A whole Monte-Carlo error-rate estimate at one SNR point: the samples with global indices first_sample ..
 * first_sample + total_samples - 1 run in launches of m's batch size, each launch being
 * model_gen_bits -> model_forward -> model_count_errors with the launch's sample offset, so the result does not
 * depend on how the range is cut into launches.  When total_samples is not a multiple of m's batch, the last,
 * shorter launch runs on m_tail, a second handle of the same network created with exactly that remaining batch
 * (NULL otherwise).  m must be a binary32 model from k symbols (in:kx1x1) to k soft bits.
 *   params  : device, binary32[n_params]       x_buf, y_buf : device scratch, binary32 [m's batch][k] each
 *   bit_err, blk_err : device 64-bit counters the caller zeroes before and reads after (they accumulate):
 *   BER = bit_err / (k * total_samples), BLER = blk_err / total_samples.
 * Everything is enqueued on `stream`; nothing is read back or synchronised. */
int model_monte_carlo(ae_model* m, ae_model* m_tail, const void* params, float snr_db, uint64_t seed,
                      uint64_t first_sample, uint64_t total_samples, float* x_buf, float* y_buf, uint64_t* bit_err,
                      uint64_t* blk_err, void* stream);

/* Introspection for tests.  The pipeline is executed as fused steps; step s has
 * one saved output tensor.  model_step_info reports, for step s, the index of the
 * LAST spec token (0-based, not counting "in:") folded into it and its output
 * shape; model_get_activation writes that saved output as binary32 NCHW. */
int model_num_steps(const ae_model* m, int* n_steps);
int model_step_info(const ae_model* m, int step, int* last_token, int64_t chw[3]);
int model_get_activation(ae_model* m, int step, float* out_nchw, void* stream);
/* A step that applies batch-norm and/or max-pooling keeps the convolution's own output (bias included, before
 * batch-norm, activation and pooling) for the backward pass, which takes its ReLU masks and pool winners from it.
 * chw (nullable) receives that tensor's shape, out_nchw (nullable: query the shape only) the tensor as binary32
 * NCHW.  AE_EINVAL for a step that keeps no such tensor, AE_ESTATE before the first forward pass. */
int model_get_conv_output(ae_model* m, int step, int64_t chw[3], float* out_nchw, void* stream);

/* Per-kernel timing for benchmarks.  While enabled, every kernel the executor
 * launches is bracketed by two HIP events on the caller's stream (a few
 * microseconds of host time per launch).  Slots are named
 * "stepNN.<fwd|bwd>.<kernel>"; model_timing_read waits for the slot's events,
 * adds their elapsed times to the slot's total and reports the algorithmic
 * floating-point operations and bytes of one launch (2*M*N*K for the convolution
 * family; bytes every operand must cross HBM at least once).  name may be NULL. */
int model_timing_enable(ae_model* m, int on);
/* Scheduling of the backward pass (an execution detail, not part of the method).  By
 * default (on = 1) model_backward enqueues the weight-gradient kernels on a second stream
 * owned by the handle, ordered against the caller's stream by events in both directions:
 * everything enqueued on the caller's stream after model_backward returns sees all
 * gradients.  on = 0 keeps every kernel on the caller's stream in program order (also the
 * behaviour while per-kernel timing is enabled, so that each measured duration belongs to
 * one kernel alone).  Results are identical either way. */
int model_set_overlap(ae_model* m, int on);
/* Inference mode (on = 1): forward passes keep nothing for a backward pass — model_backward, model_get_activation
 * and model_get_conv_output then return AE_ESTATE — which lets the executor take paths that never write the
 * intermediate tensors.  Today that is the three-launch path for small-image networks of the shape
 *   conv3,bn,relu,pool2, conv3,bn,relu,pool2, flatten, fc, pnorm, awgn, fc, reshape, up2,conv3,relu, up2,conv3,sigmoid
 * (binary32, batch statistics, images up to 32 x 32, at most 4 channels in and out, hidden channel counts
 * multiples of 16), where one workgroup keeps a sample's tensors in LDS; every other network runs its usual
 * kernels.  Results are the same definitions in binary32 (summation order differs).  Default: off. */
int model_set_inference(ae_model* m, int on);
/* Every pass converts the binary32 parameter blob into the kernels' operand layouts (the blob may change between
 * calls).  on = 1 is the caller's promise that the CONTENTS of params stay the same from call to call (repeated
 * evaluation, Monte-Carlo launches): the conversion then runs only in the first forward and the first backward
 * pass after this call, and again whenever a different params pointer is passed.  Call it again (on = 1) after
 * changing the values in place, or with on = 0 to return to converting in every pass (the default). */
int model_set_params_static(ae_model* m, int on);
/* Recomputation instead of storage (an execution detail, not part of the method).  When the first layer is a 3x3
 * convolution of at most 4 input channels into 32 or 64 channels followed by batch-norm, ReLU and 2x2 max-pooling
 * (bfloat16, image a whole number of 256-pixel patches), its convolution output — the largest tensor of the
 * network — is by default (on = 1) never written: the statistics pass, the normalise-activate-pool pass and the
 * two passes of its backward step each recompute it from the input (K = 27), and model_get_conv_output rebuilds it
 * from the x and params of the last model_forward, which must still be valid then.  on = 0 stores it as for any
 * other layer.  Every stored value is computed by the same arithmetic either way (sums run in another order).
 * A backward pass needs a forward pass after the last change of this setting. */
int model_set_recompute(ae_model* m, int on);
/* Fused backward epilogues (an execution detail, not part of the method).  By default (on = 1), in bfloat16 models the
 * kernel that computes the gradient with respect to a layer's output also does, while it stores each tile, the part
 * of that layer's backward step which only needs the layer's saved activation beside the gradient: for a conv + ReLU
 * layer the ReLU backward and the column sums of the bias gradient, for a conv + batch-norm + ReLU (+ pool2) layer
 * the two sums of the batch-norm backward (sum dy, sum dy * xhat).  on = 0 runs these as passes of their own.  The
 * stored values are the same either way; the sums are taken in another order. */
int model_set_fused_backward(ae_model* m, int on);
int model_timing_slots(const ae_model* m, int* n_slots);
int model_timing_read(ae_model* m, int slot, char* name, int name_len, double* total_ms, int64_t* launches,
                      double* flops_per_launch, double* bytes_per_launch);
int model_timing_reset(ae_model* m);

/* MX block quantisation Q(x) of the paper's Section "MX quantization", Eq. (1), applied to a
 * row-major [rows][d] tensor (device memory, dtype AE_F32 or AE_BF16): every block of `block`
 * consecutive elements of a row gets the power-of-two scale s = 2^(floor(log2 max|x_j|) - r_max)
 * and every element becomes s * Q_e(x_j / s), Q_e being the FP4 E2M1 element quantiser (magnitudes
 * 0, 0.5, 1, 1.5, 2, 3, 4, 6; r_max = 2; nearest value, ties to the even code, saturating at 6).
 * An all-zero block yields zeros; the scale exponent is clamped to [-127, 127].  q has the shape
 * and dtype of x and may be x itself.  d must be a positive multiple of block (32 in the paper's
 * experiments); any block size works, sizes of 8 elements (bf16) / 4 (fp32) times a power of two
 * up to 64 lanes, with 16-byte aligned pointers, take the vector path.  AE_EINVAL on bad arguments.
 * model_mx_quantize_elem: the same with the element format chosen (the paper names FP4, INT4 and FP8 elements):
 *   elem 0: FP4 E2M1 as above;  2: FP8 E4M3 of the OCP 8-bit floating point specification (r_max = 8, largest value
 *   448, subnormals below 2^-6);  1: a 4-bit integer element, which is not a standard MX format and which the paper
 *   does not define — reading: magnitudes k/4, k = 0..7, r_max = 0, nearest, ties to even, saturating at 1.75. */
int model_mx_quantize(const void* x, void* q, int64_t rows, int64_t d, int block, int dtype, void* stream);
int model_mx_quantize_elem(const void* x, void* q, int64_t rows, int64_t d, int block, int elem, int dtype, void* stream);

/* Transformation mean squared error of the paper (Definition "Transformation Mean Squared Error",
 * Eq. 2, and the block-wise error E_B^i of its numerical analysis) for the affine map
 * T(x) = A x + v over `rows` tokens x[rows][d] (device, row-major, dtype AE_F32 or AE_BF16):
 *     yq = Q(T(x))                      written to yq[rows][d] (same dtype; T(x) is rounded to the
 *                                       storage type before it is quantised, Q as in model_mx_quantize),
 *     r  = x - T^-1(yq),  T^-1(y) = A^-1 y - A^-1 v   (never stored),
 *     e_blocks[i] = mean over tokens of 1/block * sum over block i of r_j^2   (d/block floats, device),
 *     e_total[0]  = 1/d * mean over tokens of ||r||^2                          (device).
 * a_mat = A and a_inv = A^-1 are [d][d] row-major in the tensor's dtype (the caller supplies the inverse),
 * v and inv_shift = -A^-1 v are binary32 [d].  Both products run on the matrix cores with binary32
 * accumulation; the quantiser and the squared-error sums are epilogues of the two GEMMs.
 * workspace: model_transform_mse_workspace bytes of device memory.  block: a power of two, 8 (bf16) / 4 (fp32) to 64; d a multiple of
 * 128, rows a multiple of 256 (bf16) or 128 (fp32), every tensor below 2 GiB: AE_EINVAL otherwise. */
int model_transform_mse_workspace(int64_t rows, int64_t d, int dtype, int64_t* bytes);
/* The constant term of the inverse map of the same definition, T^-1(y) = A^-1 y - A^-1 v:
 * inv_shift[i] = -sum_j a_inv[i][j] v[j]  (a_inv [d][d] row-major in dtype, v and inv_shift binary32 [d], device;
 * double-precision accumulation).  1 <= d <= 46340, AE_EINVAL otherwise. */
int model_inverse_shift(const void* a_inv, const float* v, int64_t d, int dtype, float* inv_shift, void* stream);
int model_transform_mse(const void* x, const void* a_mat, const float* v, const void* a_inv, const float* inv_shift,
                        int64_t rows, int64_t d, int block, int dtype, void* yq, void* workspace, float* e_blocks,
                        float* e_total, void* stream);
/* The same with the element format of Q chosen as in model_mx_quantize_elem (0 FP4 E2M1, 1 the 4-bit integer
 * reading, 2 FP8 E4M3). */
int model_transform_mse_elem(const void* x, const void* a_mat, const float* v, const void* a_inv, const float* inv_shift,
                             int64_t rows, int64_t d, int block, int elem, int dtype, void* yq, void* workspace,
                             float* e_blocks, float* e_total, void* stream);

/* model_transform_mse_elem for callers that cannot allocate device memory or bring a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, definitions and results, but the
 * per-tile partial sums live in a 4 MiB buffer built into the library's device code (each GPU the library runs on
 * holds its own copy until the process ends; its address is looked up on the first call on that device).  The call
 * allocates nothing.  Shapes whose model_transform_mse_workspace exceeds 4 MiB (rows/256 * d > 524 288 for bf16,
 * rows/128 * d for fp32) are AE_EINVAL.  All calls on one GPU share the buffer: calls that overlap in time on one GPU
 * (two streams, two threads) race; calls ordered on one stream do not. */
int model_transform_mse_static(const void* x, const void* a_mat, const float* v, const void* a_inv, const float* inv_shift,
                               int64_t rows, int64_t d, int block, int elem, int dtype, void* yq, float* e_blocks,
                               float* e_total, void* stream);

/* LU parametrisation of a learnable invertible matrix (the paper's Section on learning affine transformations,
 * Eq. 4):  A = P L (U + diag(s)).  Free parameters (device pointers, binary32 master copies): lp, up [d][d]
 * row-major, of which only the strictly lower part of lp and the strictly upper part of up are read (L has a
 * unit diagonal, U a zero diagonal); log_s [d] with s = sign_s * exp(log_s) (sign_s [d] holds +-1 and is not
 * learned); perm [d] (int32): the fixed permutation, (P M)[i] = M[perm[i]] — it must be a permutation of
 * 0..d-1 (an entry outside that range is treated as i; duplicates give unspecified rows, never an access out
 * of bounds).  dtype: storage type of the matrix operands and results (AE_F32 or AE_BF16); products run on the
 * matrix cores with binary32 accumulation.  d: a multiple of 32, 32..16384, else AE_EINVAL.  workspace:
 * model_lu_workspace bytes of device memory (the same size serves both calls); the workspace and every [d][d]
 * array must be 16-byte aligned.
 * model_lu_compose  writes a_out = A [d][d] in dtype.
 * model_lu_backward given g = dLoss/dA [d][d] in dtype, writes the gradients of the free parameters in binary32:
 *   d_lp [d][d] (strictly lower part, zero elsewhere), d_up [d][d] (strictly upper part, zero elsewhere),
 *   d_log_s [d].  The products are rounded to dtype before they are cut to the triangles.  The lower-triangle
 *   branch runs on a stream the library owns (default priority), forked from and joined back into `stream` inside
 *   the call: for the caller everything is ordered on `stream` as usual.
 * model_vol_penalty the volume regulariser in the form used in practice (Eq. 6 and the paragraph after it):
 *   *value = (sum_i log_s[i])^2 (device pointer), d_log_s (device, nullable) its gradient 2 sum. */
int model_lu_workspace(int64_t d, int dtype, int64_t* bytes);
int model_lu_compose(const float* lp, const float* up, const float* log_s, const float* sign_s, const int* perm,
                     int64_t d, int dtype, void* a_out, void* workspace, void* stream);
int model_lu_backward(const void* g, const float* lp, const float* up, const float* log_s, const float* sign_s,
                      const int* perm, int64_t d, int dtype, float* d_lp, float* d_up, float* d_log_s,
                      void* workspace, void* stream);
int model_vol_penalty(const float* log_s, int64_t d, float* value, float* d_log_s, void* stream);
/* The inverse of the parametrised matrix, A^-1 = (U + diag s)^-1 L^-1 P^T (what the transformation error and the
 * folding take beside A): a_inv_out [d][d] in dtype.  Both triangular factors are inverted by a blocked recursion
 * (128 x 128 diagonal blocks by substitution, then neighbouring blocks merged, two products and a transposing copy per level), all in
 * binary32 on the matrix cores; s must not contain zeros.  d: a multiple of 128, at most 16384.  The recursion works
 * at dp = 128 times the smallest power of two that reaches d, on the factors extended by an identity block (pairs,
 * tiles and K ranges wholly inside the padding are skipped); the last product and the output are d x d again.
 * workspace: model_lu_inverse_workspace bytes (eight dp x dp binary32 matrices), 16-byte aligned.  The two
 * triangular inversions run side by side, one of them on a stream the library owns, forked from and joined back
 * into `stream` inside the call. */
int model_lu_inverse_workspace(int64_t d, int64_t* bytes);
int model_lu_inverse(const float* lp, const float* up, const float* log_s, const float* sign_s, const int* perm, int64_t d,
                     int dtype, void* a_inv_out, void* workspace, void* stream);
/* The same three operations for MANY SMALL matrices in one launch each (the per-block transformations: one d x d
 * parameter set per transformer block, d the head dimension): `count` independent parameter sets stored one after
 * the other — lp, up [count][d][d], log_s, sign_s [count][d], perm [count][d] (each a permutation of 0..d-1) — and
 * results laid out the same way (a_out, a_inv_out, g: [count][d][d] in dtype; d_lp, d_up [count][d][d], d_log_s
 * [count][d] in binary32).  One workgroup owns one matrix, which lives in LDS; all arithmetic is binary32, only the
 * stored a_out / a_inv_out (and the given g) are in dtype.  1 <= d <= 128 (larger matrices take the calls above),
 * 1 <= count <= 2^20, no workspace, no alignment requirement beyond the element types'.  Same definitions, same
 * treatment of perm and of zeros in s as model_lu_compose / model_lu_backward / model_lu_inverse. */
int model_lu_compose_batch(const float* lp, const float* up, const float* log_s, const float* sign_s, const int* perm,
                           int64_t count, int64_t d, int dtype, void* a_out, void* stream);
int model_lu_backward_batch(const void* g, const float* lp, const float* up, const float* log_s, const float* sign_s,
                            const int* perm, int64_t count, int64_t d, int dtype, float* d_lp, float* d_up,
                            float* d_log_s, void* stream);
int model_lu_inverse_batch(const float* lp, const float* up, const float* log_s, const float* sign_s, const int* perm,
                           int64_t count, int64_t d, int dtype, void* a_inv_out, void* stream);
/* Measurement aid (not thread safe): returns in *gemm_ms / *launches (host, nullable) the time and count of the
 * matrix-core products model_lu_compose / model_lu_backward launched since the last call, then clears both and
 * switches the timing on (enable != 0) or off.  While it is on, every product is bracketed by HIP events on its
 * stream and waited for, so the calls become synchronous. */
int model_lu_timing(int enable, double* gemm_ms, int64_t* launches);

/* QR parametrisation of a learnable invertible matrix (Eq. 5 of the same section):
 *     Q = exp((G - G^T) / 2),   A = Q (R + diag(s)).
 * Free parameters (device, binary32 master copies): g [d][d] (only its skew-symmetric part acts), rp [d][d] of which
 * the strictly upper part is read, log_s, sign_s [d] as for the LU form.  The exponential is scaling and squaring
 * in binary32 on the matrix cores: X = S / 2^squarings, the Taylor polynomial of order 8 (evaluated in powers of X^3), then
 * `squarings` squarings; choose squarings with 2^squarings >= 2 ||S||_2 (5 covers ||S|| <= 16; 0 .. 16 accepted).
 * d: a multiple of 32, 32..16384.  workspace: model_qr_workspace bytes ((16 + 2 squarings) d x d binary32 matrices),
 * 16-byte aligned like every [d][d] array.
 * model_qr_compose   writes a_out = A [d][d] in dtype and leaves the intermediate matrices in the workspace.
 * model_qr_backward  given g_a = dLoss/dA [d][d] in dtype and THE SAME workspace, untouched since model_qr_compose
 *   ran on the same parameters, writes d_g [d][d] (skew-symmetric), d_rp [d][d] (strictly upper part, zero
 *   elsewhere) and d_log_s [d] in binary32.
 * model_qr_inverse   A^-1 = (R + diag s)^-1 Q^T into a_inv_out [d][d] in dtype: Q is read from qr_workspace (the
 *   workspace model_qr_compose left, same parameters and squarings), the triangular factor is inverted as in
 *   model_lu_inverse; d: a multiple of 128; workspace: model_lu_inverse_workspace(d) bytes. */
int model_qr_workspace(int64_t d, int squarings, int64_t* bytes);
/* The number of squarings model_qr_compose needs for the generator g: the smallest J with 2^J >= 2 ||S||_inf,
 * S = (G - G^T)/2 (the row-sum norm bounds the spectral norm of a skew-symmetric matrix), written to *squarings
 * (host).  model_qr_compose itself trusts its `squarings` argument: with too few the polynomial is evaluated
 * outside the range where its truncation error is at rounding level, and the result is an inaccurate (though
 * still nearly orthogonal) factor without any error being reported — call this when the norm of the generator
 * is not known to be small.  SYNCHRONOUS, unlike the other calls: it runs three small kernels on `stream`, waits
 * for them and reads one float back.  workspace: at least model_qr_workspace(d, 0) bytes (contents destroyed).
 * AE_EINVAL when the generator holds a NaN / infinity or would need more than 16 squarings. */
int model_qr_squarings(const float* g, int64_t d, void* workspace, int* squarings, void* stream);
int model_qr_compose(const float* g, const float* rp, const float* log_s, const float* sign_s, int64_t d, int dtype,
                     int squarings, void* a_out, void* workspace, void* stream);
int model_qr_backward(const void* g_a, const float* rp, const float* log_s, const float* sign_s, int64_t d, int dtype,
                      int squarings, float* d_g, float* d_rp, float* d_log_s, void* workspace, void* stream);
int model_qr_inverse(const float* rp, const float* log_s, const float* sign_s, int64_t d, int dtype, int squarings,
                     const void* qr_workspace, void* a_inv_out, void* workspace, void* stream);

/* Folding of affine transformations T(x) = A x + v into a linear layer f(x) = W x + b (the paper's appendix
 * "Folding & Transformation Structure"): the layer x -> T_l(f(T_r^-1(x))) has
 *     w_out = A_l W A_r^-1 ,   b_out = A_l b - w_out v_r + v_l .
 * w, w_out: [out][in] row-major in dtype (AE_F32 / AE_BF16), device, distinct; b (nullable = zero), b_out: binary32
 * [out].  a_left (nullable): [p][p] in dtype, applied to every group of p output features (p divides out; p = out:
 * one matrix for the whole side), v_left (nullable, needs a_left): binary32 [p], replicated.  a_right_inv (nullable):
 * the INVERSE matrix A_r^-1 [q][q] in dtype, applied to every group of q input features; v_right (nullable, needs
 * a_right_inv): binary32 [q], the shift of T_r, replicated.  p, q: multiples of 32 (bf16) / 16 (fp32), at least 32.
 * Products on the matrix cores with binary32 accumulation, each rounded to dtype; the bias uses the stored w_out.
 * workspace: model_fold_workspace bytes; matrices and workspace 16-byte aligned.  AE_EINVAL otherwise.
 * model_fold_embedding: every row w_j of the table e [vocab][d] becomes A w_j + v (a [d][d] in dtype, v binary32
 * [d] or null), written to e_out (distinct from e). */
int model_fold_workspace(int64_t out, int64_t in, int64_t p, int64_t q, int dtype, int64_t* bytes);
int model_fold_linear(const void* w, const float* b, int64_t out, int64_t in, const void* a_left, int64_t p,
                      const float* v_left, const void* a_right_inv, int64_t q, const float* v_right, int dtype,
                      void* w_out, float* b_out, void* workspace, void* stream);
int model_fold_embedding(const void* e, int64_t vocab, int64_t d, const void* a, const float* v, int dtype, void* e_out,
                         void* stream);

/* Measurement aid: TFLOP/s of a loop of nothing but independent 32x32x16 bf16 matrix-core
 * instructions on every compute unit (two workgroups of four wavefronts each, two wavefronts per
 * SIMD), the practical ceiling beside the nominal peak; with lds_reads = 6 each wavefront also reads
 * the six 16-byte fragments per lane that eight such instructions need in a 128x64 wave tile.
 * random_data = 0: every operand is 1.0; 1: operands with random signs, mantissas and exponents
 * (the shader clock under matrix-core load is power-managed and depends on the operand data).
 * Synchronous: times `iters` iterations with HIP events on `stream` and waits.  scratch_dev: at least
 * 2 KiB of 8-byte aligned device memory (its first 16 bytes are written).  shader_mhz (host, may be
 * null): the shader clock during the loop, from the kernel's cycle counter against its 100 MHz
 * wall clock.  lds_reads is 0 or 6, iters 1 .. 2^20: AE_EINVAL otherwise. */
int model_calibrate_mfma(int lds_reads, int random_data, int iters, float* scratch_dev, double* tflops,
                         double* shader_mhz, void* stream);

const char* model_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* AEMODEL_H */
