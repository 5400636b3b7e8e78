// ae_oracle.cpp — CPU oracle for the noisy-channel autoencoder hot path.
//
// THIS FILE IS TEST INFRASTRUCTURE.  It is a slow, plain, obviously-correct
// implementation of what the GPU library computes: every layer written as its
// textbook definition in naive loops with double-precision storage and
// accumulation.  Only tests, the smoke check and the benchmark's CPU-baseline
// leg may call it; the product path never does.  It shares no code, header,
// table or constant generator with the HIP sources.
//
// Source of each definition: the contract's statement of the pipeline
// (conv / fc encoder with batch-norm, ReLU, 2x2 max-pool; per-sample power
// normalisation; additive white Gaussian noise from a Philox counter-based
// generator at a requested SNR; nearest-upsampling conv / fc decoder; MSE
// loss) and its five workload descriptions.  The attached paper's text does
// not describe this pipeline, so each function below states the textbook
// definition it implements; the choices made where several definitions are
// possible are listed next to the functions.
//
// Pins (tests that tie this file to something other than itself):
//   philox4x32_10      published known-answer vectors of the generator
//   gauss_pair         double-precision libm Box-Muller on the same words,
//                      moments and a Kolmogorov-Smirnov test against Phi
//   conv / fc          identity and single-tap kernels, numpy brute force
//   bn                 zero mean / unit variance, affine invariance
//   pool / up          brute force, adjoint identity
//   pnorm              unit mean power, scale invariance
//   awgn               sample mean / variance against 10^(-snr/10)
//   backward (all)     central finite differences in double precision
//   mse                closed form on constant tensors
//
// Build: g++ -O2 -fopenmp -ffp-contract=off -shared -fPIC (see build.py).
// -ffp-contract=off matters: the u32 -> normal transform is defined as a fixed
// sequence of correctly rounded binary32 operations and must not be fused
// differently by the compiler.

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

// ---------------------------------------------------------------------------
// Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
// as 1, 2, 3", SC'11).  Ten rounds; the key is bumped by the Weyl constants
// between rounds (nine bumps).
// ---------------------------------------------------------------------------
void philox_block(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    if (round > 0) {
      k0 += 0x9E3779B9u;
      k1 += 0xBB67AE85u;
    }
    uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
    uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    uint32_t n1 = (uint32_t)p1;
    uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Counter layout used by the whole pipeline:
//   key     = (seed low word, seed high word)
//   counter = (sample low word, sample high word, quad index, stream)
// `sample` is the GLOBAL index of the sample (launch offset + index within the
// batch), `quad` selects four consecutive elements of that sample, `stream`
// separates uses: 0 = channel noise, 1 = Monte-Carlo message bits.
void philox_at(uint64_t seed, uint64_t sample, uint32_t quad, uint32_t stream, uint32_t out[4]) {
  uint32_t ctr[4] = {(uint32_t)sample, (uint32_t)(sample >> 32), quad, stream};
  uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  philox_block(ctr, key, out);
}

// ---------------------------------------------------------------------------
// Two 32-bit words -> two standard normal deviates (Box-Muller), defined as a
// fixed sequence of binary32 operations so that an independent implementation
// can reproduce it bit for bit.  Every arithmetic step below is a single
// correctly rounded IEEE operation (convert, fma, multiply, add, sqrt).
//
//   u     = fma(float(w0), 2^-32, 2^-33)                 in (0, 1]
//   ln u  : u = m * 2^e with m in [sqrt(1/2), sqrt(2)), f = m - 1 (exact),
//           ln(1+f) = f + f^2 * Q(f), Q a degree-8 polynomial (Horner, fma),
//           ln u = fma(float(e), LN2, ln(1+f))
//   rho   = sqrt(-2 * ln u)
//   angle : quadrant = top two bits of w1; t = next 24 bits * 2^-24 in [0,1)
//           is the fraction of a quarter turn.  r = min(t, 1 - t) (exact),
//           s = r * S(r^2) ~ sin(pi/2 r), c = C(r^2) ~ cos(pi/2 r); swapped if
//           t > 1/2; then rotated by the quadrant (exact sign / swap).
//   g0 = rho * cos, g1 = rho * sin.
// The polynomial coefficients are part of the definition (binary32 literals).
// ---------------------------------------------------------------------------
inline uint32_t f2u(float f) { uint32_t u; std::memcpy(&u, &f, 4); return u; }
inline float u2f(uint32_t u) { float f; std::memcpy(&f, &u, 4); return f; }

float ln_unit(float u) {  // u in (0, 1], normal numbers only (u >= 2^-33)
  uint32_t bits = f2u(u);
  int e = (int)(bits >> 23) - 127;
  uint32_t mant = bits & 0x007FFFFFu;
  float m = u2f(mant | 0x3F800000u);  // [1, 2)
  if (mant > 0x003504F3u) {           // m > sqrt(2): halve it (exact)
    m = m * 0.5f;
    e += 1;
  }
  float f = m - 1.0f;  // exact (Sterbenz)
  float q = -0x1.383e66p-4f;
  q = fmaf(q, f, 0x1.084e9p-3f);
  q = fmaf(q, f, -0x1.0f3778p-3f);
  q = fmaf(q, f, 0x1.227084p-3f);
  q = fmaf(q, f, -0x1.542744p-3f);
  q = fmaf(q, f, 0x1.99a402p-3f);
  q = fmaf(q, f, -0x1.000428p-2f);
  q = fmaf(q, f, 0x1.55555p-2f);
  q = fmaf(q, f, -0x1.fffff8p-2f);
  float f2 = f * f;
  float l1 = fmaf(f2, q, f);
  return fmaf((float)e, 0x1.62e43p-1f, l1);
}

void gauss_pair(uint32_t w0, uint32_t w1, float* g0, float* g1) {
  float u = fmaf((float)w0, 0x1p-32f, 0x1p-33f);
  float lnu = ln_unit(u);
  float rho = sqrtf(-2.0f * lnu);
  uint32_t quadrant = w1 >> 30;
  float t = (float)((w1 >> 6) & 0x00FFFFFFu) * 0x1p-24f;  // exact
  bool swap = t > 0.5f;
  float r = swap ? (1.0f - t) : t;  // exact, in [0, 1/2]
  float z = r * r;
  float sp = -0x1.2d9302p-8f;
  sp = fmaf(sp, z, 0x1.465e92p-4f);
  sp = fmaf(sp, z, -0x1.4abbbap-1f);
  sp = fmaf(sp, z, 0x1.921fb6p+0f);
  float s = r * sp;
  float c = 0x1.d99f54p-11f;
  c = fmaf(c, z, -0x1.55c4eap-6f);
  c = fmaf(c, z, 0x1.03c1dap-2f);
  c = fmaf(c, z, -0x1.3bd3ccp+0f);
  c = fmaf(c, z, 1.0f);
  if (swap) { float tmp = s; s = c; c = tmp; }
  float cq, sq;  // rotate by quadrant * 90 degrees
  switch (quadrant) {
    case 0: cq = c; sq = s; break;
    case 1: cq = -s; sq = c; break;
    case 2: cq = -c; sq = -s; break;
    default: cq = s; sq = -c; break;
  }
  *g0 = rho * cq;
  *g1 = rho * sq;
}

// The same map written with the mathematical definition in double precision
// (libm log / sin / cos): used only to pin gauss_pair to Box-Muller itself.
void gauss_pair_f64(uint32_t w0, uint32_t w1, double* g0, double* g1) {
  double u = ((double)w0 + 0.5) * 0x1p-32;
  double rho = std::sqrt(-2.0 * std::log(u));
  double turn = ((double)(w1 >> 30) + (double)((w1 >> 6) & 0x00FFFFFFu) * 0x1p-24) * 0.25;
  double ang = 2.0 * M_PI * turn;
  *g0 = rho * std::cos(ang);
  *g1 = rho * std::sin(ang);
}

// Standard-normal deviate for element i of global sample g (stream 0).
// Element i uses word pair (i&3)>>1 of quad i>>2: words (0,1) give elements
// 0,1 and words (2,3) give elements 2,3 of the quad.
float noise_element(uint64_t seed, uint64_t sample, int64_t i) {
  uint32_t w[4];
  philox_at(seed, sample, (uint32_t)(i >> 2), 0u, w);
  float a, b;
  int pair = (int)((i & 3) >> 1);
  gauss_pair(w[2 * pair], w[2 * pair + 1], &a, &b);
  return (i & 1) ? b : a;
}

// ---------------------------------------------------------------------------
// Network description
// ---------------------------------------------------------------------------
enum OpKind { OP_CONV, OP_BN, OP_RELU, OP_SIGMOID, OP_POOL2, OP_UP2, OP_FLATTEN, OP_FC, OP_RESHAPE, OP_PNORM, OP_AWGN };

struct Op {
  OpKind kind;
  int k = 0;           // conv kernel size (1 or 3)
  int cin = 0, hin = 0, win = 0;
  int cout = 0, hout = 0, wout = 0;
  int64_t param_off = 0;  // offset of this op's first parameter in the blob
};

struct Net {
  int batch = 0;
  int bn_mode = 0;  // 0 = batch statistics, 1 = stored (running) statistics
  // Storage-format emulation for the bfloat16 workloads ("bf16 storage, fp32 accumulate").
  // When set, every tensor the format stores is rounded to bfloat16 (nearest, ties to
  // even): the output of each conv / fc (bias included), the output of each maximal run
  // of bn / relu / sigmoid / pool2 ops, and the output of the pnorm / awgn run.  The
  // arithmetic in between stays in double.  This puts the discrete decisions that
  // depend on stored values (ReLU masks, max-pool winners) in the precision the format
  // prescribes, which is what a gradient comparison needs; without it the oracle is the
  // plain real-number definition.  The backward pass follows the same rule: the gradient
  // with respect to a stored tensor is itself a stored tensor of the format (the gradient
  // a layer hands to the layer before it), so it is rounded to bfloat16 too; gradients
  // with respect to parameters are not (they are returned in binary32 / double).
  int store_bf16 = 0;
  int c0 = 0, h0 = 0, w0 = 0;
  std::vector<Op> ops;
  int64_t n_params = 0;
  // state saved by forward (all double, NCHW): acts[0] = input, acts[i+1] = output of op i
  std::vector<std::vector<double>> acts;
  std::vector<std::vector<double>> bn_mean, bn_invstd;  // per op (empty unless BN)
  std::vector<double> pn_r;                             // per-sample r of the (single) pnorm
  bool have_forward = false;
  // Given decisions (oracle_set_decisions; empty = none).  A ReLU mask bit and a max-pool winner are discrete
  // decisions on forward values; two correct implementations whose forward values differ by rounding disagree
  // on a few of them, and the gradient is discontinuous there.  A test that wants to compare the ARITHMETIC of
  // two backward passes can therefore state the decisions: per op, one byte per element of the op's OUTPUT —
  // relu: 1 = the gradient passes; pool2: index 0..3 of the window element that receives the gradient, in the
  // scan order (0,0),(0,1),(1,0),(1,1).  The backward definitions are otherwise unchanged.
  std::vector<std::vector<uint8_t>> decisions;
};

bool parse_dims(const std::string& s, int* c, int* h, int* w) {
  return std::sscanf(s.c_str(), "%dx%dx%d", c, h, w) == 3 && *c > 0 && *h > 0 && *w > 0;
}

// Grammar: comma-separated tokens; the first must be in:CxHxW.
//   conv3:N conv1:N bn relu sigmoid pool2 up2 flatten fc:N reshape:CxHxW pnorm awgn
bool parse_spec(const char* spec, int batch, int bn_mode, Net* net) {
  net->batch = batch;
  net->bn_mode = bn_mode;
  std::string s(spec);
  std::vector<std::string> toks;
  size_t pos = 0;
  while (pos <= s.size()) {
    size_t q = s.find(',', pos);
    if (q == std::string::npos) q = s.size();
    std::string t = s.substr(pos, q - pos);
    // trim blanks
    size_t a = t.find_first_not_of(" \t\n"), b = t.find_last_not_of(" \t\n");
    if (a == std::string::npos) return false;
    toks.push_back(t.substr(a, b - a + 1));
    pos = q + 1;
  }
  if (toks.empty() || toks[0].rfind("in:", 0) != 0) return false;
  int c, h, w;
  if (!parse_dims(toks[0].substr(3), &c, &h, &w)) return false;
  net->c0 = c; net->h0 = h; net->w0 = w;
  int64_t off = 0;
  for (size_t i = 1; i < toks.size(); ++i) {
    const std::string& t = toks[i];
    Op op;
    op.cin = c; op.hin = h; op.win = w;
    op.cout = c; op.hout = h; op.wout = w;
    op.param_off = off;
    if (t.rfind("conv3:", 0) == 0 || t.rfind("conv1:", 0) == 0) {
      op.kind = OP_CONV;
      op.k = t[4] - '0';
      op.cout = std::atoi(t.c_str() + 6);
      if (op.cout <= 0) return false;
      off += (int64_t)op.cout * c * op.k * op.k + op.cout;
    } else if (t.rfind("fc:", 0) == 0) {
      if (h != 1 || w != 1) return false;
      op.kind = OP_FC;
      op.cout = std::atoi(t.c_str() + 3);
      if (op.cout <= 0) return false;
      off += (int64_t)op.cout * c + op.cout;
    } else if (t == "bn") {
      op.kind = OP_BN;
      off += (bn_mode == 1 ? 4 : 2) * (int64_t)c;
    } else if (t == "relu") {
      op.kind = OP_RELU;
    } else if (t == "sigmoid") {
      op.kind = OP_SIGMOID;
    } else if (t == "pool2") {
      if ((h & 1) || (w & 1)) return false;
      op.kind = OP_POOL2;
      op.hout = h / 2; op.wout = w / 2;
    } else if (t == "up2") {
      op.kind = OP_UP2;
      op.hout = 2 * h; op.wout = 2 * w;
    } else if (t == "flatten") {
      op.kind = OP_FLATTEN;
      op.cout = c * h * w; op.hout = 1; op.wout = 1;
    } else if (t.rfind("reshape:", 0) == 0) {
      op.kind = OP_RESHAPE;
      int rc, rh, rw;
      if (!parse_dims(t.substr(8), &rc, &rh, &rw)) return false;
      if ((int64_t)rc * rh * rw != (int64_t)c * h * w) return false;
      op.cout = rc; op.hout = rh; op.wout = rw;
    } else if (t == "pnorm") {
      op.kind = OP_PNORM;
    } else if (t == "awgn") {
      op.kind = OP_AWGN;
    } else {
      return false;
    }
    c = op.cout; h = op.hout; w = op.wout;
    net->ops.push_back(op);
  }
  net->n_params = off;
  return true;
}

// nearest bfloat16 (8 significant bits), ties to even; exact zero, inf and nan pass through
inline double round_bf16(double v) {
  if (v == 0.0 || !std::isfinite(v)) return v;
  int e;
  double m = std::frexp(v, &e);               // |m| in [0.5, 1)
  return std::ldexp(std::nearbyint(m * 256.0), e - 8);
}

inline bool is_pointwise_chain_op(OpKind k) { return k == OP_BN || k == OP_RELU || k == OP_SIGMOID || k == OP_POOL2; }

// does the storage format materialise the output of op i?
bool stored_output(const Net& net, size_t i) {
  const OpKind k = net.ops[i].kind;
  const bool has_next = i + 1 < net.ops.size();
  const OpKind nk = has_next ? net.ops[i + 1].kind : OP_CONV;
  if (k == OP_CONV || k == OP_FC || k == OP_AWGN) return true;
  if (is_pointwise_chain_op(k)) return !(has_next && is_pointwise_chain_op(nk));
  if (k == OP_PNORM) return !(has_next && nk == OP_AWGN);
  return false;  // up2 / flatten / reshape copy already-rounded values
}

inline int64_t vol(const Op& o, bool out) {
  return out ? (int64_t)o.cout * o.hout * o.wout : (int64_t)o.cin * o.hin * o.win;
}

// ---------------------------------------------------------------------------
// Forward definitions.  All tensors NCHW, double.
// ---------------------------------------------------------------------------

// Cross-correlation, stride 1, zero padding (k-1)/2, with bias:
//   y[n,co,h,w] = b[co] + sum_{ci,r,s} W[co,ci,r,s] * x[n,ci,h+r-p,w+s-p]
void conv_forward(const Op& o, int B, const float* W, const float* bias, const std::vector<double>& x,
                  std::vector<double>& y) {
  const int k = o.k, p = (k - 1) / 2, H = o.hin, Wd = o.win, Ci = o.cin, Co = o.cout;
  y.assign((size_t)B * Co * H * Wd, 0.0);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < B; ++n)
    for (int co = 0; co < Co; ++co)
      for (int h = 0; h < H; ++h)
        for (int w = 0; w < Wd; ++w) {
          double acc = (double)bias[co];
          for (int ci = 0; ci < Ci; ++ci)
            for (int r = 0; r < k; ++r) {
              int hh = h + r - p;
              if (hh < 0 || hh >= H) continue;
              for (int s = 0; s < k; ++s) {
                int ww = w + s - p;
                if (ww < 0 || ww >= Wd) continue;
                acc += (double)W[(((size_t)co * Ci + ci) * k + r) * k + s] *
                       x[(((size_t)n * Ci + ci) * H + hh) * Wd + ww];
              }
            }
          y[(((size_t)n * Co + co) * H + h) * Wd + w] = acc;
        }
}

// y[n,o] = b[o] + sum_i W[o,i] x[n,i]
void fc_forward(const Op& o, int B, const float* W, const float* bias, const std::vector<double>& x,
                std::vector<double>& y) {
  const int In = o.cin, Out = o.cout;
  y.assign((size_t)B * Out, 0.0);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < B; ++n)
    for (int j = 0; j < Out; ++j) {
      double acc = (double)bias[j];
      for (int i = 0; i < In; ++i) acc += (double)W[(size_t)j * In + i] * x[(size_t)n * In + i];
      y[(size_t)n * Out + j] = acc;
    }
}

// Batch normalisation over (n,h,w) per channel: biased variance, eps = 1e-5.
const double BN_EPS = 1e-5;
void bn_forward(const Op& o, int B, int mode, const float* prm, const std::vector<double>& x,
                std::vector<double>& y, std::vector<double>& mean, std::vector<double>& invstd) {
  const int C = o.cin;
  const int64_t HW = (int64_t)o.hin * o.win;
  const float* gamma = prm;
  const float* beta = prm + C;
  y.assign(x.size(), 0.0);
  mean.assign(C, 0.0);
  invstd.assign(C, 0.0);
#pragma omp parallel for schedule(static)
  for (int c = 0; c < C; ++c) {
    double mu, var;
    if (mode == 1) {
      mu = (double)prm[2 * C + c];
      var = (double)prm[3 * C + c];
    } else {
      double s = 0.0;
      for (int n = 0; n < B; ++n)
        for (int64_t i = 0; i < HW; ++i) s += x[((size_t)n * C + c) * HW + i];
      mu = s / (double)(B * HW);
      double v = 0.0;
      for (int n = 0; n < B; ++n)
        for (int64_t i = 0; i < HW; ++i) {
          double d = x[((size_t)n * C + c) * HW + i] - mu;
          v += d * d;
        }
      var = v / (double)(B * HW);
    }
    double is = 1.0 / std::sqrt(var + BN_EPS);
    mean[c] = mu;
    invstd[c] = is;
    for (int n = 0; n < B; ++n)
      for (int64_t i = 0; i < HW; ++i) {
        size_t idx = ((size_t)n * C + c) * HW + i;
        y[idx] = (double)gamma[c] * ((x[idx] - mu) * is) + (double)beta[c];
      }
  }
}

// 2x2 window, stride 2.  The window is scanned in the order (0,0),(0,1),(1,0),(1,1)
// and the first maximum wins (matters only for the backward routing of ties).
inline int pool_argmax(const double v[4]) {
  int best = 0;
  for (int i = 1; i < 4; ++i)
    if (v[i] > v[best]) best = i;
  return best;
}

void pool_forward(const Op& o, int B, const std::vector<double>& x, std::vector<double>& y) {
  const int C = o.cin, H = o.hin, W = o.win, Ho = o.hout, Wo = o.wout;
  y.assign((size_t)B * C * Ho * Wo, 0.0);
#pragma omp parallel for schedule(static)
  for (int64_t nc = 0; nc < (int64_t)B * C; ++nc)
    for (int i = 0; i < Ho; ++i)
      for (int j = 0; j < Wo; ++j) {
        const double* px = &x[(size_t)nc * H * W];
        double v[4] = {px[(2 * i) * W + 2 * j], px[(2 * i) * W + 2 * j + 1], px[(2 * i + 1) * W + 2 * j],
                       px[(2 * i + 1) * W + 2 * j + 1]};
        y[((size_t)nc * Ho + i) * Wo + j] = v[pool_argmax(v)];
      }
}

// Nearest-neighbour x2: out[c,2i+a,2j+b] = in[c,i,j], a,b in {0,1}.
void up_forward(const Op& o, int B, const std::vector<double>& x, std::vector<double>& y) {
  const int C = o.cin, H = o.hin, W = o.win, Ho = o.hout, Wo = o.wout;
  y.assign((size_t)B * C * Ho * Wo, 0.0);
#pragma omp parallel for schedule(static)
  for (int64_t nc = 0; nc < (int64_t)B * C; ++nc)
    for (int i = 0; i < Ho; ++i)
      for (int j = 0; j < Wo; ++j) y[((size_t)nc * Ho + i) * Wo + j] = x[((size_t)nc * H + i / 2) * W + j / 2];
}

// Power normalisation per sample over the whole latent vector of n elements:
//   r = sqrt(mean_i z_i^2),  x = z / r   (x = 0 when r = 0).
void pnorm_forward(int B, int64_t n, const std::vector<double>& z, std::vector<double>& x, std::vector<double>& r) {
  x.assign(z.size(), 0.0);
  r.assign(B, 0.0);
  for (int b = 0; b < B; ++b) {
    double s = 0.0;
    for (int64_t i = 0; i < n; ++i) s += z[(size_t)b * n + i] * z[(size_t)b * n + i];
    double rr = std::sqrt(s / (double)n);
    r[b] = rr;
    if (rr > 0.0)
      for (int64_t i = 0; i < n; ++i) x[(size_t)b * n + i] = z[(size_t)b * n + i] / rr;
  }
}

// Real AWGN channel on a unit-power signal: noise variance per element
// sigma^2 = 10^(-snr_db/10).  sigma is rounded to binary32 and the noise sample
// sigma * g is a binary32 product (so the noise tensor itself is reproducible
// bit for bit); the addition to the signal is done in double.
float sigma_from_snr(float snr_db) { return (float)std::pow(10.0, -(double)snr_db / 20.0); }

void awgn_forward(int B, int64_t n, float snr_db, uint64_t seed, uint64_t first_sample, const std::vector<double>& x,
                  std::vector<double>& y) {
  y.assign(x.size(), 0.0);
  const float sigma = sigma_from_snr(snr_db);
#pragma omp parallel for schedule(static)
  for (int b = 0; b < B; ++b)
    for (int64_t i = 0; i < n; ++i) {
      float g = noise_element(seed, first_sample + (uint64_t)b, i);
      float ns = sigma * g;
      y[(size_t)b * n + i] = x[(size_t)b * n + i] + (double)ns;
    }
}

// ---------------------------------------------------------------------------
// Backward definitions (adjoints of the above).
// ---------------------------------------------------------------------------
void conv_backward(const Op& o, int B, const float* W, const std::vector<double>& x, const std::vector<double>& dy,
                   std::vector<double>& dx, double* dW, double* db) {
  const int k = o.k, p = (k - 1) / 2, H = o.hin, Wd = o.win, Ci = o.cin, Co = o.cout;
  dx.assign((size_t)B * Ci * H * Wd, 0.0);
  // dW[co,ci,r,s] = sum_{n,h,w} dy[n,co,h,w] x[n,ci,h+r-p,w+s-p];  db[co] = sum dy
#pragma omp parallel for schedule(static)
  for (int co = 0; co < Co; ++co) {
    double sb = 0.0;
    for (int n = 0; n < B; ++n)
      for (int i = 0; i < H * Wd; ++i) sb += dy[((size_t)n * Co + co) * H * Wd + i];
    db[co] = sb;
    for (int ci = 0; ci < Ci; ++ci)
      for (int r = 0; r < k; ++r)
        for (int s = 0; s < k; ++s) {
          double acc = 0.0;
          for (int n = 0; n < B; ++n)
            for (int h = 0; h < H; ++h) {
              int hh = h + r - p;
              if (hh < 0 || hh >= H) continue;
              for (int w = 0; w < Wd; ++w) {
                int ww = w + s - p;
                if (ww < 0 || ww >= Wd) continue;
                acc += dy[(((size_t)n * Co + co) * H + h) * Wd + w] * x[(((size_t)n * Ci + ci) * H + hh) * Wd + ww];
              }
            }
          dW[(((size_t)co * Ci + ci) * k + r) * k + s] = acc;
        }
  }
  // dx[n,ci,hh,ww] = sum_{co,r,s} W[co,ci,r,s] dy[n,co,hh-r+p,ww-s+p]
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < B; ++n)
    for (int ci = 0; ci < Ci; ++ci)
      for (int hh = 0; hh < H; ++hh)
        for (int ww = 0; ww < Wd; ++ww) {
          double acc = 0.0;
          for (int co = 0; co < Co; ++co)
            for (int r = 0; r < k; ++r) {
              int h = hh - r + p;
              if (h < 0 || h >= H) continue;
              for (int s = 0; s < k; ++s) {
                int w = ww - s + p;
                if (w < 0 || w >= Wd) continue;
                acc += (double)W[(((size_t)co * Ci + ci) * k + r) * k + s] * dy[(((size_t)n * Co + co) * H + h) * Wd + w];
              }
            }
          dx[(((size_t)n * Ci + ci) * H + hh) * Wd + ww] = acc;
        }
}

void fc_backward(const Op& o, int B, const float* W, const std::vector<double>& x, const std::vector<double>& dy,
                 std::vector<double>& dx, double* dW, double* db) {
  const int In = o.cin, Out = o.cout;
  dx.assign((size_t)B * In, 0.0);
#pragma omp parallel for schedule(static)
  for (int j = 0; j < Out; ++j) {
    double sb = 0.0;
    for (int n = 0; n < B; ++n) sb += dy[(size_t)n * Out + j];
    db[j] = sb;
    for (int i = 0; i < In; ++i) {
      double acc = 0.0;
      for (int n = 0; n < B; ++n) acc += dy[(size_t)n * Out + j] * x[(size_t)n * In + i];
      dW[(size_t)j * In + i] = acc;
    }
  }
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < B; ++n)
    for (int i = 0; i < In; ++i) {
      double acc = 0.0;
      for (int j = 0; j < Out; ++j) acc += (double)W[(size_t)j * In + i] * dy[(size_t)n * Out + j];
      dx[(size_t)n * In + i] = acc;
    }
}

// With xh = (x-mu)*invstd, M = B*H*W:
//   dbeta = sum dy, dgamma = sum dy*xh
//   batch statistics : dx = gamma*invstd*(dy - dbeta/M - xh*dgamma/M)
//   stored statistics: dx = gamma*invstd*dy
void bn_backward(const Op& o, int B, int mode, const float* prm, const std::vector<double>& x,
                 const std::vector<double>& mean, const std::vector<double>& invstd, const std::vector<double>& dy,
                 std::vector<double>& dx, double* dprm) {
  const int C = o.cin;
  const int64_t HW = (int64_t)o.hin * o.win;
  const double M = (double)B * (double)HW;
  dx.assign(x.size(), 0.0);
#pragma omp parallel for schedule(static)
  for (int c = 0; c < C; ++c) {
    double sdy = 0.0, sdyx = 0.0;
    for (int n = 0; n < B; ++n)
      for (int64_t i = 0; i < HW; ++i) {
        size_t idx = ((size_t)n * C + c) * HW + i;
        double xh = (x[idx] - mean[c]) * invstd[c];
        sdy += dy[idx];
        sdyx += dy[idx] * xh;
      }
    dprm[c] = sdyx;      // dgamma
    dprm[C + c] = sdy;   // dbeta
    if (mode == 1) { dprm[2 * C + c] = 0.0; dprm[3 * C + c] = 0.0; }
    double g = (double)prm[c] * invstd[c];
    for (int n = 0; n < B; ++n)
      for (int64_t i = 0; i < HW; ++i) {
        size_t idx = ((size_t)n * C + c) * HW + i;
        double xh = (x[idx] - mean[c]) * invstd[c];
        dx[idx] = (mode == 1) ? g * dy[idx] : g * (dy[idx] - sdy / M - xh * sdyx / M);
      }
  }
}

void pool_backward(const Op& o, int B, const std::vector<double>& x, const std::vector<double>& dy,
                   std::vector<double>& dx, const std::vector<uint8_t>* given = nullptr) {
  const int C = o.cin, H = o.hin, W = o.win, Ho = o.hout, Wo = o.wout;
  dx.assign(x.size(), 0.0);
#pragma omp parallel for schedule(static)
  for (int64_t nc = 0; nc < (int64_t)B * C; ++nc)
    for (int i = 0; i < Ho; ++i)
      for (int j = 0; j < Wo; ++j) {
        const double* px = &x[(size_t)nc * H * W];
        double v[4] = {px[(2 * i) * W + 2 * j], px[(2 * i) * W + 2 * j + 1], px[(2 * i + 1) * W + 2 * j],
                       px[(2 * i + 1) * W + 2 * j + 1]};
        int a = given ? ((*given)[((size_t)nc * Ho + i) * Wo + j] & 3) : pool_argmax(v);
        dx[(size_t)nc * H * W + (2 * i + a / 2) * W + 2 * j + (a & 1)] = dy[((size_t)nc * Ho + i) * Wo + j];
      }
}

void up_backward(const Op& o, int B, const std::vector<double>& dy, std::vector<double>& dx) {
  const int C = o.cin, H = o.hin, W = o.win, Ho = o.hout, Wo = o.wout;
  dx.assign((size_t)B * C * H * W, 0.0);
#pragma omp parallel for schedule(static)
  for (int64_t nc = 0; nc < (int64_t)B * C; ++nc)
    for (int i = 0; i < Ho; ++i)
      for (int j = 0; j < Wo; ++j) dx[((size_t)nc * H + i / 2) * W + j / 2] += dy[((size_t)nc * Ho + i) * Wo + j];
}

// x = z/r, r = sqrt(mean z^2):  dz = (g - x * mean(g . x)) / r
void pnorm_backward(int B, int64_t n, const std::vector<double>& xout, const std::vector<double>& r,
                    const std::vector<double>& g, std::vector<double>& dz) {
  dz.assign(g.size(), 0.0);
  for (int b = 0; b < B; ++b) {
    if (!(r[b] > 0.0)) continue;
    double dot = 0.0;
    for (int64_t i = 0; i < n; ++i) dot += g[(size_t)b * n + i] * xout[(size_t)b * n + i];
    dot /= (double)n;
    for (int64_t i = 0; i < n; ++i) dz[(size_t)b * n + i] = (g[(size_t)b * n + i] - xout[(size_t)b * n + i] * dot) / r[b];
  }
}

}  // namespace

// ===========================================================================
// C interface (loaded through ctypes by tests / smoke / bench cpu_baseline)
// ===========================================================================
extern "C" {

void oracle_philox4x32_10(const uint32_t* ctr, const uint32_t* key, uint32_t* out) { philox_block(ctr, key, out); }

void oracle_gauss_pair(uint32_t w0, uint32_t w1, float* g) { gauss_pair(w0, w1, &g[0], &g[1]); }

void oracle_gauss_pair_f64(uint32_t w0, uint32_t w1, double* g) { gauss_pair_f64(w0, w1, &g[0], &g[1]); }

// Vectorised pins: n word pairs -> 2n deviates.
void oracle_gauss_many(const uint32_t* w, int64_t n, float* g32, double* g64) {
  for (int64_t i = 0; i < n; ++i) {
    gauss_pair(w[2 * i], w[2 * i + 1], &g32[2 * i], &g32[2 * i + 1]);
    if (g64) gauss_pair_f64(w[2 * i], w[2 * i + 1], &g64[2 * i], &g64[2 * i + 1]);
  }
}

// Standard-normal tensor [batch][n] for samples first_sample .. first_sample+batch-1.
void oracle_noise(uint64_t seed, uint64_t first_sample, int64_t batch, int64_t n, float* out) {
#pragma omp parallel for schedule(static)
  for (int64_t b = 0; b < batch; ++b)
    for (int64_t i = 0; i < n; ++i) out[b * n + i] = noise_element(seed, first_sample + (uint64_t)b, i);
}

float oracle_sigma(float snr_db) { return sigma_from_snr(snr_db); }

// Monte-Carlo message source: bit j of sample g is bit (j&31) of word (j>>5)&3
// of quad j>>7 of Philox stream 1; the symbol is +1 for a set bit, -1 otherwise.
void oracle_gen_bits(uint64_t seed, uint64_t first_sample, int64_t batch, int k, float* x_pm1) {
  for (int64_t b = 0; b < batch; ++b)
    for (int j = 0; j < k; ++j) {
      uint32_t w[4];
      philox_at(seed, first_sample + (uint64_t)b, (uint32_t)(j >> 7), 1u, w);
      uint32_t bit = (w[(j >> 5) & 3] >> (j & 31)) & 1u;
      x_pm1[b * k + j] = bit ? 1.0f : -1.0f;
    }
}

// Hard decision at 1/2 on the decoder output; a block is in error if any bit is.
void oracle_count_errors(const double* y, const float* x_pm1, int64_t batch, int k, uint64_t* bit_err,
                         uint64_t* blk_err) {
  uint64_t be = 0, ke = 0;
  for (int64_t b = 0; b < batch; ++b) {
    int any = 0;
    for (int j = 0; j < k; ++j) {
      int dec = y[b * k + j] > 0.5;
      int tx = x_pm1[b * k + j] > 0.0f;
      if (dec != tx) { ++be; any = 1; }
    }
    ke += any;
  }
  *bit_err = be;
  *blk_err = ke;
}

void* oracle_create(const char* spec, int batch, int bn_mode, int store_bf16) {
  Net* net = new Net();
  net->store_bf16 = store_bf16;
  if (batch <= 0 || !parse_spec(spec, batch, bn_mode, net)) {
    delete net;
    return nullptr;
  }
  return net;
}

void oracle_destroy(void* h) { delete (Net*)h; }

int64_t oracle_param_count(void* h) { return ((Net*)h)->n_params; }
int oracle_num_ops(void* h) { return (int)((Net*)h)->ops.size(); }

// shape[0..2] = output C,H,W of op i (i = -1: the network input); returns kind (or -1)
int oracle_op_info(void* h, int i, int64_t* shape, int64_t* param_off) {
  Net* net = (Net*)h;
  if (i == -1) { shape[0] = net->c0; shape[1] = net->h0; shape[2] = net->w0; *param_off = 0; return -1; }
  const Op& o = net->ops[i];
  shape[0] = o.cout; shape[1] = o.hout; shape[2] = o.wout;
  *param_off = o.param_off;
  return (int)o.kind;
}

// Forward pass.  params: float[n_params] in op order (conv: W[co][ci][k][k], b[co];
// fc: W[out][in], b[out]; bn: gamma[C], beta[C] (+ mean[C], var[C] when bn_mode = 1)).
// x: float NCHW.  y (nullable): double, shape of the last op's output.
int oracle_forward(void* h, const float* params, const float* x, float snr_db, uint64_t seed, uint64_t first_sample,
                   double* y) {
  Net* net = (Net*)h;
  const int B = net->batch;
  const size_t nops = net->ops.size();
  net->acts.assign(nops + 1, {});
  net->bn_mean.assign(nops, {});
  net->bn_invstd.assign(nops, {});
  size_t n_in = (size_t)B * net->c0 * net->h0 * net->w0;
  net->acts[0].resize(n_in);
  for (size_t i = 0; i < n_in; ++i) net->acts[0][i] = (double)x[i];
  for (size_t i = 0; i < nops; ++i) {
    const Op& o = net->ops[i];
    const std::vector<double>& in = net->acts[i];
    std::vector<double>& out = net->acts[i + 1];
    const float* prm = params + o.param_off;
    switch (o.kind) {
      case OP_CONV: conv_forward(o, B, prm, prm + (size_t)o.cout * o.cin * o.k * o.k, in, out); break;
      case OP_FC: fc_forward(o, B, prm, prm + (size_t)o.cout * o.cin, in, out); break;
      case OP_BN: bn_forward(o, B, net->bn_mode, prm, in, out, net->bn_mean[i], net->bn_invstd[i]); break;
      case OP_RELU:
        out.resize(in.size());
        for (size_t j = 0; j < in.size(); ++j) out[j] = in[j] > 0.0 ? in[j] : 0.0;
        break;
      case OP_SIGMOID:
        out.resize(in.size());
        for (size_t j = 0; j < in.size(); ++j) out[j] = 1.0 / (1.0 + std::exp(-in[j]));
        break;
      case OP_POOL2: pool_forward(o, B, in, out); break;
      case OP_UP2: up_forward(o, B, in, out); break;
      case OP_FLATTEN:
      case OP_RESHAPE: out = in; break;  // NCHW memory order is unchanged
      case OP_PNORM: pnorm_forward(B, vol(o, false), in, out, net->pn_r); break;
      case OP_AWGN: awgn_forward(B, vol(o, false), snr_db, seed, first_sample, in, out); break;
    }
    if (net->store_bf16 && stored_output(*net, i))
      for (size_t j = 0; j < out.size(); ++j) out[j] = round_bf16(out[j]);
  }
  net->have_forward = true;
  if (y) std::memcpy(y, net->acts[nops].data(), net->acts[nops].size() * sizeof(double));
  return 0;
}

// Copy the output of op i (i = -1: input) saved by the last forward.
int64_t oracle_get_activation(void* h, int i, double* out) {
  Net* net = (Net*)h;
  if (!net->have_forward || i < -1 || i + 1 >= (int)net->acts.size()) return -1;
  const std::vector<double>& a = net->acts[i + 1];
  if (out) std::memcpy(out, a.data(), a.size() * sizeof(double));
  return (int64_t)a.size();
}

// Backward pass through the graph of the last forward.  dy: double, shape of the
// output.  grads: double[n_params], same layout as params.  dx (nullable): gradient
// with respect to the input.
int oracle_backward(void* h, const float* params, const double* dy, double* grads, double* dx) {
  Net* net = (Net*)h;
  if (!net->have_forward) return -1;
  const int B = net->batch;
  const size_t nops = net->ops.size();
  std::vector<double> g(dy, dy + net->acts[nops].size());
  std::vector<double> gprev;
  for (int64_t i = 0; i < net->n_params; ++i) grads[i] = 0.0;
  for (size_t ii = nops; ii-- > 0;) {
    const Op& o = net->ops[ii];
    const std::vector<double>& in = net->acts[ii];
    const std::vector<double>& out = net->acts[ii + 1];
    const float* prm = params + o.param_off;
    double* gp = grads + o.param_off;
    switch (o.kind) {
      case OP_CONV: conv_backward(o, B, prm, in, g, gprev, gp, gp + (size_t)o.cout * o.cin * o.k * o.k); break;
      case OP_FC: fc_backward(o, B, prm, in, g, gprev, gp, gp + (size_t)o.cout * o.cin); break;
      case OP_BN: bn_backward(o, B, net->bn_mode, prm, in, net->bn_mean[ii], net->bn_invstd[ii], g, gprev, gp); break;
      case OP_RELU:  // derivative 0 for x <= 0
        gprev.resize(g.size());
        if (ii < net->decisions.size() && !net->decisions[ii].empty())
          for (size_t j = 0; j < g.size(); ++j) gprev[j] = net->decisions[ii][j] ? g[j] : 0.0;
        else
          for (size_t j = 0; j < g.size(); ++j) gprev[j] = in[j] > 0.0 ? g[j] : 0.0;
        break;
      case OP_SIGMOID:  // s'(x) = s(x)(1-s(x)), evaluated from the op's input (the stored output may be rounded)
        gprev.resize(g.size());
        for (size_t j = 0; j < g.size(); ++j) {
          double sg = 1.0 / (1.0 + std::exp(-in[j]));
          gprev[j] = g[j] * sg * (1.0 - sg);
        }
        break;
      case OP_POOL2:
        pool_backward(o, B, in, g, gprev, (ii < net->decisions.size() && !net->decisions[ii].empty()) ? &net->decisions[ii] : nullptr);
        break;
      case OP_UP2: up_backward(o, B, g, gprev); break;
      case OP_FLATTEN:
      case OP_RESHAPE: gprev = g; break;
      case OP_PNORM: pnorm_backward(B, vol(o, false), out, net->pn_r, g, gprev); break;
      case OP_AWGN: gprev = g; break;  // additive noise: identity
    }
    // storage-format emulation: gprev is the gradient w.r.t. this op's input, i.e. w.r.t. the output of op ii-1
    if (net->store_bf16 && (ii == 0 || stored_output(*net, ii - 1)))
      for (double& v : gprev) v = round_bf16(v);
    g.swap(gprev);
  }
  if (dx) std::memcpy(dx, g.data(), g.size() * sizeof(double));
  return 0;
}

// State the decisions of op i (relu: pass bits; pool2: winner indices; n = elements of the op's output) for the
// following oracle_backward calls; data = NULL withdraws them.  Returns 0, or -1 for a wrong op or size.
int oracle_set_decisions(void* h, int i, const uint8_t* data, int64_t n) {
  Net* net = (Net*)h;
  if (i < 0 || i >= (int)net->ops.size()) return -1;
  const Op& o = net->ops[i];
  if (o.kind != OP_RELU && o.kind != OP_POOL2) return -1;
  if (net->decisions.size() != net->ops.size()) net->decisions.assign(net->ops.size(), std::vector<uint8_t>());
  if (!data) { net->decisions[i].clear(); return 0; }
  if (n != (int64_t)net->batch * o.cout * o.hout * o.wout) return -1;
  net->decisions[i].assign(data, data + n);
  return 0;
}

// L = mean((y-t)^2) over all n elements; dy (nullable) = 2 (y-t) / n.
double oracle_loss_mse(const double* y, const double* t, int64_t n, double* dy) {
  double s = 0.0;
  for (int64_t i = 0; i < n; ++i) {
    double d = y[i] - t[i];
    s += d * d;
    if (dy) dy[i] = 2.0 * d / (double)n;
  }
  return s / (double)n;
}

// Number of OpenMP threads the loops may use from now on (timing only: results do not depend on it).
void oracle_set_num_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

}  // extern "C"
