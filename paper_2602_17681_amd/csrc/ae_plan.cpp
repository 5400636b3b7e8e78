// ae_plan.cpp — host-only: layer-spec parser, shape inference, fusion of spec
// tokens into executable steps, parameter-blob offsets and workspace sizing.
// No GPU call is made here, so model_describe works on a machine without a device.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>

#include "ae_internal.h"

namespace ae {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

const char* last_error() { return g_err; }

namespace {

enum TokKind { T_CONV, T_FC, T_BN, T_RELU, T_SIGMOID, T_POOL, T_UP, T_FLATTEN, T_RESHAPE, T_PNORM, T_AWGN };

struct Tok {
  TokKind kind;
  int a = 0, b = 0, c = 0;  // conv: k, cout; fc: cout; reshape: c,h,w
};

// a positive decimal integer of at most 9 digits (so it fits an int with room to spare), nothing else
bool read_int(const std::string& s, int* v) {
  if (s.empty() || s.size() > 9) return false;
  int64_t acc = 0;
  for (char ch : s) {
    if (ch < '0' || ch > '9') return false;
    acc = acc * 10 + (ch - '0');
  }
  *v = (int)acc;
  return acc > 0;
}

// "CxHxW": three such integers
bool read_dims(const std::string& s, int* c, int* h, int* w) {
  const size_t p1 = s.find('x');
  if (p1 == std::string::npos) return false;
  const size_t p2 = s.find('x', p1 + 1);
  if (p2 == std::string::npos) return false;
  return read_int(s.substr(0, p1), c) && read_int(s.substr(p1 + 1, p2 - p1 - 1), h) && read_int(s.substr(p2 + 1), w);
}

// Every tensor of a model (activations of the whole batch, weights of a layer) must stay below 2 GiB in
// binary32: the kernels index elements with 32-bit integers and address memory through 32-bit buffer ranges.
constexpr int64_t kMaxTensorElems = ((int64_t)1 << 29) - 1;
bool tensor_fits(int64_t batch, int64_t c, int64_t h, int64_t w) {
  if (c > kMaxTensorElems || h > kMaxTensorElems || w > kMaxTensorElems) return false;
  const int64_t hw = h * w;                       // < 2^58
  if (hw > kMaxTensorElems) return false;
  const int64_t chw = c * hw;                     // < 2^58
  if (chw > kMaxTensorElems) return false;
  return batch * chw <= kMaxTensorElems;          // batch < 2^31: < 2^60
}

int tokenize(const char* spec, int* c0, int* h0, int* w0, std::vector<Tok>* toks) {
  if (!spec) return fail(AE_EINVAL, "layer_spec is null");
  std::vector<std::string> parts;
  std::string cur;
  for (const char* p = spec;; ++p) {
    if (*p == ',' || *p == 0) {
      size_t a = cur.find_first_not_of(" \t\r\n");
      size_t b = cur.find_last_not_of(" \t\r\n");
      if (a == std::string::npos) return fail(AE_ESPEC, "empty token in layer spec");
      parts.push_back(cur.substr(a, b - a + 1));
      cur.clear();
      if (*p == 0) break;
    } else {
      cur.push_back(*p);
    }
  }
  if (parts.empty() || parts[0].compare(0, 3, "in:") != 0 || !read_dims(parts[0].substr(3), c0, h0, w0))
    return fail(AE_ESPEC, "layer spec must start with in:CxHxW");
  for (size_t i = 1; i < parts.size(); ++i) {
    const std::string& t = parts[i];
    Tok k;
    if (t.compare(0, 6, "conv3:") == 0 || t.compare(0, 6, "conv1:") == 0) {
      k.kind = T_CONV;
      k.a = t[4] - '0';
      if (!read_int(t.substr(6), &k.b)) return fail(AE_ESPEC, "bad channel count in '%s'", t.c_str());
    } else if (t.compare(0, 3, "fc:") == 0) {
      k.kind = T_FC;
      if (!read_int(t.substr(3), &k.b)) return fail(AE_ESPEC, "bad width in '%s'", t.c_str());
    } else if (t.compare(0, 8, "reshape:") == 0) {
      k.kind = T_RESHAPE;
      if (!read_dims(t.substr(8), &k.a, &k.b, &k.c)) return fail(AE_ESPEC, "bad shape in '%s'", t.c_str());
    } else if (t == "bn") k.kind = T_BN;
    else if (t == "relu") k.kind = T_RELU;
    else if (t == "sigmoid") k.kind = T_SIGMOID;
    else if (t == "pool2") k.kind = T_POOL;
    else if (t == "up2") k.kind = T_UP;
    else if (t == "flatten") k.kind = T_FLATTEN;
    else if (t == "pnorm") k.kind = T_PNORM;
    else if (t == "awgn") k.kind = T_AWGN;
    else return fail(AE_ESPEC, "unknown token '%s'", t.c_str());
    toks->push_back(k);
  }
  return AE_OK;
}

int64_t align_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

}  // namespace

int build_plan(const char* spec, int batch, int dtype, int bn_mode, Plan* plan) {
  if (batch <= 0) return fail(AE_EINVAL, "batch must be positive");
  if (dtype != AE_F32 && dtype != AE_BF16) return fail(AE_EINVAL, "dtype must be AE_F32 or AE_BF16");
  if (bn_mode != 0 && bn_mode != 1) return fail(AE_EINVAL, "bn_mode must be 0 or 1");
  std::vector<Tok> toks;
  int c, h, w;
  AE_TRY(tokenize(spec, &c, &h, &w, &toks));
  if (toks.empty()) return fail(AE_ESPEC, "layer spec has no layers");
  plan->batch = batch; plan->dtype = dtype; plan->bn_mode = bn_mode;
  if (!tensor_fits(batch, c, h, w)) return fail(AE_ESHAPE, "the input tensor of the batch exceeds 2 GiB");
  plan->c0 = c; plan->h0 = h; plan->w0 = w;
  plan->steps.clear();
  int64_t off = 0;
  const int64_t B = batch;

  auto add_transpose = [&](int rows, int cols, int last_token, int oc, int oh, int ow) {
    Step st;
    st.kind = ST_TRANSPOSE;
    st.last_token = last_token;
    st.cin = c; st.hin = h; st.win = w;
    st.cout = oc; st.hout = oh; st.wout = ow;
    st.t_rows = rows; st.t_cols = cols;
    plan->steps.push_back(st);
  };

  // boundary NCHW -> stored NHWC
  if (c > 1 && h * w > 1) add_transpose(c, h * w, -1, c, h, w);

  bool seen_param_step = false;
  size_t i = 0;
  while (i < toks.size()) {
    const Tok& t = toks[i];
    if (t.kind == T_UP || t.kind == T_CONV || t.kind == T_FC) {
      Step st;
      st.kind = ST_CONV;
      st.cin = c; st.hin = h; st.win = w;
      size_t j = i;
      if (t.kind == T_UP) {
        st.up = 1;
        ++j;
        if (j >= toks.size() || toks[j].kind != T_CONV)
          return fail(AE_ESPEC, "up2 must be followed by conv1/conv3");
      }
      const Tok& cv = toks[j];
      if (cv.kind == T_FC) {
        if (h != 1 || w != 1) return fail(AE_ESHAPE, "fc needs a flattened input (use flatten first)");
        st.k = 1;
      } else {
        if (cv.a != 1 && cv.a != 3) return fail(AE_ESPEC, "only conv1 and conv3 exist");
        st.k = cv.a;
      }
      st.cout = cv.b;
      if (!tensor_fits(batch, std::max(st.cin, st.cout), (int64_t)h << st.up, (int64_t)w << st.up) ||
          !tensor_fits(1, st.cout, st.cin, st.k * st.k))
        return fail(AE_ESHAPE, "token %d: an activation or weight tensor of this layer exceeds 2 GiB", (int)j);
      st.hc = h << st.up; st.wc = w << st.up;
      st.w_off = off;
      off += (int64_t)st.cout * st.cin * st.k * st.k;
      st.b_off = off;
      off += st.cout;
      ++j;
      if (j < toks.size() && toks[j].kind == T_BN) {
        st.has_bn = 1;
        st.bn_off = off;
        off += (int64_t)(bn_mode == 1 ? 4 : 2) * st.cout;
        ++j;
      }
      if (j < toks.size() && (toks[j].kind == T_RELU || toks[j].kind == T_SIGMOID)) {
        st.act = toks[j].kind == T_RELU ? ACT_RELU : ACT_SIGMOID;
        ++j;
      }
      if (j < toks.size() && toks[j].kind == T_POOL) {
        if ((st.hc & 1) || (st.wc & 1)) return fail(AE_ESHAPE, "pool2 needs even height and width");
        st.pool = 1;
        ++j;
      }
      st.hout = st.hc >> st.pool; st.wout = st.wc >> st.pool;
      st.last_token = (int)j - 1;
      st.needs_dx = seen_param_step;
      seen_param_step = true;
      c = st.cout; h = st.hout; w = st.wout;
      plan->steps.push_back(st);
      i = j;
    } else if (t.kind == T_FLATTEN) {
      if (c > 1 && h * w > 1) add_transpose(h * w, c, (int)i, c * h * w, 1, 1);
      else if (!plan->steps.empty()) plan->steps.back().last_token = (int)i;
      c = c * h * w; h = 1; w = 1;
      ++i;
    } else if (t.kind == T_RESHAPE) {
      if (h != 1 || w != 1) return fail(AE_ESPEC, "reshape needs a flattened input");
      if (!tensor_fits(batch, t.a, t.b, t.c) || (int64_t)t.a * t.b * t.c != (int64_t)c)
        return fail(AE_ESHAPE, "reshape changes the element count");
      if (t.a > 1 && t.b * t.c > 1) add_transpose(t.a, t.b * t.c, (int)i, t.a, t.b, t.c);
      else if (!plan->steps.empty()) plan->steps.back().last_token = (int)i;
      c = t.a; h = t.b; w = t.c;
      ++i;
    } else if (t.kind == T_PNORM || t.kind == T_AWGN) {
      Step st;
      st.kind = ST_CHANNEL;
      st.cin = st.cout = c; st.hin = st.hout = h; st.win = st.wout = w;
      size_t j = i;
      if (toks[j].kind == T_PNORM) { st.do_pnorm = 1; ++j; }
      if (j < toks.size() && toks[j].kind == T_AWGN) { st.do_awgn = 1; ++j; }
      st.last_token = (int)j - 1;
      plan->latent_n = (int64_t)c * h * w;
      plan->steps.push_back(st);
      i = j;
    } else {
      return fail(AE_ESPEC, "token %d (bn/relu/sigmoid/pool2) must follow a conv or fc", (int)i);
    }
  }
  if (plan->steps.empty()) return fail(AE_ESPEC, "layer spec has no layers");
  plan->cl = c; plan->hl = h; plan->wl = w;
  // stored NHWC -> boundary NCHW
  if (c > 1 && h * w > 1) add_transpose(h * w, c, (int)toks.size() - 1, c, h, w);
  plan->n_params = off;

  // ---- thin first / last layer: the planar boundary tensor is read / written by the conv itself
  {
    std::vector<Step>& S = plan->steps;
    int fc = -1, lc = -1;
    for (size_t q = 0; q < S.size(); ++q)
      if (S[q].kind == ST_CONV) { if (fc < 0) fc = (int)q; lc = (int)q; }
    if (fc >= 0 && (fc == 0 || (fc == 1 && S[0].kind == ST_TRANSPOSE && S[0].last_token == -1))) {
      Step& st = S[fc];
      if (st.cin <= 4 && thin_in_supported(st.cin, st.cout, st.k, st.up)) {
        st.thin = 1;
        if (fc == 1) { S.erase(S.begin()); --lc; }
      }
    }
    if (lc >= 0) {
      const bool tail_ok = lc == (int)S.size() - 1 || (lc == (int)S.size() - 2 && S.back().kind == ST_TRANSPOSE);
      Step& st = S[lc];
      if (tail_ok && st.thin == 0 && !st.has_bn && !st.pool && st.cout <= 4 && thin_out_supported(st.cout, st.cin, st.k, dtype) &&
          thin_in_supported(st.cout, st.cin, st.k, 0)) {
        st.thin = 2;
        st.out_planar = true;
        if (lc == (int)S.size() - 2) { st.last_token = S.back().last_token; S.pop_back(); }
      }
    }
  }

  // ---- workspace layout ---------------------------------------------------
  const int64_t es = (int64_t)dtype_size(dtype);
  int64_t total = 0;
  auto take = [&](int64_t bytes) {
    int64_t at = total;
    total += align_up(bytes > 0 ? bytes : 4, 256);
    return at;
  };
  plan->max_act_elems = B * plan->c0 * plan->h0 * plan->w0;
  plan->max_raw_elems = plan->max_full_elems = plan->max_partial_floats = plan->max_wgrad_floats = plan->max_splitk_floats = 0;
  plan->max_wgrad_inorder_floats = 0;
  for (Step& st : plan->steps) {
    int64_t out_elems = B * st.cout * st.hout * st.wout;
    int64_t in_elems = B * st.cin * st.hin * st.win;
    plan->max_act_elems = std::max(plan->max_act_elems, std::max(out_elems, in_elems));
    st.off_out = take(out_elems * es);
    if (st.kind == ST_CONV) {
      int64_t rows = B * st.hc * st.wc;
      int64_t raw_elems = rows * st.cout;
      plan->max_raw_elems = std::max(plan->max_raw_elems, raw_elems);
      if (st.has_bn || st.pool) st.off_raw = take(raw_elems * es);
      else if (st.act == ACT_SIGMOID && dtype == AE_BF16) st.off_aux = take(raw_elems * 4);
      plan->max_full_elems = std::max(plan->max_full_elems, rows * st.cin);
      int64_t wel = (int64_t)st.cout * st.cin * st.k * st.k;
      // thin layers keep their weights repacked as MFMA operand rows of the wide side
      // (the summed-weight forms of an upsampled 3x3 conv hold 16 taps instead of 9)
      const int64_t wpk = (st.up && st.k == 3 ? (int64_t)16 * st.cout * st.cin : wel) * es;
      st.off_wpack = take(std::max(wpk, st.thin == 1 ? thin_wfrag_bytes(st.cout)
                                        : st.thin == 2 ? thin_out_wz_bytes(st.cout, st.cin) : (int64_t)0));
      st.off_wpack_d = take(std::max(wpk, st.thin == 2 ? thin_wfrag_bytes(st.cin) : (int64_t)0));
      if (st.has_bn) st.off_bn = take(6 * (int64_t)st.cout * 4);
      int64_t blocks = std::max<int64_t>((rows + 127) / 128, reduce_blocks(rows));  // finest partial-sum granularity
      if (st.thin == 1) blocks = std::max<int64_t>(blocks, thin_in_mfma_blocks(batch, st.hc, st.wc));
      plan->max_partial_floats = std::max(plan->max_partial_floats, blocks * 2 * std::max(st.cout, st.cin));
      WgradArgs wa;
      wa.x = wa.dy = nullptr; wa.dw_canonical = nullptr;
      wa.n = batch; wa.hc = st.hc; wa.wc = st.wc; wa.cin = st.cin; wa.cout = st.cout; wa.k = st.k; wa.up = st.up;
      wa.dtype = dtype;
      if (st.thin == 0) {
        // split-K scratch of the forward conv and of the conv that yields the input gradient
        ConvArgs ca;
        ca.x = ca.w = nullptr; ca.bias = nullptr; ca.y = nullptr; ca.partial = nullptr; ca.y_aux = nullptr;
        ca.n = batch; ca.hc = st.hc; ca.wc = st.wc; ca.cin = st.cin; ca.cout = st.cout; ca.k = st.k; ca.up = st.up;
        ca.act = ACT_NONE; ca.dtype = dtype;
        if (!st.has_bn) plan->max_splitk_floats = std::max(plan->max_splitk_floats, conv_mfma_splitk_floats(ca));
        ca.cin = st.cout; ca.cout = st.cin; ca.up = 0;
        plan->max_splitk_floats = std::max(plan->max_splitk_floats, conv_mfma_splitk_floats(ca));
        if (st.up && conv_up_dgrad_usable(ca)) {
          ca.geom = CONV_UP_DGRAD;
          plan->max_splitk_floats = std::max(plan->max_splitk_floats, conv_mfma_splitk_floats(ca));
        }
      }
      if (st.thin == 1) {
        plan->max_wgrad_floats = std::max(plan->max_wgrad_floats, thin_wgrad_workspace_floats(rows, st.cin, st.cout));
        if (thin_wgrad_mfma_supported(st.cin, st.cout, st.wc, dtype))
          plan->max_wgrad_floats = std::max(plan->max_wgrad_floats,
                                            thin_wgrad_mfma_workspace_floats(batch, st.hc, st.wc, st.cout));
      }
      else if (st.thin == 2) {
        plan->max_wgrad_floats = std::max(plan->max_wgrad_floats,
                                          thin_wgrad_workspace_floats(B * st.hin * st.win, st.cout, st.cin));
        if (thin_wgrad_mfma_supported(st.cout, st.cin, st.win, dtype))
          plan->max_wgrad_floats = std::max(plan->max_wgrad_floats,
                                            thin_wgrad_mfma_workspace_floats(batch, st.hin, st.win, st.cin));
      }
      else if (wgrad_mfma_supported(wa))
        plan->max_wgrad_floats = std::max(plan->max_wgrad_floats, wgrad_mfma_workspace_floats(wa));
      else
        plan->max_wgrad_floats = std::max(plan->max_wgrad_floats, wgrad_direct_workspace_floats(wa));
      // a layer without batch-norm, activation or pooling has no conv-output gradient buffer of its own: its
      // weight gradient runs in order on the caller's stream, with scratch apart from the side stream's
      if (!st.has_bn && !st.pool && st.act == ACT_NONE && st.thin == 0)
        plan->max_wgrad_inorder_floats = std::max(plan->max_wgrad_inorder_floats,
                                                  wgrad_mfma_supported(wa) ? wgrad_mfma_workspace_floats(wa)
                                                                           : wgrad_direct_workspace_floats(wa));
      if (st.thin == 2)
        plan->max_partial_floats = std::max(plan->max_partial_floats,
                                            B * plane_sums_split((int64_t)st.hc * st.wc) * 2 * (int64_t)st.cout);
    }
  }
  plan->off_grad_a = take(plan->max_act_elems * es);      // gradient ping-pong
  plan->off_grad_b = take(plan->max_act_elems * es);
  plan->off_draw = take(plan->max_raw_elems * es);        // gradient at conv resolution (two buffers: consecutive
  plan->off_draw2 = take(plan->max_raw_elems * es);       // layers alternate, see the side stream of the backward pass)
  plan->off_dfull = take(plan->max_full_elems * es);      // input gradient before the 2x2 sum of an upsampled conv
  plan->off_partial = take(plan->max_partial_floats * 4);
  plan->off_wgrad = take(plan->max_wgrad_floats * 4);
  plan->off_wgrad_inorder = take(plan->max_wgrad_inorder_floats * 4);
  plan->off_splitk = take(plan->max_splitk_floats * 4);
  plan->ws_bytes = total;
  return AE_OK;
}

}  // namespace ae
