// ae_api.hip — the exported C functions: model lifetime, and the host-side
// executor that walks the plan and enqueues one kernel sequence per step.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <map>
#include <new>
#include <string>
#include <utility>
#include <vector>

#include "ae_internal.h"

// Optional per-kernel timing: when enabled, every kernel launch of the executor is
// bracketed by two HIP events on the caller's stream; model_timing_read turns the
// pairs into accumulated milliseconds.  Slots are keyed by "<step>.<phase>.<kernel>".
//
// Backward pass, two streams.  The weight gradient of a layer is needed by nobody until the
// pass ends, while the input gradient and the elementwise kernels of the next layer form the
// critical path; the two kinds of work also want different resources (matrix cores vs. memory
// bandwidth).  The weight-gradient kernels therefore run on a second ("side") stream of the
// handle: forked by an event once the layer's conv-output gradient exists, joined by an event
// before that gradient's buffer is written again (two such buffers alternate between layers)
// and at the end of the pass.  With per-kernel timing enabled, or overlap switched off,
// everything runs on the caller's stream in program order.
struct TimeSlot {
  std::string name;
  double flops = 0.0, bytes = 0.0;  // algorithmic work of one launch
  std::vector<std::pair<hipEvent_t, hipEvent_t>> pending;
  double total_ms = 0.0;
  int64_t launches = 0;
};

struct ae_model {
  ae::Plan plan;
  bool timing = false;
  std::vector<TimeSlot> slots;
  std::map<std::string, int> slot_index;
  std::vector<hipEvent_t> free_events;
  char* ws = nullptr;
  void* grad_a = nullptr;
  void* grad_b = nullptr;
  void* draw = nullptr;            // the conv-output gradient buffer of the current layer ...
  void* draw_buf[2] = {nullptr, nullptr};   // ... one of these two, alternating
  int draw_sel = 0;
  void* dfull = nullptr;
  float* partial = nullptr;
  float* wgrad_ws = nullptr;       // used on the side stream only (or on the caller's when not overlapping)
  float* wgrad_ws_inorder = nullptr;   // for the weight gradients that stay in order on the caller's stream
  float* splitk_ws = nullptr;
  bool overlap = true;
  hipStream_t side = nullptr;
  hipEvent_t ev_fork = nullptr;
  hipEvent_t ev_wdone[2] = {nullptr, nullptr};   // weight gradient reading draw_buf[i] has finished
  bool wpending[2] = {false, false};
  hipEvent_t ev_pack = nullptr;    // the weight repacking enqueued on the side stream has finished ...
  hipEvent_t ev_pack_fc = nullptr; // ... and that of the big fully-connected layers, which comes last
  bool pack_pending = false, pack_fc_pending = false;
  uint64_t first_sample = 0;
  bool have_forward = false;
  bool packed_in_batch = false;     // the current pass repacked all its weights with one launch
  bool inference = false;           // forward passes keep nothing for a backward pass (model_set_inference)
  bool fused_small = false;         // the plan has the shape of the three-launch small-image path
  ae::FusedSmall fused;
  bool params_static = false;       // the caller promises unchanged parameters: repack only once per direction
  const void* fwd_packed = nullptr; // parameter blob whose forward / input-gradient packing is still valid
  const void* bwd_packed = nullptr;
  bool fuse_bwd = true;             // ReLU backward / batch-norm backward sums in the epilogue of the kernel that produces the gradient (model_set_fused_backward)
  int pre_mode = 0;                 // what the input-gradient kernel of the layer above already did for the current layer:
  int pre_blocks = 0;               //   1: ReLU-masked gradient in the draw buffer, bias column sums in `partial` (pre_blocks row blocks);
                                    //   2: the two batch-norm backward sums in `partial`
  bool recompute = true;            // first-layer conv output recomputed instead of stored where the plan allows (model_set_recompute)
  const void* last_x = nullptr;     // input and parameters of the last forward pass: a first layer whose conv output is
  const void* last_params = nullptr; // recomputed rather than stored rebuilds it from these for model_get_conv_output
};

using namespace ae;

namespace {

class TimedScope {
 public:
  TimedScope(ae_model* m, hipStream_t s, int step, const char* tag, double flops, double bytes) : m_(m), s_(s) {
    if (!m->timing) return;
    char key[96];
    snprintf(key, sizeof(key), "step%02d.%s", step, tag);
    auto it = m->slot_index.find(key);
    if (it == m->slot_index.end()) {
      it = m->slot_index.emplace(key, (int)m->slots.size()).first;
      m->slots.emplace_back();
      m->slots.back().name = key;
    }
    slot_ = it->second;
    m->slots[slot_].flops = flops;
    m->slots[slot_].bytes = bytes;
    start_ = take();
    stop_ = take();
    if (start_ && stop_) (void)hipEventRecord(start_, s_);
  }
  ~TimedScope() {
    if (slot_ < 0 || !start_ || !stop_) return;
    (void)hipEventRecord(stop_, s_);
    m_->slots[slot_].pending.emplace_back(start_, stop_);
  }

 private:
  hipEvent_t take() {
    if (!m_->free_events.empty()) {
      hipEvent_t e = m_->free_events.back();
      m_->free_events.pop_back();
      return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
  }
  ae_model* m_;
  hipStream_t s_;
  int slot_ = -1;
  hipEvent_t start_ = nullptr, stop_ = nullptr;
};

#define TIMED_ON(stream, step, tag, flops, bytes, call)            \
  do {                                                              \
    TimedScope ts_(m, (stream), (step), (tag), (flops), (bytes));   \
    AE_TRY(call);                                                   \
  } while (0)
#define TIMED(step, tag, flops, bytes, call) TIMED_ON(s, step, tag, flops, bytes, call)

// Side stream of the backward pass: created on first use; null when the pass runs on one stream.
hipStream_t side_stream(ae_model* m) {
  if (!m->overlap || m->timing) return nullptr;
  if (!m->side) {
    if (hipStreamCreateWithFlags(&m->side, hipStreamNonBlocking) != hipSuccess) { m->side = nullptr; return nullptr; }
    bool ok = hipEventCreateWithFlags(&m->ev_fork, hipEventDisableTiming) == hipSuccess;
    for (int i = 0; i < 2 && ok; ++i) ok = hipEventCreateWithFlags(&m->ev_wdone[i], hipEventDisableTiming) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&m->ev_pack, hipEventDisableTiming) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&m->ev_pack_fc, hipEventDisableTiming) == hipSuccess;
    if (!ok) { m->overlap = false; return nullptr; }
  }
  return m->side;
}
// the caller's stream waits for the weight gradients still reading draw_buf[sel]
int join_side(ae_model* m, int sel, hipStream_t s) {
  if (m->wpending[sel]) {
    AE_HIP(hipStreamWaitEvent(s, m->ev_wdone[sel], 0));
    m->wpending[sel] = false;
  }
  return AE_OK;
}

int nblocks_for(int64_t rows) { return reduce_blocks(rows); }

// input tensor of step i: the previous step's saved output, or the caller's x
const void* step_input(const ae_model* m, size_t i, const void* x) { return i == 0 ? x : m->plan.steps[i - 1].out; }

// forward: does this conv step read repacked weights?
bool needs_fwd_pack(const Plan& P, const Step& st) {
  return st.kind == ST_CONV && st.thin == 0 && !(st.k == 1 && P.dtype == AE_F32 && !st.mfma);
}
bool needs_dgrad_pack(const Step& st) { return st.kind == ST_CONV && st.thin == 0 && st.needs_dx; }

// Repack the weights of every layer of a pass with one launch (more layers than a batch
// holds: the per-layer launches remain).
bool is_big_fc(const Step& st) { return st.k == 1 && (int64_t)st.cout * st.cin >= (1 << 20); }

// part 0: everything but the big fully-connected layers; part 1: those (they take long and are
// needed late in the forward pass, so they go last and get an event of their own)
int pack_all(ae_model* m, const float* params, bool dgrad, hipStream_t s, int part) {
  const Plan& P = m->plan;
  PackBatch pb;
  pb.n = 0;
  double bytes = 0.0;
  if (part == 0) m->packed_in_batch = false;
  for (const Step& st : P.steps) {
    const bool want = dgrad ? needs_dgrad_pack(st) : needs_fwd_pack(P, st);
    if (!want) continue;
    if ((part == 1) != (is_big_fc(st) && !(dgrad ? st.up_dgrad : st.up_phases))) continue;
    if (dgrad ? st.up_dgrad : st.up_phases) {
      // upsampled conv in its cheaper form: summed weights, a kernel of their own
      TIMED(0, dgrad ? "bwd.pack_weights_up" : "fwd.pack_weights_up", 0.0,
            (double)st.cout * st.cin * (36.0 + 16.0 * (double)dtype_size(P.dtype)),
            launch_pack_weights_up(params + st.w_off, dgrad ? st.wpack_d : st.wpack, st.cout, st.cin, P.dtype,
                                   dgrad ? CONV_UP_DGRAD : CONV_UP_PHASES, s));
      continue;
    }
    if (is_big_fc(st)) {
      // big fully-connected layers: bandwidth-bound conversion / transpose kernels of their own
      TIMED(0, dgrad ? "bwd.pack_weights_fc" : "fwd.pack_weights_fc", 0.0,
            (double)st.cout * st.cin * (4.0 + (double)dtype_size(P.dtype)),
            launch_pack_weights_1x1(params + st.w_off, dgrad ? st.wpack_d : st.wpack, st.cout, st.cin, P.dtype, dgrad, s));
      continue;
    }
    if (pb.n == kMaxPackJobs) return AE_OK;      // too many layers: fall back to per-layer packing
    PackJob& j = pb.job[pb.n++];
    j.w = params + st.w_off; j.wp = dgrad ? st.wpack_d : st.wpack;
    j.cout = st.cout; j.cin = st.cin; j.k = st.k; j.dgrad = dgrad ? 1 : 0; j.first_block = 0;
    j.frag = (dgrad ? st.wfrag_d : st.wfrag) ? 1 : 0;
    bytes += (double)st.cout * st.cin * st.k * st.k * (4.0 + (double)dtype_size(P.dtype));
  }
  if (pb.n > 0)
    TIMED(0, dgrad ? "bwd.pack_weights_all" : "fwd.pack_weights_all", 0.0, bytes, launch_pack_weights_batch(pb, P.dtype, s));
  if (part == 0) m->packed_in_batch = true;
  return AE_OK;
}

// The repacking of a pass's weights runs on the side stream, beside the first (thin) layer of
// the pass, which has a packing kernel of its own: forked after everything the caller's stream
// holds (the writers of params, the readers of the packed copies), joined before the first
// kernel that reads a packed copy and, at the latest, at the end of the pass.
int pack_all_beside(ae_model* m, const float* params, bool dgrad, hipStream_t s) {
  hipStream_t side = side_stream(m);
  if (!side) {
    AE_TRY(pack_all(m, params, dgrad, s, 0));
    return pack_all(m, params, dgrad, s, 1);
  }
  AE_HIP(hipEventRecord(m->ev_fork, s));
  AE_HIP(hipStreamWaitEvent(side, m->ev_fork, 0));
  AE_TRY(pack_all(m, params, dgrad, side, 0));
  AE_HIP(hipEventRecord(m->ev_pack, side));
  m->pack_pending = true;
  AE_TRY(pack_all(m, params, dgrad, side, 1));
  AE_HIP(hipEventRecord(m->ev_pack_fc, side));
  m->pack_fc_pending = true;
  return AE_OK;
}
// before the first kernel that reads a packed copy (big_fc: that of a big fully-connected layer)
int join_pack(ae_model* m, hipStream_t s, bool big_fc = false) {
  if (m->pack_pending) {
    AE_HIP(hipStreamWaitEvent(s, m->ev_pack, 0));
    m->pack_pending = false;
  }
  if (big_fc && m->pack_fc_pending) {
    AE_HIP(hipStreamWaitEvent(s, m->ev_pack_fc, 0));
    m->pack_fc_pending = false;
  }
  return AE_OK;
}

int forward_conv(ae_model* m, int si, Step& st, const float* params, const void* in, hipStream_t s) {
  const Plan& P = m->plan;
  if (st.thin == 0) AE_TRY(join_pack(m, s, is_big_fc(st)));
  const double es = (double)dtype_size(P.dtype);
  const int64_t rows = (int64_t)P.batch * st.hc * st.wc;
  const double wel = (double)st.cout * st.cin * st.k * st.k;
  const double in_el = (double)P.batch * st.cin * st.hin * st.win, raw_el = (double)rows * st.cout;
  const double out_el = (double)P.batch * st.cout * st.hout * st.wout;
  if (st.thin == 2) {
    if (thin_out_mfma_supported(st.cout, st.cin, st.k, P.dtype))
      TIMED(si, "fwd.conv_thin_out_mfma", 2.0 * raw_el * st.cin * st.k * st.k, (in_el + raw_el) * es,
            launch_thin_out_mfma(in, params + st.w_off, st.wpack, params + st.b_off, st.out, st.aux, P.batch, st.hc,
                                 st.wc, st.cout, st.cin, st.up, st.act, P.dtype, s));
    else
      TIMED(si, "fwd.conv_thin_out", 2.0 * raw_el * st.cin * st.k * st.k, (in_el + raw_el) * es,
            launch_thin_out_conv(in, params + st.w_off, params + st.b_off, st.out, st.aux, P.batch, st.hc, st.wc, st.cout,
                                 st.cin, st.up, st.act, P.dtype, s));
    return AE_OK;
  }
  const void* w = nullptr;
  if (st.thin == 1) {
    // canonical weights are read directly
  } else if (st.k == 1 && P.dtype == AE_F32 && !st.mfma) {
    w = params + st.w_off;  // [C_out][C_in] is already the packed order (the MFMA loader wants a 16-byte aligned copy)
  } else {
    if (!m->packed_in_batch) {
      if (st.up_phases)
        TIMED(si, "fwd.pack_weights_up", 0.0, wel * 4.0 + 16.0 * st.cout * st.cin * es,
              launch_pack_weights_up(params + st.w_off, st.wpack, st.cout, st.cin, P.dtype, CONV_UP_PHASES, s));
      else
        TIMED(si, "fwd.pack_weights", 0.0, wel * (4.0 + es),
              launch_pack_weights(params + st.w_off, st.wpack, st.cout, st.cin, st.k, P.dtype, false, s, st.wfrag));
    }
    w = st.wpack;
  }
  const bool second_pass = st.has_bn || st.pool;
  ConvArgs a;
  a.x = in; a.w = w; a.bias = params + st.b_off;
  a.y = second_pass ? st.raw : st.out;
  a.n = P.batch; a.hc = st.hc; a.wc = st.wc; a.cin = st.cin; a.cout = st.cout; a.k = st.k; a.up = st.up;
  a.act = second_pass ? ACT_NONE : st.act;
  a.dtype = P.dtype;
  a.partial = nullptr;
  a.y_aux = second_pass ? nullptr : st.aux;
  a.splitk_ws = m->splitk_ws;
  a.splitk_floats = P.max_splitk_floats;
  if (st.up_phases) a.geom = CONV_UP_PHASES;
  a.w_frag = st.wfrag;
  int nblk = 0;
  const double conv_flops = 2.0 * raw_el * st.cin * st.k * st.k;
  const double conv_bytes = (in_el + raw_el + wel) * es;
  if (st.recompute && m->recompute) {
    // statistics pass, finalize, then convolution + batch-norm + ReLU + pool in one kernel: the conv output stays on chip
    const float* gb = params + st.bn_off;
    const float* wsrc = params + st.w_off;
    if (P.bn_mode == 0) {
      TIMED(si, "fwd.thin_first_stats", conv_flops, in_el * es,
            launch_thin_first(0, in, wsrc, st.wpack, a.bias, nullptr, nullptr, nullptr, m->partial, nullptr, P.batch, st.hc,
                              st.wc, st.cin, st.cout, s));
      wsrc = nullptr;   // packed by the statistics pass
      TIMED(si, "fwd.bn_finalize", 0.0, (double)thin_first_blocks(P.batch, st.hc, st.wc, st.cout, 0) * 2 * st.cout * 4,
            launch_bn_finalize(m->partial, thin_first_blocks(P.batch, st.hc, st.wc, st.cout, 0), rows, st.cout, gb, nullptr, a.bias,
                               st.bn_vec, s));
    } else {
      TIMED(si, "fwd.bn_finalize", 0.0, 0.0,
            launch_bn_finalize(nullptr, 0, rows, st.cout, gb, gb + 2 * st.cout, nullptr, st.bn_vec, s));
    }
    TIMED(si, "fwd.thin_first_bn_act_pool", conv_flops, (in_el + out_el) * es,
          launch_thin_first(1, in, wsrc, st.wpack, a.bias, st.bn_vec, nullptr, st.out, nullptr, nullptr, P.batch, st.hc,
                            st.wc, st.cin, st.cout, s));
    return AE_OK;
  }
  if (st.thin == 1 && thin_in_mfma_supported(st.cin, st.cout, st.k, st.up, P.dtype) && !a.y_aux) {
    if (st.has_bn && P.bn_mode == 0) {
      a.partial = m->partial;
      nblk = thin_in_mfma_blocks(P.batch, st.hc, st.wc);
    }
    TIMED(si, "fwd.conv_thin_in_mfma", conv_flops, conv_bytes,
          launch_thin_in_mfma(in, params + st.w_off, st.wpack, a.bias, a.y, a.partial, P.batch, st.hc, st.wc, st.cin,
                              st.cout, 0, a.act, 0, P.dtype, s));
  } else if (st.thin == 1) {
    if (st.has_bn && P.bn_mode == 0) {
      a.partial = m->partial;
      nblk = (int)((rows + thin_in_partial_rows() - 1) / thin_in_partial_rows());
    }
    TIMED(si, "fwd.conv_thin_in", conv_flops, conv_bytes,
          launch_thin_in_conv(in, params + st.w_off, a.bias, a.y, a.partial, P.batch, st.hc, st.wc, st.cin, st.cout, 0,
                              a.act, P.dtype, s));
  } else if (st.mfma) {
    if (st.has_bn && P.bn_mode == 0) {
      a.partial = m->partial;
      const int pr = conv_partial_rows(a, true);
      nblk = (int)((rows + pr - 1) / pr);
    }
    // (slot FLOPs are the algorithmic ones of the definition; the four-phase form of an upsampled conv,
    // named apart, executes 4/9 of them)
    TIMED(si, st.up_phases ? "fwd.conv_mfma_phases" : "fwd.conv_mfma", conv_flops, conv_bytes, launch_conv_mfma(a, s));
  } else {
    TIMED(si, "fwd.conv_direct", conv_flops, conv_bytes, launch_conv_direct(a, s));
  }
  if (st.has_bn) {
    const float* gb = params + st.bn_off;
    if (P.bn_mode == 0) {
      const float* about = a.bias;    // the conv epilogues take their column statistics about the bias
      if (!a.partial) {
        TIMED(si, "fwd.col_stats", 0.0, raw_el * es, launch_col_stats(st.raw, rows, st.cout, P.dtype, m->partial, s));
        nblk = nblocks_for(rows);
        about = nullptr;
      }
      TIMED(si, "fwd.bn_finalize", 0.0, (double)nblk * 2 * st.cout * 4,
            launch_bn_finalize(m->partial, nblk, rows, st.cout, gb, nullptr, about, st.bn_vec, s));
    } else {
      TIMED(si, "fwd.bn_finalize", 0.0, 0.0,
            launch_bn_finalize(nullptr, 0, rows, st.cout, gb, gb + 2 * st.cout, nullptr, st.bn_vec, s));
    }
  }
  if (second_pass)
    TIMED(si, "fwd.bn_act_pool", 0.0, (raw_el + out_el) * es,
          launch_post_forward(st.raw, st.has_bn ? st.bn_vec : nullptr, st.out, P.batch, st.hc, st.wc, st.cout, st.act,
                              st.pool, P.dtype, s));
  return AE_OK;
}

int backward_conv(ae_model* m, int si, Step& st, const float* params, const void* in, const void* g, void* gnext,
                  float* grads, hipStream_t s) {
  const Plan& P = m->plan;
  const double es = (double)dtype_size(P.dtype);
  const int64_t rows = (int64_t)P.batch * st.hc * st.wc;
  const double wel = (double)st.cout * st.cin * st.k * st.k;
  const double in_el = (double)P.batch * st.cin * st.hin * st.win, raw_el = (double)rows * st.cout;
  const double out_el = (double)P.batch * st.cout * st.hout * st.wout;
  const double conv_flops = 2.0 * raw_el * st.cin * st.k * st.k;
  if (st.recompute && m->recompute) {
    // sums of the batch-norm backward and the weight gradient, each from the recomputed conv output; the
    // conv-output gradient exists only as LDS slabs inside the second kernel
    const int nb = thin_first_blocks(P.batch, st.hc, st.wc, st.cout, 2);
    TIMED(si, "bwd.thin_first_sums", conv_flops, (in_el + out_el) * es,
          launch_thin_first(2, in, nullptr, st.wpack, params + st.b_off, st.bn_vec, g, nullptr, m->partial, nullptr, P.batch,
                            st.hc, st.wc, st.cin, st.cout, s));
    TIMED(si, "bwd.bn_finalize", 0.0, 0.0,
          launch_bn_bwd_finalize(m->partial, nb, rows, st.cout, grads + st.b_off, st.bn_vec, grads + st.bn_off,
                                 P.bn_mode == 0, s));
    hipStream_t ws = s;
    hipStream_t side = side_stream(m);
    if (side) {
      AE_HIP(hipEventRecord(m->ev_fork, s));
      AE_HIP(hipStreamWaitEvent(side, m->ev_fork, 0));
      ws = side;
    } else {
      AE_TRY(join_side(m, 0, s));
      AE_TRY(join_side(m, 1, s));
    }
    TIMED_ON(ws, si, "bwd.thin_first_wgrad", 2.0 * conv_flops, (in_el + out_el) * es + wel * 4,
             launch_thin_first(3, in, nullptr, st.wpack, params + st.b_off, st.bn_vec, g, nullptr, m->wgrad_ws,
                               grads + st.w_off, P.batch, st.hc, st.wc, st.cin, st.cout, ws));
    if (ws != s) {
      AE_HIP(hipEventRecord(m->ev_wdone[m->draw_sel], ws));
      m->wpending[m->draw_sel] = true;
    }
    return AE_OK;   // the first layer needs no input gradient
  }
  const void* dr = g;  // gradient w.r.t. the conv output (bias included)
  bool bias_done = st.has_bn;   // a batch-norm step gets its bias gradient from bn_bwd_finalize
  const int pre = m->pre_mode;  // what the input-gradient kernel of the layer above already did for this layer
  m->pre_mode = 0;
  if ((st.has_bn || st.pool || st.act != ACT_NONE) && pre != 1) {
    // this layer's conv-output gradient goes to the other buffer than the previous layer's, and
    // only after the weight gradient that read this buffer two layers ago has finished
    m->draw_sel ^= 1;
    m->draw = m->draw_buf[m->draw_sel];
    AE_TRY(join_side(m, m->draw_sel, s));
  }
  if (st.has_bn || st.pool) {
    if (st.has_bn) {
      const int64_t prow = (int64_t)P.batch * st.hout * st.wout;
      if (pre == 2) {
        // the sums came out of the epilogue that wrote g (channels of scale 0 are redone by the finalize kernel)
        TIMED(si, "bwd.bn_finalize", 0.0, 0.0,
              launch_bn_bwd_finalize(m->partial, m->pre_blocks, rows, st.cout, grads + st.b_off, st.bn_vec,
                                     grads + st.bn_off, P.bn_mode == 0, s, st.raw, g, P.batch, st.hc, st.wc, st.pool));
      } else {
        TIMED(si, "bwd.bn_reduce", 0.0, (st.act == ACT_RELU ? 2.0 * out_el : raw_el + out_el) * es,
              launch_post_bwd_reduce(st.raw, g, st.out, st.bn_vec, P.batch, st.hc, st.wc, st.cout, st.act, st.pool,
                                     P.dtype, m->partial, s));
        TIMED(si, "bwd.bn_finalize", 0.0, 0.0,
              launch_bn_bwd_finalize(m->partial, nblocks_for(prow), rows, st.cout, grads + st.b_off, st.bn_vec,
                                     grads + st.bn_off, P.bn_mode == 0, s));
      }
    }
    TIMED(si, "bwd.bn_act_pool", 0.0, (2.0 * raw_el + out_el) * es,
          launch_post_bwd_apply(st.raw, g, st.has_bn ? st.bn_vec : nullptr, m->draw, P.batch, st.hc, st.wc, st.cout,
                                st.act, st.pool, st.has_bn, P.dtype, s));
    dr = m->draw;
  } else if (st.act != ACT_NONE && st.thin == 2) {
    TIMED(si, "bwd.act", 0.0, 3.0 * raw_el * es,
          launch_act_bwd(st.out, st.aux, g, m->draw, rows * st.cout, st.act, P.dtype, s));
    dr = m->draw;
  } else if (st.act != ACT_NONE && pre == 1) {
    // the kernel that produced the gradient masked it and left the bias gradient's column sums
    dr = m->draw;
    bias_done = true;
    TIMED(si, "bwd.bias_finalize", 0.0, 0.0,
          launch_colsum_finalize(m->partial, m->pre_blocks, st.cout, grads + st.b_off, s));
  } else if (st.act != ACT_NONE) {
    // activation backward and the bias gradient's column sums in one pass
    TIMED(si, "bwd.act_colsum", 0.0, 3.0 * raw_el * es,
          launch_act_bwd_colsum(st.out, st.aux, g, m->draw, rows, st.cout, st.act, P.dtype, m->partial, s));
    dr = m->draw;
    bias_done = true;
    TIMED(si, "bwd.bias_finalize", 0.0, 0.0,
          launch_colsum_finalize(m->partial, nblocks_for(rows), st.cout, grads + st.b_off, s));
  }
  // Fork: the weight gradient reads dr and the saved input.  When dr is one of the two
  // alternating buffers it may run beside the rest of the pass; a dr that is the incoming
  // gradient itself is overwritten by the very next layer, so that case stays in order.
  hipStream_t ws = s;
  if (dr == m->draw) {
    hipStream_t side = side_stream(m);
    if (side) {
      AE_HIP(hipEventRecord(m->ev_fork, s));
      AE_HIP(hipStreamWaitEvent(side, m->ev_fork, 0));
      ws = side;
    }
  }
  // Scratch of the weight-gradient kernels: a layer that stays in order because its conv-output
  // gradient is the incoming buffer has scratch of its own, so that it need not wait for the
  // side stream; any other launch on the caller's stream shares the side stream's scratch and
  // waits for what is still running there.
  float* const wws = (dr == m->draw || st.thin != 0) ? m->wgrad_ws : m->wgrad_ws_inorder;
  if (ws == s && wws == m->wgrad_ws) {
    AE_TRY(join_side(m, 0, s));
    AE_TRY(join_side(m, 1, s));
  }
  auto wgrad_enqueued = [&]() -> int {
    if (ws != s) {
      AE_HIP(hipEventRecord(m->ev_wdone[m->draw_sel], ws));
      m->wpending[m->draw_sel] = true;
    }
    return AE_OK;
  };
  if (st.thin == 2) {
    // dr is planar [n][C_out][H][W]
    TIMED(si, "bwd.bias_planesum", 0.0, raw_el * es,
          launch_plane_sums(dr, P.batch, st.cout, (int64_t)st.hc * st.wc, P.dtype, m->partial, s));
    TIMED(si, "bwd.bias_finalize", 0.0, 0.0,
          launch_colsum_finalize(m->partial, P.batch * plane_sums_split((int64_t)st.hc * st.wc), st.cout, grads + st.b_off, s));
    if (thin_wgrad_mfma_supported(st.cout, st.cin, st.win, P.dtype))
      TIMED_ON(ws, si, "bwd.wgrad_thin_mfma", conv_flops, (in_el + raw_el) * es + wel * 4,
               launch_thin_wgrad_mfma(dr, in, m->wgrad_ws, grads + st.w_off, P.batch, st.hin, st.win, st.cout, st.cin, 1,
                                      st.up, P.dtype, ws));
    else
      TIMED_ON(ws, si, "bwd.wgrad_thin", conv_flops, (in_el + raw_el) * es + wel * 4,
               launch_thin_wgrad(dr, in, m->wgrad_ws, grads + st.w_off, P.batch, st.hin, st.win, st.cout, st.cin, 1, st.up,
                                 P.dtype, ws));
    AE_TRY(wgrad_enqueued());
    bool with_relu = false;
    if (st.needs_dx && m->fuse_bwd && st.up == 1 && si > 0 &&
        thin_first_supported(st.cout, st.cin, st.k, 0, P.dtype, st.hc, st.wc)) {
      const Step& pv = P.steps[si - 1];
      if (pv.kind == ST_CONV && pv.thin == 0 && pv.act == ACT_RELU && !pv.has_bn && !pv.pool && !pv.out_planar) {
        // the input gradient goes straight into the conv-output gradient buffer of the layer below (the other one
        // than this layer's), already masked by that layer's ReLU, with the column sums of its bias gradient
        with_relu = true;
        m->draw_sel ^= 1;
        m->draw = m->draw_buf[m->draw_sel];
        AE_TRY(join_side(m, m->draw_sel, s));
        TIMED(si, "bwd.dgrad_thin_relu_mfma", conv_flops, (raw_el + 2.0 * in_el) * es,
              launch_thin_first(4, dr, params + st.w_off, st.wpack_d, nullptr, nullptr, pv.out, m->draw, m->partial, nullptr,
                                P.batch, st.hc, st.wc, st.cout, st.cin, s));
        m->pre_mode = 1;
        m->pre_blocks = thin_first_blocks(P.batch, st.hc, st.wc, st.cin, 4);
      }
    }
    if (st.needs_dx && !with_relu) {
      const double full_el = (double)rows * st.cin;
      if (thin_in_mfma_supported(st.cout, st.cin, st.k, 0, P.dtype)) {
        // the 2x2 sum that undoes the upsample happens in the kernel's epilogue
        TIMED(si, "bwd.dgrad_thin_mfma", conv_flops, (raw_el + in_el) * es,
              launch_thin_in_mfma(dr, params + st.w_off, st.wpack_d, nullptr, gnext, nullptr, P.batch, st.hc, st.wc,
                                  st.cout, st.cin, 1, ACT_NONE, st.up, P.dtype, s));
      } else {
        TIMED(si, "bwd.dgrad_thin", conv_flops, (raw_el + full_el) * es,
              launch_thin_in_conv(dr, params + st.w_off, nullptr, st.up ? m->dfull : gnext, nullptr, P.batch, st.hc,
                                  st.wc, st.cout, st.cin, 1, ACT_NONE, P.dtype, s));
        if (st.up)
          TIMED(si, "bwd.upsum", 0.0, (full_el + in_el) * es,
                launch_upsum(m->dfull, gnext, P.batch, st.hin, st.win, st.cin, P.dtype, s));
      }
    }
    return AE_OK;
  }
  // bias gradient: column sums of the conv-output gradient
  if (!bias_done) {
    TIMED(si, "bwd.bias_colsum", 0.0, raw_el * es, launch_col_stats(dr, rows, st.cout, P.dtype, m->partial, s));
    TIMED(si, "bwd.bias_finalize", 0.0, 0.0,
          launch_colsum_finalize(m->partial, nblocks_for(rows), st.cout, grads + st.b_off, s));
  }
  if (st.thin == 1) {
    if (thin_wgrad_mfma_supported(st.cin, st.cout, st.wc, P.dtype))
      TIMED_ON(ws, si, "bwd.wgrad_thin_mfma", conv_flops, (in_el + raw_el) * es + wel * 4,
               launch_thin_wgrad_mfma(in, dr, m->wgrad_ws, grads + st.w_off, P.batch, st.hc, st.wc, st.cin, st.cout, 0, 0, P.dtype, ws));
    else
      TIMED_ON(ws, si, "bwd.wgrad_thin", conv_flops, (in_el + raw_el) * es + wel * 4,
               launch_thin_wgrad(in, dr, m->wgrad_ws, grads + st.w_off, P.batch, st.hc, st.wc, st.cin, st.cout, 0, 0,
                                 P.dtype, ws));
    AE_TRY(wgrad_enqueued());
    return AE_OK;   // the first layer needs no input gradient
  }
  // weight gradient
  WgradArgs wa;
  wa.x = in; wa.dy = dr; wa.dw_canonical = grads + st.w_off;
  wa.n = P.batch; wa.hc = st.hc; wa.wc = st.wc; wa.cin = st.cin; wa.cout = st.cout; wa.k = st.k; wa.up = st.up;
  wa.dtype = P.dtype;
  if (wgrad_mfma_supported(wa)) {
    // (slot FLOPs are the algorithmic ones of the definition; the phase form of an upsampled layer, named apart, executes 4/9 of them)
    TIMED_ON(ws, si, wgrad_mfma_up_phases(wa) ? "bwd.wgrad_mfma_phases" : "bwd.wgrad_mfma", conv_flops,
             (in_el + raw_el) * es + wel * 4, launch_wgrad_mfma(wa, wws, ws));
  } else {
    TIMED_ON(ws, si, "bwd.wgrad_direct", conv_flops, (in_el + raw_el) * es + wel * 4,
             launch_wgrad_direct(wa, wws, wws == m->wgrad_ws ? P.max_wgrad_floats : P.max_wgrad_inorder_floats, ws));
  }
  AE_TRY(wgrad_enqueued());
  // input gradient: convolution of dr with the flipped, transposed weights at conv resolution
  if (st.needs_dx) {
    AE_TRY(join_pack(m, s, is_big_fc(st)));
    if (!m->packed_in_batch) {
      if (st.up_dgrad)
        TIMED(si, "bwd.pack_weights_up", 0.0, wel * 4.0 + 16.0 * st.cout * st.cin * es,
              launch_pack_weights_up(params + st.w_off, st.wpack_d, st.cout, st.cin, P.dtype, CONV_UP_DGRAD, s));
      else
        TIMED(si, "bwd.pack_weights", 0.0, wel * (4.0 + es),
              launch_pack_weights(params + st.w_off, st.wpack_d, st.cout, st.cin, st.k, P.dtype, true, s, st.wfrag_d));
    }
    ConvArgs a;
    a.x = dr; a.w = st.wpack_d; a.bias = nullptr;
    a.y = (st.up && !st.up_dgrad) ? m->dfull : gnext;
    if (st.up_dgrad) a.geom = CONV_UP_DGRAD;   // straight to the stored resolution: no full-size gradient, no 2x2 sum
    a.w_frag = st.wfrag_d;
    a.n = P.batch; a.hc = st.hc; a.wc = st.wc; a.cin = st.cout; a.cout = st.cin; a.k = st.k; a.up = 0;
    a.act = ACT_NONE; a.dtype = P.dtype; a.partial = nullptr; a.y_aux = nullptr;
    a.splitk_ws = m->splitk_ws;
    a.splitk_floats = P.max_splitk_floats;
    const double full_el = (double)rows * st.cin;
    // Work of the layer below that fits this kernel's epilogue (it reads that layer's saved activation beside the
    // gradient tile it is about to store): the ReLU backward + bias column sums of a conv + ReLU layer, or the two
    // sums of the batch-norm backward of a conv + bn + ReLU (+ pool) layer.
    if (m->fuse_bwd && si > 0 && a.y == gnext && conv_mfma_supported(a)) {
      const Step& pv = P.steps[si - 1];
      const int mode = (pv.kind != ST_CONV || pv.thin != 0 || pv.act != ACT_RELU || pv.out_planar || (pv.recompute && m->recompute)) ? 0
                       : (!pv.has_bn && !pv.pool) ? 1 : (pv.has_bn ? 2 : 0);
      const int nb = mode ? conv_comp_blocks(a) : 0;
      if (nb > 0) {
        a.comp = pv.out; a.comp_mode = mode; a.partial = m->partial;
        if (mode == 1) {
          // straight into the layer's conv-output gradient buffer (the other one than this layer's)
          m->draw_sel ^= 1;
          m->draw = m->draw_buf[m->draw_sel];
          AE_TRY(join_side(m, m->draw_sel, s));
          a.y = m->draw;
        } else {
          a.comp_bn = pv.bn_vec;
        }
        m->pre_mode = mode;
        m->pre_blocks = nb;
      }
    }
    if (conv_mfma_supported(a))
      // (the 4x4 stride-2 form, named apart, executes 4/9 of the algorithmic multiply-adds and writes the stored resolution)
      TIMED(si, st.up_dgrad ? "bwd.dgrad_mfma_stride2" : "bwd.dgrad_mfma", conv_flops,
            (raw_el + (st.up_dgrad ? in_el : full_el) + wel) * es, launch_conv_mfma(a, s));
    else
      TIMED(si, "bwd.dgrad_direct", conv_flops, (raw_el + full_el + wel) * es, launch_conv_direct(a, s));
    if (st.up && !st.up_dgrad)
      TIMED(si, "bwd.upsum", 0.0, (full_el + in_el) * es,
            launch_upsum(m->dfull, gnext, P.batch, st.hin, st.win, st.cin, P.dtype, s));
  }
  return AE_OK;
}

}  // namespace

extern "C" {

const char* model_last_error(void) { return ae::last_error(); }

int model_describe(const char* layer_spec, int batch, int dtype, int bn_mode, int64_t* n_params, int64_t in_chw[3],
                   int64_t out_chw[3], int64_t* latent_n, int64_t* workspace_bytes) {
  Plan P;
  AE_TRY(build_plan(layer_spec, batch, dtype, bn_mode, &P));
  if (n_params) *n_params = P.n_params;
  if (in_chw) { in_chw[0] = P.c0; in_chw[1] = P.h0; in_chw[2] = P.w0; }
  if (out_chw) { out_chw[0] = P.cl; out_chw[1] = P.hl; out_chw[2] = P.wl; }
  if (latent_n) *latent_n = P.latent_n;
  if (workspace_bytes) *workspace_bytes = P.ws_bytes;
  return AE_OK;
}

int model_create(const char* layer_spec, int batch, int dtype, int bn_mode, ae_model** out) {
  if (!out) return fail(AE_EINVAL, "model_create: out is null");
  *out = nullptr;
  ae_model* m = new (std::nothrow) ae_model();
  if (!m) return fail(AE_ENOMEM, "model_create: host allocation failed");
  int rc = build_plan(layer_spec, batch, dtype, bn_mode, &m->plan);
  if (rc != AE_OK) { delete m; return rc; }
  hipError_t e = hipMalloc((void**)&m->ws, (size_t)m->plan.ws_bytes);
  if (e != hipSuccess) {
    delete m;
    return fail(e == hipErrorOutOfMemory ? AE_ENOMEM : AE_EHIP, "model_create: hipMalloc(%lld bytes): %s",
                (long long)m->plan.ws_bytes, hipGetErrorString(e));
  }
  Plan& P = m->plan;
  for (Step& st : P.steps) {
    st.out = st.off_out >= 0 ? m->ws + st.off_out : nullptr;
    st.raw = st.off_raw >= 0 ? m->ws + st.off_raw : nullptr;
    st.wpack = st.off_wpack >= 0 ? m->ws + st.off_wpack : nullptr;
    st.wpack_d = st.off_wpack_d >= 0 ? m->ws + st.off_wpack_d : nullptr;
    st.bn_vec = st.off_bn >= 0 ? (float*)(m->ws + st.off_bn) : nullptr;
    st.aux = st.off_aux >= 0 ? (float*)(m->ws + st.off_aux) : nullptr;
    if (st.kind == ST_CONV) {
      ConvArgs a;
      memset(&a, 0, sizeof(a));
      a.n = P.batch; a.hc = st.hc; a.wc = st.wc; a.cin = st.cin; a.cout = st.cout; a.k = st.k; a.up = st.up;
      a.dtype = P.dtype;
      st.mfma = conv_mfma_supported(a);
      st.recompute = st.thin == 1 && !st.needs_dx && st.has_bn && st.act == ACT_RELU && st.pool &&
                     thin_first_supported(st.cin, st.cout, st.k, st.up, P.dtype, st.hc, st.wc);
      // the launches as forward_conv / backward_conv will describe them (of the pointers only null / non-null matters)
      ConvArgs f = a;
      f.act = (st.has_bn || st.pool) ? ACT_NONE : st.act;
      f.partial = (st.has_bn && P.bn_mode == 0) ? (float*)m->ws : nullptr;
      f.y_aux = (st.has_bn || st.pool) ? nullptr : st.aux;
      ConvArgs d = a;
      d.cin = st.cout; d.cout = st.cin; d.up = 0; d.act = ACT_NONE;
      if (st.mfma && st.thin == 0 && st.up && st.k == 3) {
        // the cheaper forms of an upsampled conv, decided once (the weight packing depends on it)
        st.up_phases = conv_up_phases_usable(f);
        st.up_dgrad = st.needs_dx && conv_up_dgrad_usable(d);
      }
      if (st.mfma && st.thin == 0) {
        // likewise the order of the packed weights
        if (st.up_phases) f.geom = CONV_UP_PHASES;
        if (st.up_dgrad) d.geom = CONV_UP_DGRAD;
        st.wfrag = conv_weights_frag_order(f);
        st.wfrag_d = st.needs_dx && conv_weights_frag_order(d);
      }
    }
  }
  m->grad_a = m->ws + P.off_grad_a;
  m->grad_b = m->ws + P.off_grad_b;
  m->draw_buf[0] = m->ws + P.off_draw;
  m->draw_buf[1] = m->ws + P.off_draw2;
  m->draw = m->draw_buf[0];
  m->dfull = m->ws + P.off_dfull;
  m->partial = (float*)(m->ws + P.off_partial);
  m->wgrad_ws = (float*)(m->ws + P.off_wgrad);
  m->wgrad_ws_inorder = (float*)(m->ws + P.off_wgrad_inorder);
  m->splitk_ws = (float*)(m->ws + P.off_splitk);
  m->fused_small = fused_small_match(P, &m->fused);
  *out = m;
  return AE_OK;
}

void model_destroy(ae_model* m) {
  if (!m) return;
  if (m->side) {
    (void)hipStreamSynchronize(m->side);
    (void)hipStreamDestroy(m->side);
  }
  if (m->ev_fork) (void)hipEventDestroy(m->ev_fork);
  if (m->ev_pack) (void)hipEventDestroy(m->ev_pack);
  if (m->ev_pack_fc) (void)hipEventDestroy(m->ev_pack_fc);
  for (hipEvent_t e : m->ev_wdone)
    if (e) (void)hipEventDestroy(e);
  if (m->ws) (void)hipFree(m->ws);
  for (TimeSlot& sl : m->slots)
    for (auto& pr : sl.pending) { (void)hipEventDestroy(pr.first); (void)hipEventDestroy(pr.second); }
  for (hipEvent_t e : m->free_events) (void)hipEventDestroy(e);
  delete m;
}

int model_timing_enable(ae_model* m, int on) {
  if (!m) return fail(AE_EINVAL, "model_timing_enable: null model");
  m->timing = on != 0;
  return AE_OK;
}

int model_set_overlap(ae_model* m, int on) {
  if (!m) return fail(AE_EINVAL, "model_set_overlap: null model");
  m->overlap = on != 0;
  return AE_OK;
}

int model_set_inference(ae_model* m, int on) {
  if (!m) return fail(AE_EINVAL, "model_set_inference: null model");
  m->inference = on != 0;
  m->have_forward = false;
  return AE_OK;
}

int model_set_recompute(ae_model* m, int on) {
  if (!m) return fail(AE_EINVAL, "model_set_recompute: null model");
  m->recompute = on != 0;
  m->have_forward = false;      // a backward pass needs a forward pass taken the same way
  return AE_OK;
}

int model_set_fused_backward(ae_model* m, int on) {
  if (!m) return fail(AE_EINVAL, "model_set_fused_backward: null model");
  m->fuse_bwd = on != 0;
  return AE_OK;
}

int model_set_params_static(ae_model* m, int on) {
  if (!m) return fail(AE_EINVAL, "model_set_params_static: null model");
  m->params_static = on != 0;
  m->fwd_packed = m->bwd_packed = nullptr;    // the next pass in each direction repacks
  return AE_OK;
}

int model_timing_slots(const ae_model* m, int* n_slots) {
  if (!m || !n_slots) return fail(AE_EINVAL, "model_timing_slots: null argument");
  *n_slots = (int)m->slots.size();
  return AE_OK;
}

int model_timing_read(ae_model* m, int slot, char* name, int name_len, double* total_ms, int64_t* launches,
                      double* flops_per_launch, double* bytes_per_launch) {
  if (!m || slot < 0 || slot >= (int)m->slots.size()) return fail(AE_EINVAL, "model_timing_read: bad slot");
  TimeSlot& sl = m->slots[slot];
  for (auto& pr : sl.pending) {
    AE_HIP(hipEventSynchronize(pr.second));
    float ms = 0.0f;
    AE_HIP(hipEventElapsedTime(&ms, pr.first, pr.second));
    sl.total_ms += (double)ms;
    sl.launches += 1;
    m->free_events.push_back(pr.first);
    m->free_events.push_back(pr.second);
  }
  sl.pending.clear();
  if (name && name_len > 0) snprintf(name, (size_t)name_len, "%s", sl.name.c_str());
  if (total_ms) *total_ms = sl.total_ms;
  if (launches) *launches = sl.launches;
  if (flops_per_launch) *flops_per_launch = sl.flops;
  if (bytes_per_launch) *bytes_per_launch = sl.bytes;
  return AE_OK;
}

int model_timing_reset(ae_model* m) {
  if (!m) return fail(AE_EINVAL, "model_timing_reset: null model");
  for (TimeSlot& sl : m->slots) {
    for (auto& pr : sl.pending) { m->free_events.push_back(pr.first); m->free_events.push_back(pr.second); }
    sl.pending.clear();
    sl.total_ms = 0.0;
    sl.launches = 0;
  }
  return AE_OK;
}

int model_param_count(const ae_model* m, int64_t* n_params) {
  if (!m || !n_params) return fail(AE_EINVAL, "model_param_count: null argument");
  *n_params = m->plan.n_params;
  return AE_OK;
}

int model_io_shape(const ae_model* m, int64_t in_chw[3], int64_t out_chw[3], int64_t* latent_n) {
  if (!m) return fail(AE_EINVAL, "model_io_shape: null model");
  const Plan& P = m->plan;
  if (in_chw) { in_chw[0] = P.c0; in_chw[1] = P.h0; in_chw[2] = P.w0; }
  if (out_chw) { out_chw[0] = P.cl; out_chw[1] = P.hl; out_chw[2] = P.wl; }
  if (latent_n) *latent_n = P.latent_n;
  return AE_OK;
}

int model_set_sample_offset(ae_model* m, uint64_t first_sample) {
  if (!m) return fail(AE_EINVAL, "model_set_sample_offset: null model");
  m->first_sample = first_sample;
  return AE_OK;
}

int model_forward(ae_model* m, const void* params, const void* x, float snr_db, uint64_t seed, void* y, void* stream) {
  if (!m || !x || !y) return fail(AE_EINVAL, "model_forward: null argument");
  Plan& P = m->plan;
  if (!params && P.n_params > 0) return fail(AE_EINVAL, "model_forward: params is null");
  if (!(snr_db == snr_db) || isinf(snr_db)) return fail(AE_EINVAL, "model_forward: snr_db is not finite");
  hipStream_t s = (hipStream_t)stream;
  const float* prm = (const float*)params;
  const float sigma = (float)pow(10.0, -(double)snr_db / 20.0);
  m->have_forward = false;
  const size_t ns = P.steps.size();
  if (m->inference && m->fused_small) {
    // small-image network, nothing to keep: three launches (see ae_fused_small.hip)
    const double io = ((double)P.batch * (P.c0 * P.h0 * P.w0 + P.cl * P.hl * P.wl) + (double)P.n_params) * 4.0;
    TIMED(0, "fwd.fused_small", 0.0, io,
          launch_fused_small(P, m->fused, prm, (const float*)x, (float*)y, (float*)P.steps[0].raw, (float*)P.steps[1].raw,
                             m->partial, sigma, seed, m->first_sample, s));
    return AE_OK;
  }
  m->last_x = x;
  m->last_params = params;
  AE_TRY(join_pack(m, s, true));
  if (m->params_static && m->fwd_packed == params) {
    m->packed_in_batch = true;     // the packed copies of an earlier call are still valid
  } else {
    AE_TRY(pack_all_beside(m, prm, false, s));
    // valid for later calls only if this call packed every layer up front (not layer by layer on the way)
    m->fwd_packed = (m->params_static && m->packed_in_batch) ? params : nullptr;
  }
  for (size_t i = 0; i < ns; ++i) {
    Step& st = P.steps[i];
    const void* in = step_input(m, i, x);
    switch (st.kind) {
      case ST_TRANSPOSE: {
        // the last step of a plan that ends in a transpose writes the caller's y directly
        void* dst = (i + 1 == ns) ? y : st.out;
        TIMED((int)i, "fwd.transpose", 0.0, 2.0 * P.batch * st.t_rows * st.t_cols * dtype_size(P.dtype),
              launch_transpose(in, dst, P.batch, st.t_rows, st.t_cols, P.dtype, s));
        break;
      }
      case ST_CONV:
        AE_TRY(forward_conv(m, (int)i, st, prm, in, s));
        break;
      case ST_CHANNEL:
        TIMED((int)i, "fwd.pnorm_awgn", 0.0, 2.0 * P.batch * st.cin * st.hin * st.win * dtype_size(P.dtype),
              launch_pnorm_awgn(in, st.out, P.batch, st.cin, st.hin * st.win, P.dtype, st.do_pnorm, st.do_awgn, sigma,
                                seed, m->first_sample, s));
        break;
    }
  }
  if (P.steps[ns - 1].kind != ST_TRANSPOSE) {
    const Step& st = P.steps[ns - 1];
    size_t bytes = (size_t)P.batch * st.cout * st.hout * st.wout * dtype_size(P.dtype);
    AE_HIP(hipMemcpyAsync(y, st.out, bytes, hipMemcpyDeviceToDevice, s));
  }
  AE_TRY(join_pack(m, s, true));
  m->have_forward = !m->inference;
  return AE_OK;
}

int model_backward(ae_model* m, const void* params, const void* x, const void* dy, void* grads, void* stream) {
  if (!m || !x || !dy) return fail(AE_EINVAL, "model_backward: null argument");
  Plan& P = m->plan;
  if ((!params || !grads) && P.n_params > 0) return fail(AE_EINVAL, "model_backward: params or grads is null");
  if (!m->have_forward) return fail(AE_ESTATE, "model_backward: no forward pass on this handle to differentiate");
  m->pre_mode = 0;
  hipStream_t s = (hipStream_t)stream;
  const float* prm = (const float*)params;
  float* gr = (float*)grads;
  const void* g = dy;
  const size_t ns = P.steps.size();
  // gradients flow only down to the first parametrised step
  size_t first_param = ns;
  for (size_t i = 0; i < ns; ++i)
    if (P.steps[i].kind == ST_CONV) { first_param = i; break; }
  // weight gradients a failed earlier call may have left on the side stream
  AE_TRY(join_side(m, 0, s));
  AE_TRY(join_side(m, 1, s));
  AE_TRY(join_pack(m, s, true));
  if (m->params_static && m->bwd_packed == params) {
    m->packed_in_batch = true;
  } else {
    AE_TRY(pack_all_beside(m, prm, true, s));
    m->bwd_packed = (m->params_static && m->packed_in_batch) ? params : nullptr;
  }
  for (size_t ii = ns; ii-- > first_param;) {
    Step& st = P.steps[ii];
    void* gnext = (g == m->grad_a) ? m->grad_b : m->grad_a;
    const void* in = step_input(m, ii, x);
    switch (st.kind) {
      case ST_TRANSPOSE:
        TIMED((int)ii, "bwd.transpose", 0.0, 2.0 * P.batch * st.t_rows * st.t_cols * dtype_size(P.dtype),
              launch_transpose(g, gnext, P.batch, st.t_cols, st.t_rows, P.dtype, s));
        g = gnext;
        break;
      case ST_CHANNEL:
        if (st.do_pnorm) {
          TIMED((int)ii, "bwd.pnorm", 0.0, 3.0 * P.batch * st.cin * st.hin * st.win * dtype_size(P.dtype),
                launch_pnorm_bwd(in, g, gnext, P.batch, (int64_t)st.cin * st.hin * st.win, P.dtype, s));
          g = gnext;
        }
        break;
      case ST_CONV:
        AE_TRY(backward_conv(m, (int)ii, st, prm, in, g, gnext, gr, s));
        if (st.needs_dx) g = gnext;
        break;
    }
  }
  // join: work enqueued on the caller's stream after this call sees every gradient
  AE_TRY(join_side(m, 0, s));
  AE_TRY(join_side(m, 1, s));
  AE_TRY(join_pack(m, s, true));
  return AE_OK;
}

int model_loss_mse(const void* y, const void* target, int64_t n_elem, int dtype, float* loss_dev, void* dy,
                   void* stream) {
  if (!y || !target || !loss_dev) return fail(AE_EINVAL, "model_loss_mse: null argument");
  if (n_elem <= 0) return fail(AE_EINVAL, "model_loss_mse: n_elem must be positive");
  if (dtype != AE_F32 && dtype != AE_BF16) return fail(AE_EINVAL, "model_loss_mse: bad dtype");
  return launch_mse(y, target, n_elem, dtype, loss_dev, dy, (hipStream_t)stream);
}

int model_noise(uint64_t seed, uint64_t first_sample, int64_t batch, int64_t n, float* out, void* stream) {
  if (!out) return fail(AE_EINVAL, "model_noise: out is null");
  if (batch < 0 || n < 0 || n > ((int64_t)1 << 33)) return fail(AE_EINVAL, "model_noise: bad size");
  if (batch == 0 || n == 0) return AE_OK;
  return launch_noise(seed, first_sample, batch, n, out, (hipStream_t)stream);
}

int model_pnorm_awgn(const void* z, void* y, int64_t batch, int64_t n, int dtype, float snr_db, uint64_t seed,
                     uint64_t first_sample, void* stream) {
  if (!z || !y) return fail(AE_EINVAL, "model_pnorm_awgn: null argument");
  if (batch < 0 || n <= 0 || n > 0x7FFFFFFF) return fail(AE_EINVAL, "model_pnorm_awgn: bad size");
  if (dtype != AE_F32 && dtype != AE_BF16) return fail(AE_EINVAL, "model_pnorm_awgn: bad dtype");
  if (batch == 0) return AE_OK;
  const float sigma = (float)pow(10.0, -(double)snr_db / 20.0);
  return launch_pnorm_awgn(z, y, batch, (int)n, 1, dtype, 1, 1, sigma, seed, first_sample, (hipStream_t)stream);
}

int model_gen_bits(uint64_t seed, uint64_t first_sample, int64_t batch, int k, float* x_pm1, void* stream) {
  if (!x_pm1) return fail(AE_EINVAL, "model_gen_bits: null argument");
  if (batch < 0 || k <= 0) return fail(AE_EINVAL, "model_gen_bits: bad size");
  if (batch == 0) return AE_OK;
  return launch_gen_bits(seed, first_sample, batch, k, x_pm1, (hipStream_t)stream);
}

int model_count_errors(const float* y, const float* x_pm1, int64_t batch, int k, uint64_t* bit_err, uint64_t* blk_err,
                       void* stream) {
  if (!y || !x_pm1 || !bit_err || !blk_err) return fail(AE_EINVAL, "model_count_errors: null argument");
  if (batch < 0 || k <= 0) return fail(AE_EINVAL, "model_count_errors: bad size");
  if (batch == 0) return AE_OK;
  return launch_count_errors(y, x_pm1, batch, k, bit_err, blk_err, (hipStream_t)stream);
}

// Monte-Carlo error-rate run: samples first_sample .. first_sample + total_samples - 1 in launches of m's batch,
// the remainder (if any) on m_tail, whose batch must be exactly that remainder.  Per launch: message bits ->
// forward -> error counts; everything is enqueued on `stream`, nothing is read back.
int model_monte_carlo(ae_model* m, ae_model* m_tail, const void* params, float snr_db, uint64_t seed,
                      uint64_t first_sample, uint64_t total_samples, float* x_buf, float* y_buf, uint64_t* bit_err,
                      uint64_t* blk_err, void* stream) {
  if (!m || !x_buf || !y_buf || !bit_err || !blk_err) return fail(AE_EINVAL, "model_monte_carlo: null argument");
  const Plan& P = m->plan;
  if (P.dtype != AE_F32 || P.h0 != 1 || P.w0 != 1 || P.hl != 1 || P.wl != 1 || P.cl != P.c0)
    return fail(AE_EINVAL, "model_monte_carlo: needs a binary32 model that maps k message symbols (in:kx1x1) to k soft bits");
  const uint64_t B = (uint64_t)P.batch;
  const uint64_t full = total_samples / B, rest = total_samples % B;
  if (rest != 0) {
    if (!m_tail) return fail(AE_EINVAL, "model_monte_carlo: %llu samples leave a last launch of %llu: pass a model of that batch as m_tail",
                             (unsigned long long)total_samples, (unsigned long long)rest);
    const Plan& T = m_tail->plan;
    if ((uint64_t)T.batch != rest || T.dtype != P.dtype || T.c0 != P.c0 || T.cl != P.cl || T.h0 != 1 || T.w0 != 1 ||
        T.hl != 1 || T.wl != 1 || T.n_params != P.n_params)
      return fail(AE_EINVAL, "model_monte_carlo: m_tail must be the same network with batch %llu", (unsigned long long)rest);
  }
  if (first_sample + total_samples < first_sample) return fail(AE_EINVAL, "model_monte_carlo: sample range wraps around 2^64");
  const int k = P.c0;
  for (uint64_t l = 0; l < full + (rest ? 1 : 0); ++l) {
    ae_model* mm = l < full ? m : m_tail;
    const int64_t nb = l < full ? (int64_t)B : (int64_t)rest;
    const uint64_t first = first_sample + l * B;
    AE_TRY(model_gen_bits(seed, first, nb, k, x_buf, stream));
    AE_TRY(model_set_sample_offset(mm, first));
    AE_TRY(model_forward(mm, params, x_buf, snr_db, seed, y_buf, stream));
    AE_TRY(model_count_errors(y_buf, x_buf, nb, k, bit_err, blk_err, stream));
  }
  return AE_OK;
}

int model_num_steps(const ae_model* m, int* n_steps) {
  if (!m || !n_steps) return fail(AE_EINVAL, "model_num_steps: null argument");
  *n_steps = (int)m->plan.steps.size();
  return AE_OK;
}

int model_step_info(const ae_model* m, int step, int* last_token, int64_t chw[3]) {
  if (!m || step < 0 || step >= (int)m->plan.steps.size()) return fail(AE_EINVAL, "model_step_info: bad step");
  const Step& st = m->plan.steps[step];
  if (last_token) *last_token = st.last_token;
  if (chw) { chw[0] = st.cout; chw[1] = st.hout; chw[2] = st.wout; }
  return AE_OK;
}

int model_get_activation(ae_model* m, int step, float* out_nchw, void* stream) {
  if (!m || !out_nchw || step < 0 || step >= (int)m->plan.steps.size())
    return fail(AE_EINVAL, "model_get_activation: bad argument");
  if (!m->have_forward) return fail(AE_ESTATE, "model_get_activation: no forward pass yet");
  const Plan& P = m->plan;
  const Step& st = P.steps[step];
  if (step + 1 == (int)P.steps.size() && st.kind == ST_TRANSPOSE)
    return fail(AE_EINVAL, "model_get_activation: the final layout step writes y directly and keeps no copy");
  if (st.out_planar)  // already [n][C][H][W]: convert only
    return launch_to_f32_nchw(st.out, out_nchw, P.batch, st.cout * st.hout * st.wout, 1, P.dtype, (hipStream_t)stream);
  return launch_to_f32_nchw(st.out, out_nchw, P.batch, st.cout, st.hout * st.wout, P.dtype, (hipStream_t)stream);
}

int model_get_conv_output(ae_model* m, int step, int64_t chw[3], float* out_nchw, void* stream) {
  if (!m || step < 0 || step >= (int)m->plan.steps.size()) return fail(AE_EINVAL, "model_get_conv_output: bad argument");
  const Plan& P = m->plan;
  const Step& st = P.steps[step];
  if (st.kind != ST_CONV || !(st.has_bn || st.pool) || !st.raw)
    return fail(AE_EINVAL, "model_get_conv_output: step %d keeps no convolution output apart from its saved output", step);
  if (chw) { chw[0] = st.cout; chw[1] = st.hc; chw[2] = st.wc; }
  if (!out_nchw) return AE_OK;
  if (!m->have_forward) return fail(AE_ESTATE, "model_get_conv_output: no forward pass yet");
  if (st.recompute && m->recompute) {
    // not kept by the forward pass: computed again, into the buffer the plan reserves for it
    const float* prm = (const float*)m->last_params;
    AE_TRY(launch_thin_in_mfma(m->last_x, prm + st.w_off, st.wpack, prm + st.b_off, st.raw, nullptr, P.batch, st.hc, st.wc,
                               st.cin, st.cout, 0, ACT_NONE, 0, P.dtype, (hipStream_t)stream));
  }
  return launch_to_f32_nchw(st.raw, out_nchw, P.batch, st.cout, st.hc * st.wc, P.dtype, (hipStream_t)stream);
}

}  // extern "C"
