"""Helpers of the GPU parity tests: run the same seeded case through the HIP library
(via its C boundary) and through the CPU oracle, and compare tensor by tensor."""
import json
import os

import numpy as np

import oracle.ae_oracle as orc
import workloads as wl

TOL = {"f32": 1e-4, "bf16": 2e-2}
# The stated tolerances are applied to the relative L2 norm of each tensor.  The largest single deviation, relative to
# the largest reference magnitude, gets the same bar in fp32.  In bf16 it is the tail of 1e5..1e8 independent
# rounding errors (4.5-5.5 standard deviations); measured over every case of the suite: at most 2.4e-2 against the
# oracle that emulates the storage format (all tensors, all sizes), 2.9e-2 for internal activations against the plain
# oracle, 5.5e-2 for the output y of the deepest network at full size against the plain oracle (the sigmoid output
# after twelve stored layers).  Hence: 3e-2 against the storage oracle and for gradients, 4e-2 for internal activations
# and 6e-2 for y against the plain oracle.
TOL_MAX = {"f32": 1e-4, "bf16": 3e-2}
TOL_MAX_ACT_PLAIN = {"f32": 1e-4, "bf16": 4e-2}
TOL_MAX_Y_PLAIN = {"f32": 1e-4, "bf16": 6e-2}
# Internal activations of a bf16 model against the PLAIN (real-number) oracle: the output y is
# held to 2e-2, but the error against real-number arithmetic grows with depth (every stored
# tensor adds a rounding of relative size 2^-9, and zero-mean weights cancel the mean of the
# all-positive ReLU outputs but not the errors: ~1.2x per layer).  At cfg5's full size it reaches
# 2.1e-2 after 12 stored layers while the same tensors agree with the bf16-storage oracle — the
# format's own semantics — to 9e-3.  So: 2e-2 against the storage oracle everywhere, 2e-2 against
# the plain oracle for y, 3e-2 against the plain oracle for internal activations.
TOL_ACT_PLAIN = {"f32": 1e-4, "bf16": 3e-2}

# Gradients of networks whose ReLU masks / max-pool winners differ between the two sides (deep bf16 networks: two
# correct implementations of the format differ by one bf16 ulp on a small fraction of stored values, and after a few
# layers 1e-3..1e-2 of the decisions differ; full-size fp32 networks: a few tens of 1e7 pre-activations lie within
# fp32 rounding of a decision).  The gradient is discontinuous in those decisions, so such cases are compared twice
# (run_case(flips=True)):
#  (1) against the oracle's own chain, with a bar that follows from COUNTING the disagreements
#      (decisions_of_both_sides: the device's saved tensors against the oracle's; nothing is fed from one side to
#      the other): every gradient tensor of a layer in step s is held to
#          relative L2 error  <=  base tolerance  +  FLIP_C * sqrt( sum over steps t >= s of flipped fraction f_t ):
#      a flipped decision in step t >= s replaces one term of the gradient signal that reaches layer s by another of
#      typical size (relative change sqrt(f_t) in L2, independent between steps); FLIP_C covers the spread of the
#      flipped terms' magnitudes around the typical one (measured (error - base) / sqrt(sum f): 1.0 .. 1.9 on the bf16
#      networks with 1e-3 .. 1e-2 of the decisions flipped, 3.2 on full-size cfg2 in fp32 where ~20 flipped decisions
#      among 1.7e7 carry the whole error).  No flips at or behind a layer => the plain 1e-4 / 2e-2 bar;
#  (2) against the oracle's backward pass run under the DEVICE's decisions (only the pass bits and winner indices
#      are stated to it, oracle/ae_oracle.cpp "given decisions"; every value it uses is its own), where every gradient
#      tensor must meet the plain 1e-4 / 2e-2 bar: this is the comparison that would catch a kernel that loses a few
#      per cent of a gradient (measured: <= 1.9e-2 on every bf16 case incl. cfg3 and cfg5 at full size, 4e-6 on cfg2).
FLIP_C = 4.0


def rel_errors(a, o):
    """(relative L2 error, max error relative to the largest reference magnitude)."""
    a = np.asarray(a, dtype=np.float64).ravel()
    o = np.asarray(o, dtype=np.float64).ravel()
    assert a.shape == o.shape, (a.shape, o.shape)
    assert np.all(np.isfinite(a))
    n2 = np.linalg.norm(o)
    mx = np.abs(o).max() if o.size else 0.0
    d = a - o
    l2 = np.linalg.norm(d) / n2 if n2 > 0 else np.linalg.norm(d)
    lm = np.abs(d).max() / mx if mx > 0 else (np.abs(d).max() if d.size else 0.0)
    return float(l2), float(lm)


STRICT = os.environ.get("AE_PARITY_NONSTRICT", "") == ""   # unset (debugging only) to collect errors instead of asserting
REPORT = os.environ.get("AE_PARITY_REPORT", "")              # a file that receives one JSON line per case (measurements)


def assert_close(a, o, tol, what, tol_max=None):
    l2, lm = rel_errors(a, o)
    tm = tol if tol_max is None else tol_max
    if STRICT:
        assert l2 <= tol and lm <= tm, "%s: rel L2 %.3e (tol %.1e), rel max %.3e (tol %.1e)" % (what, l2, tol, lm, tm)
    return l2, lm


def to_dev(a, dtype, torch):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16).contiguous() if dtype == "bf16" else t


def _winners(a):
    """Index (scan order (0,0),(0,1),(1,0),(1,1), first maximum) of the largest value in every 2x2 window of a [B][C][H][W] array."""
    b, c, h, w = a.shape
    return a.reshape(b, c, h // 2, 2, w // 2, 2).transpose(0, 1, 2, 4, 3, 5).reshape(b, c, h // 2, w // 2, 4).argmax(axis=-1)


def decisions_of_both_sides(m, net, params, batch):
    """Per step of the device's plan that takes discrete decisions in its backward pass (ReLU pass bits, max-pool
    winners): the fraction of them on which the device's saved tensors and the oracle's disagree, and the device's
    decisions as arrays keyed by the oracle's op index (uint8, shape of that op's output: relu pass bits, pool2
    winner indices).  Test-side bookkeeping computed from the two sides' saved tensors."""
    import torch
    flips, dec, prev = {}, {}, -1
    for s in range(m.model_num_steps()):
        tok, chw = m.model_step_info(s)
        first, prev = prev + 1, tok
        kinds = [net.ops[i + 1]["kind"] for i in range(first, tok + 1)]
        if "relu" not in kinds and "pool2" not in kinds:
            continue
        buf = torch.empty((batch,) + chw, dtype=torch.float32, device="cuda")
        m.model_get_activation(s, buf)
        out_d = buf.cpu().numpy()
        del buf
        out_o = net.activation(tok).reshape(out_d.shape)
        if "pool2" in kinds:
            ipool = first + kinds.index("pool2")
            cshape = m.model_get_conv_output(s)
            raw = torch.empty((batch,) + cshape, dtype=torch.float32, device="cuda")
            m.model_get_conv_output(s, raw)
            raw_d = raw.cpu().numpy()
            del raw
            if "bn" in kinds:       # batch-norm keeps the order of a channel's values if gamma > 0 and reverses it if gamma < 0
                off = net.ops[first + kinds.index("bn") + 1]["param_off"]
                raw_d *= np.sign(params[off:off + cshape[0]]).astype(np.float32)[None, :, None, None]
            w_d = _winners(raw_d)
            del raw_d
            w_o = _winners(net.activation(ipool - 1).reshape((batch,) + cshape))
            dec[ipool] = w_d.astype(np.uint8)
            if "relu" in kinds:
                a_d, a_o = out_d > 0, out_o > 0
                flip = (a_d != a_o) | (a_d & a_o & (w_d != w_o))
                # pass bits at convolution resolution: only a window's winner can receive a gradient at all
                b, c, ho, wo = w_d.shape
                onehot = (np.arange(4, dtype=np.uint8)[None, None, None, None, :] == w_d[..., None].astype(np.uint8)) & a_d[..., None]
                dec[first + kinds.index("relu")] = np.ascontiguousarray(
                    onehot.reshape(b, c, ho, wo, 2, 2).transpose(0, 1, 2, 4, 3, 5).reshape(b, c, 2 * ho, 2 * wo).astype(np.uint8))
            else:
                flip = w_d != w_o
        else:
            flip = (out_d > 0) != (out_o > 0)
            dec[first + kinds.index("relu")] = (out_d > 0).astype(np.uint8)
        flips[s] = float(flip.mean())
    return flips, dec


def run_case(spec, batch, dtype="f32", seed=0, snr_db=10.0, first_sample=0, bn_mode=0, backward=True,
             perturb=True, check_acts=True, x=None, params=None, cot=None, grad_tol=None, grad_cos=None,
             flips=False, tag=None):
    """Run spec on both sides; assert parity of y, every saved activation and (optionally)
    every gradient.  Returns a dict of the worst errors.

    fp32 models: everything against the plain oracle at 1e-4.
    bf16 models: y and activations against the plain (real-number) oracle at 2e-2, and again
    against the oracle emulating the bfloat16 storage format; gradients against the emulating
    oracle, so that ReLU masks and max-pool winners are decided in the format's precision on
    both sides.  grad_tol / grad_cos override the gradient bar.  flips=True: the decisions on which
    the two sides differ are counted and the gradient bar of each layer follows from the count (FLIP_C).
    cot="mse": the upstream gradient is that of the mean squared error against the input, from the oracle's
    output (what a training step feeds the backward pass)."""
    import torch
    from paper_2602_17681_amd import binding as ae

    bf = dtype == "bf16"
    tol, tolm = TOL[dtype], TOL_MAX[dtype]
    gtol = tol if grad_tol is None else grad_tol
    if params is None:
        params = wl.make_params(spec, seed, bn_mode=bn_mode, perturb=perturb, bf16=bf)
    if x is None:
        x = wl.make_input(spec, batch, seed, bf16=bf)
    refs = [("plain", orc.Net(spec, batch, bn_mode))]
    if bf:
        refs.append(("bf16-storage", orc.Net(spec, batch, bn_mode, store_bf16=True)))
    y_refs = [net.forward(params, x, snr_db=snr_db, seed=seed, first_sample=first_sample) for _, net in refs]
    net = refs[-1][1]            # the one gradients are compared with

    m = ae.Model(spec, batch, ae.DTYPES[dtype], bn_mode)
    assert m.n_params == net.n_params and m.in_shape == net.in_shape and m.out_shape == net.out_shape
    p_d = torch.from_numpy(params).cuda()
    x_d = to_dev(x, dtype, torch)
    y_d = torch.empty((batch,) + m.out_shape, dtype=m.tdtype, device="cuda")
    m.model_set_sample_offset(first_sample)
    m.model_forward(p_d, x_d, snr_db, seed, y_d)
    torch.cuda.synchronize()
    worst = {}
    y_gpu = y_d.float().cpu().numpy()
    for (rname, _), y_ref in zip(refs, y_refs):
        worst["y/" + rname] = assert_close(y_gpu, y_ref, tol, "y vs %s oracle" % rname,
                                           tol_max=TOL_MAX_Y_PLAIN[dtype] if rname == "plain" else tolm)
    if check_acts:
        ns = m.model_num_steps()
        for s in range(ns):
            tok, chw = m.model_step_info(s)
            if s == ns - 1 and chw == m.out_shape and tok == net.n_ops - 1:
                continue  # the boundary layout step: its output is y itself
            buf = torch.empty((batch,) + chw, dtype=torch.float32, device="cuda")
            m.model_get_activation(s, buf)
            torch.cuda.synchronize()
            got = buf.cpu().numpy()
            for rname, rnet in refs:
                ref = rnet.activation(tok).reshape((batch,) + chw)
                atol = TOL_ACT_PLAIN[dtype] if rname == "plain" else tol
                worst["act%d/%s" % (s, rname)] = assert_close(
                    got, ref, atol, "activation of step %d (token %d) vs %s oracle" % (s, tok, rname),
                    tol_max=TOL_MAX_ACT_PLAIN[dtype] if rname == "plain" else tolm)
    step_of_op, cum, dec = {}, {}, {}
    if backward and flips:
        fl, dec = decisions_of_both_sides(m, net, params, batch)
        worst["flips"] = fl
        prev, tot = -1, 0.0
        ns = m.model_num_steps()
        toks = [m.model_step_info(s)[0] for s in range(ns)]
        for s in range(ns - 1, -1, -1):
            tot += fl.get(s, 0.0)
            cum[s] = tot
        for s in range(ns):
            for op in range(prev + 1, toks[s] + 1):
                step_of_op[op] = s
            prev = toks[s]
    if backward:
        if isinstance(cot, str) and cot == "mse":
            _, dmse = orc.loss_mse(y_refs[-1], x.astype(np.float64))
            cot = wl.round_to_bf16(dmse.astype(np.float32)) if bf else dmse.astype(np.float32)
        if cot is None:
            cot = wl.make_cotangent((batch,) + m.out_shape, seed, bf16=bf)
        g_ref, _ = net.backward(params, cot.astype(np.float64))
        dy_d = to_dev(cot, dtype, torch)
        g_d = torch.full((m.n_params,), float("nan"), dtype=torch.float32, device="cuda")
        m.model_backward(p_d, x_d, dy_d, g_d)
        torch.cuda.synchronize()
        g = g_d.cpu().numpy()
        assert np.all(np.isfinite(g))
        ent, _, _, _ = wl.param_layout(spec, bn_mode)

        def compare(g_ref, prefix, bound_of, max_of):
            for e in ent:
                sz = int(np.prod(e["shape"]))
                sl = slice(e["offset"], e["offset"] + sz)
                name = "%s %s.%s@%d" % (prefix, e["name"], e["kind"], e["op"])
                if np.abs(g_ref[sl]).max() == 0.0:
                    assert np.abs(g[sl]).max() == 0.0, name
                    continue
                if e["kind"] == "b" and _feeds_batch_bn(spec, e["op"], bn_mode):
                    # analytically zero: compare against the scale of the layer's weight gradient instead
                    wsl = [q for q in ent if q["op"] == e["op"] and q["kind"] == "w"][0]
                    scale = np.abs(g_ref[wsl["offset"]:wsl["offset"] + int(np.prod(wsl["shape"]))]).max()
                    if STRICT:
                        assert np.abs(g[sl]).max() <= max(gtol, 1e-3) * scale * 10, name
                    continue
                bound = bound_of(e)
                worst[name] = assert_close(g[sl], g_ref[sl], bound, name, tol_max=max_of(bound)) + (bound,)
                if grad_cos is not None and sz >= 16:
                    c = float(np.dot(g[sl], g_ref[sl]) / (np.linalg.norm(g[sl]) * np.linalg.norm(g_ref[sl])))
                    worst[name] = worst[name] + (c,)
                    if STRICT:
                        assert c >= grad_cos, "%s: cosine %.4f < %.4f" % (name, c, grad_cos)

        if flips:
            # (1) the oracle's own chain, untouched: bar from the counted disagreements (one flipped term can move a
            #     single entry by its full size, so the largest deviation gets ten times the L2 bound)
            compare(g_ref, "grad", lambda e: gtol + FLIP_C * float(np.sqrt(cum[step_of_op[e["op"]]])), lambda b: max(tolm, 10 * b))
            # (2) the arithmetic of the backward pass under the same decisions: the oracle is TOLD the device's pass
            #     bits and winners (decisions only; every value it uses is its own) and must then agree at the plain bar
            for i, d in dec.items():
                net.set_decisions(i, d)
            g_same, _ = net.backward(params, cot.astype(np.float64))
            for i in dec:
                net.set_decisions(i, None)
            compare(g_same, "grad/same-decisions", lambda e: gtol, lambda b: max(gtol, tolm))
        else:
            compare(g_ref, "grad", lambda e: gtol, lambda b: max(gtol, tolm))
    m.close()
    if REPORT:
        with open(REPORT, "a") as f:
            f.write(json.dumps(dict(case=tag or spec, batch=batch, dtype=dtype, worst={k: v for k, v in worst.items()})) + "\n")
    return worst


def _feeds_batch_bn(spec, op, bn_mode):
    toks = [t.strip() for t in spec.split(",")][1:]
    return bn_mode == 0 and op + 1 < len(toks) and toks[op + 1] == "bn"
