#!/usr/bin/env python3
"""Benchmark of the autoencoder-over-AWGN hot path on one MI355X.

A step is one pass of the whole hot path over one synthetic batch of the chosen
workload: forward (+ MSE loss + backward where the workload trains; + message bits and
error counting for the Monte-Carlo workload).  Inputs, parameters and outputs are
resident in HBM before the timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config cfg5] [--no-cpu-baseline] [--no-per-config]
"""
import argparse
import json
import sys
import time

import numpy as np

import workloads as wl

PEAK = {"bf16": 2500.0, "f32": 157.3}     # dense MFMA TFLOP/s, MI355X
HBM_PEAK_GBS = 8000.0
# HBM bytes per launch (fetched + written) of a kernel family, from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# summarised in the named file under profiles/ (each counter scaled by what it reads for a plain 256 MiB copy: fetch
# x2.000, write x1.000).  A figure belongs to the kernels as they were when its profile was taken: an entry is removed
# (traffic = null in the JSON line) when the kernels of its family change, until the counters are collected again.
TRAFFIC = {
    # workload -> kernel family -> measured HBM bytes per launch
    "cfg5": {"k_igemm": {"bytes_per_launch": 93.3e6,
                         "source": "profiles/cfg5_hbm_traffic.md (kernels as of commit e674093; 20 launches per step, "
                                   "59.4 MB fetched + 33.8 MB written each)"}},
}


def build_case(name, torch, ae, batch=None):
    cfg = wl.CONFIGS[name]
    bf = cfg["dtype"] == "bf16"
    B = batch or cfg["batch"]
    m = ae.Model(cfg["spec"], B, ae.DTYPES[cfg["dtype"]])
    if not cfg["backward"]:
        # forward-only Monte-Carlo workloads: nothing is kept for a backward pass, and the parameters stay the same
        # from launch to launch (no repacking after the first)
        m.model_set_inference(True)
        m.model_set_params_static(True)
    params = torch.from_numpy(wl.make_params(cfg["spec"], cfg["seed"], bf16=bf)).cuda()
    if name == "cfg4":
        x = torch.empty((B,) + m.in_shape, dtype=torch.float32, device="cuda")
    else:
        x = torch.from_numpy(wl.make_input(cfg["spec"], B, cfg["seed"], bf16=bf)).cuda().to(m.tdtype).contiguous()
    st = dict(cfg=cfg, name=name, m=m, params=params, x=x, B=B,
              y=torch.empty((B,) + m.out_shape, dtype=m.tdtype, device="cuda"))
    if cfg["backward"]:
        st["dy"] = torch.empty_like(st["y"])
        st["grads"] = torch.empty(m.n_params, dtype=torch.float32, device="cuda")
        st["loss"] = torch.zeros(1, dtype=torch.float32, device="cuda")
    if name == "cfg4":
        st["bit_err"] = torch.zeros(1, dtype=torch.int64, device="cuda")
        st["blk_err"] = torch.zeros(1, dtype=torch.int64, device="cuda")
    st["i"] = 0
    return st


def one_step(st, ae):
    cfg, m = st["cfg"], st["m"]
    snr = st.get("snr", cfg["snr_db"][0])          # one SNR point per timed block (run_timed is called per point)
    if st["name"] == "cfg4":
        first = st["i"] * st["B"]
        ae.model_gen_bits(cfg["seed"], first, st["B"], m.in_shape[0], st["x"])
        m.model_set_sample_offset(first)
        m.model_forward(st["params"], st["x"], snr, cfg["seed"], st["y"])
        ae.model_count_errors(st["y"], st["x"], st["B"], m.in_shape[0], st["bit_err"], st["blk_err"])
    else:
        m.model_set_sample_offset(st["i"] * st["B"])
        m.model_forward(st["params"], st["x"], snr, cfg["seed"], st["y"])
        if cfg["backward"]:
            ae.model_loss_mse(st["y"], st["x"], st["loss"], st["dy"])
            m.model_backward(st["params"], st["x"], st["dy"], st["grads"])
    st["i"] += 1


def run_timed(st, ae, torch, steps, warmup, timing=False):
    for _ in range(warmup):
        one_step(st, ae)
    torch.cuda.synchronize()
    st["m"].model_timing_reset()
    st["m"].model_timing_enable(timing)
    t0 = time.perf_counter()
    for _ in range(steps):
        one_step(st, ae)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    st["m"].model_timing_enable(False)
    return dt


def kernel_table(st, steps):
    rows = []
    for s in st["m"].model_timing_read():
        if s["launches"] == 0:
            continue
        avg_ms = s["total_ms"] / s["launches"]
        share = EXECUTED_SHARE.get(s["name"].split(".")[-1], 1.0)
        rows.append(dict(name=s["name"], avg_ms=avg_ms, ms_per_step=s["total_ms"] / steps,
                         tflops=(s["flops"] * share / avg_ms / 1e9) if s["flops"] > 0 and avg_ms > 0 else None,
                         gbs=(s["bytes"] / avg_ms / 1e6) if s["bytes"] > 0 and avg_ms > 0 else None,
                         flops=s["flops"], bytes=s["bytes"]))
    return rows


FAMILY = {"conv_mfma": "k_igemm", "dgrad_mfma": "k_igemm", "conv_mfma_phases": "k_igemm", "dgrad_mfma_stride2": "k_igemm",
          "wgrad_mfma": "k_wgrad", "wgrad_mfma_phases": "k_wgrad",
          "conv_thin_in_mfma": "k_thin_in_mfma", "dgrad_thin_mfma": "k_thin_in_mfma"}


# A 3x3 convolution behind a x2 upsample runs as four 2x2 phase convolutions (forward), one 4x4 stride-2
# convolution (input gradient) or sixteen phase-tap correlations (weight gradient): 4/9 of the multiply-adds of the
# definition.  The library's slots carry the algorithmic FLOPs of the definition (2*M*N*K); the share below turns
# them into the multiply-adds the kernels really perform (per-kernel `tflops` in the line are executed rates).
EXECUTED_SHARE = {"conv_mfma_phases": 4.0 / 9.0, "dgrad_mfma_stride2": 4.0 / 9.0, "wgrad_mfma_phases": 4.0 / 9.0}


_MEASURED = {}


def measured_peaks(ae):
    """What plain loops reach on THIS device in this run, beside the nominal peaks: independent 32x32x16 bf16
    matrix-core instructions on every compute unit (operands all 1.0; random operands with the LDS fragment reads of a
    128x64 wave tile, the ceiling of a real K loop under this chip's power management), and a 256 MiB device copy."""
    if _MEASURED:
        return _MEASURED
    import torch
    _MEASURED["mfma_bf16_ones_tflops"] = round(max(ae.model_calibrate_mfma(0, 0, iters=20000)[0] for _ in range(2)), 1)
    _MEASURED["mfma_bf16_random_with_lds_reads_tflops"] = round(max(ae.model_calibrate_mfma(6, 1, iters=20000)[0] for _ in range(2)), 1)
    src = torch.ones(256 << 20, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(2):
        dst.copy_(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    _MEASURED["hbm_copy_read_plus_write_gbs"] = round(2.0 * (256 << 20) * 5 / e0.elapsed_time(e1) / 1e6, 1)
    return _MEASURED


def roofline_of(rows, dtype, workload=None, ae=None):
    """The kernel family that takes the largest share of the step (all its launches together), priced against the
    roof that bounds it: work of its launches divided by their total HIP-event time.  For a matrix-core family
    `achieved` / `frac` count the multiply-adds the kernels EXECUTE (what the hardware roof bounds);
    `achieved_algorithmic` counts the FLOPs of the layers' definition (2*M*N*K), which is larger where a layer runs in
    a cheaper algebraic form; their ratio is the saving of those forms, not utilisation."""
    if not rows:
        return None
    fam = {}
    for r in rows:
        key = FAMILY.get(r["name"].split(".")[-1], r["name"].split(".")[-1])
        f = fam.setdefault(key, dict(ms=0.0, flops=0.0, flops_exec=0.0, bytes=0.0, launches=0))
        f["ms"] += r["ms_per_step"]
        f["flops"] += r["flops"]
        f["flops_exec"] += r["flops"] * EXECUTED_SHARE.get(r["name"].split(".")[-1], 1.0)
        f["bytes"] += r["bytes"]
        f["launches"] += 1
    name, top = max(fam.items(), key=lambda kv: kv[1]["ms"])
    avg_ms = top["ms"] / top["launches"]
    balance = PEAK[dtype] * 1e12 / (HBM_PEAK_GBS * 1e9)
    tr = TRAFFIC.get(workload, {}).get(name)
    common = dict(traffic=None if tr is None else tr["bytes_per_launch"], traffic_source=None if tr is None else tr["source"],
                  avg_ms=avg_ms, launches_per_step=top["launches"], bytes_per_launch=top["bytes"] / top["launches"],
                  peak_measured=measured_peaks(ae) if ae is not None else None)
    if top["flops"] > 0 and top["flops"] / max(top["bytes"], 1.0) >= balance:
        ach = top["flops"] / top["ms"] / 1e9
        ach_exec = top["flops_exec"] / top["ms"] / 1e9
        return dict(bound="mfma", kernel=name, achieved=ach_exec, peak=PEAK[dtype], unit="TFLOP/s", frac=ach_exec / PEAK[dtype],
                    achieved_algorithmic=ach, frac_algorithmic=ach / PEAK[dtype],
                    flops_per_launch=top["flops_exec"] / top["launches"],
                    flops_per_launch_algorithmic=top["flops"] / top["launches"], **common)
    ach = top["bytes"] / top["ms"] / 1e6
    return dict(bound="hbm", kernel=name, achieved=ach, peak=HBM_PEAK_GBS, unit="GB/s", frac=ach / HBM_PEAK_GBS, **common)


# measured HBM bytes per launch of k_mx_quantize on this workload (profiles/mx_quantize.md): FETCH_SIZE x2.000 + WRITE_SIZE
MX_TRAFFIC_BYTES = {"bf16": 1.0738e9}


def bench_mx_quant(torch, ae, args):
    """One step = Q(x) of a [65 536][4 096] activation tensor resident in HBM (the shape of 32 sequences of 2 048
    tokens of a 4 096-wide model; blocks of 32).  Algorithmic bytes: the tensor read once and written once."""
    rows, d, block = 65536, 4096, 32
    dtype = torch.bfloat16 if args.dtype == "bf16" else torch.float32
    gen = torch.Generator(device="cuda").manual_seed(7)
    x = torch.randn(rows, d, device="cuda", generator=gen) * torch.exp(torch.randn(1, d, device="cuda", generator=gen))
    x[:, ::509] *= 100.0                                  # a few outlier channels
    x = x.to(dtype).contiguous()
    q = torch.empty_like(x)
    for _ in range(args.warmup):
        ae.model_mx_quantize_elem(x, q, rows, d, block, args.mx_elem)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ae.model_mx_quantize_elem(x, q, rows, d, block, args.mx_elem)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # the kernel's own duration: HIP events on the stream it runs on
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        ae.model_mx_quantize_elem(x, q, rows, d, block, args.mx_elem)
    e1.record()
    torch.cuda.synchronize()
    avg_ms = e0.elapsed_time(e1) / args.steps
    nbytes = 2.0 * rows * d * x.element_size()
    ach = nbytes / avg_ms / 1e6
    # oracle on a bounded sample of the same tensor
    import oracle.mx_oracle as mxo
    sample = 256 if args.no_cpu_baseline else 32768
    xs = x[:sample].float().cpu().numpy().astype("float64")
    c0 = time.perf_counter()
    mxo.mx_quantize(xs, block, args.mx_elem)
    ct = time.perf_counter() - c0
    return {
        "metric": "tokens/sec, MX block quantisation Q(x)", "value": rows * args.steps / dt, "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": "mx_quant: Q(x), %s elements, block 32" % {"fp4": "FP4 E2M1", "fp8": "FP8 E4M3", "int4": "4-bit integer"}[args.mx_elem],
                   "tokens": rows, "d": d, "block": block},
        "roofline": {"bound": "hbm", "kernel": "k_mx_quantize", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": ach / HBM_PEAK_GBS, "traffic": MX_TRAFFIC_BYTES.get(args.dtype), "avg_ms": avg_ms,
                     "launches_per_step": 1,
                     "bytes_per_launch": nbytes},
        "cpu_baseline": {"value": sample / ct, "unit": "tokens/s", "cores": 1, "kind": "oracle",
                         "sample": "%d tokens of the same tensor, %.1f s" % (sample, ct)},
    }


# measured HBM bytes per launch of the triangular products (profiles/lu_param.md)
LU_TRAFFIC_BYTES = {"bf16": 2.07e8}

# measured HBM bytes per launch of the two GEMMs of the transformation error (profiles/transform_mse.md)
TMSE_TRAFFIC_BYTES = {"bf16": 9.62e8}   # average of the two GEMM launches (0.941 GB and 0.984 GB)


def bench_transform_mse(torch, ae, args):
    """One step = E(T) of Eq. (2) for a [16 384][4 096] activation tensor resident in HBM and a dense affine map T:
    y = Q(x A^T + v) and the residual x - T^-1(y), two 16 384 x 4 096 x 4 096 GEMMs on the matrix cores with the
    quantiser and the error sums in their epilogues.  Algorithmic FLOPs: 2 * 2 * tokens * d^2."""
    rows, d, block = 16384, 4096, 32
    bf = args.dtype == "bf16"
    td = torch.bfloat16 if bf else torch.float32
    x_h = wl.make_activations(rows, d, seed=9, bf16=bf)
    a, v, ainv = wl.make_transform(d, seed=9, bf16=bf, kind="affine")
    dev = lambda arr, t: torch.from_numpy(np.ascontiguousarray(arr, dtype=np.float32)).cuda().to(t).contiguous()
    x, at, ait = dev(x_h, td), dev(a, td), dev(ainv, td)
    vt, st = dev(v, torch.float32), torch.empty(d, device="cuda")
    ae.model_inverse_shift(ait, vt, d, st)
    yq = torch.empty_like(x)
    ws = torch.empty(ae.model_transform_mse_workspace(rows, d, ae.DTYPES[args.dtype]) // 4, dtype=torch.float32, device="cuda")
    eb = torch.empty(d // block, device="cuda")
    et = torch.empty(1, device="cuda")
    step = lambda: ae.model_transform_mse(x, at, vt, ait, st, rows, d, block, yq, ws, eb, et)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    step_ms = e0.elapsed_time(e1) / args.steps
    flops = 2.0 * 2.0 * rows * d * d
    ach = flops / step_ms / 1e9
    es = x.element_size()
    import oracle.mx_oracle as mxo
    sample = 64 if args.no_cpu_baseline else 8192
    c0 = time.perf_counter()
    e_o, _, _ = mxo.transform_mse(x_h[:sample], a, v, ainv, block, storage=args.dtype)
    ct = time.perf_counter() - c0
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = 1
    return {
        "metric": "tokens/sec, transformation error E(T) of an affine map under MX quantisation", "value": rows * args.steps / dt,
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": "transform_mse: E(T), dense affine T, FP4 E2M1 elements, block 32", "tokens": rows, "d": d,
                   "block": block, "E": float(et.item())},
        # both GEMM launches together (the two finalising kernels, a few microseconds, are inside the events)
        "roofline": {"bound": "mfma", "kernel": "k_igemm (quantising / residual epilogues)", "achieved": ach, "peak": PEAK[args.dtype],
                     "unit": "TFLOP/s", "frac": ach / PEAK[args.dtype], "traffic": TMSE_TRAFFIC_BYTES.get(args.dtype),
                     "avg_ms": step_ms / 2, "launches_per_step": 2, "flops_per_launch": flops / 2,
                     "bytes_per_launch": (2.0 * rows * d + d * d) * es},
        "cpu_baseline": {"value": sample / ct, "unit": "tokens/s", "cores": cores, "kind": "oracle",
                         "sample": "%d tokens of the same tensor, %.1f s, E=%.4g" % (sample, ct, e_o)},
    }


def bench_lu_param(torch, ae, args):
    """One step = everything the LU parametrisation A = P L (U + diag s) of Eq. (4) costs per optimiser step for one
    d x d matrix, d = 4 096: compose A from the free parameters, the volume regulariser and its gradient, and the
    parameter gradients from dLoss/dA.  Algorithmic FLOPs: three products with a triangular factor of which (backward)
    a triangle is wanted, 2 d^3 / 3 each."""
    d = args.width
    bf = args.dtype == "bf16"
    td = torch.bfloat16 if bf else torch.float32
    params = wl.make_lu_params(d, seed=11, kind="bd_hadamard", noise=1e-3)
    lp, up, ls, sg = [torch.from_numpy(a).cuda() for a in params[:4]]
    perm = torch.from_numpy(params[4]).cuda()
    g_h = np.random.default_rng(12).standard_normal((d, d)).astype(np.float32)
    g = torch.from_numpy(g_h).cuda().to(td).contiguous()
    a = torch.empty((d, d), dtype=td, device="cuda")
    dlp, dup = torch.empty((d, d), device="cuda"), torch.empty((d, d), device="cuda")
    dls, vgrad, val = torch.empty(d, device="cuda"), torch.empty(d, device="cuda"), torch.empty(1, device="cuda")
    ws = torch.empty(ae.model_lu_workspace(d, ae.DTYPES[args.dtype]), dtype=torch.uint8, device="cuda")

    def step():
        ae.model_lu_compose(lp, up, ls, sg, perm, d, a, ws)
        ae.model_vol_penalty(ls, d, val, vgrad)
        ae.model_lu_backward(g, lp, up, ls, sg, perm, d, dlp, dup, dls, ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    step_ms = e0.elapsed_time(e1) / args.steps
    # the three matrix-core products alone: HIP events around each launch inside the library
    ae.model_lu_timing(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    gemm_ms, launches = ae.model_lu_timing(False)
    avg_ms = gemm_ms / max(launches, 1)
    # beside the step: the inverse of the same matrix (what the transformation error and the folding take with A)
    inv_ms = None
    if d % 128 == 0:
        ainv = torch.empty((d, d), dtype=td, device="cuda")
        wsi = torch.empty(ae.model_lu_inverse_workspace(d), dtype=torch.uint8, device="cuda")
        for _ in range(3):
            ae.model_lu_inverse(lp, up, ls, sg, perm, d, ainv, wsi)
        e0.record()
        for _ in range(10):
            ae.model_lu_inverse(lp, up, ls, sg, perm, d, ainv, wsi)
        e1.record()
        torch.cuda.synchronize()
        inv_ms = e0.elapsed_time(e1) / 10
    # beside the step: the per-block transformations of a 32-block model (32 matrices of the head dimension 128):
    # compose + gradients + inverse of all of them, the batched calls (three launches) against the full-size calls
    # matrix by matrix
    cnt, dh = 32, 128
    sets = [wl.make_lu_params(dh, seed=100 + m, kind="bd_hadamard", noise=1e-3) for m in range(cnt)]
    st = [torch.from_numpy(np.ascontiguousarray(np.stack([p[i] for p in sets]))).cuda() for i in range(5)]
    gs = torch.randn((cnt, dh, dh), device="cuda").to(td)
    sa, si = torch.empty((cnt, dh, dh), dtype=td, device="cuda"), torch.empty((cnt, dh, dh), dtype=td, device="cuda")
    sl, su, ss = torch.empty((cnt, dh, dh), device="cuda"), torch.empty((cnt, dh, dh), device="cuda"), torch.empty((cnt, dh), device="cuda")
    wsm = torch.empty(max(ae.model_lu_workspace(dh, ae.DTYPES[args.dtype]), ae.model_lu_inverse_workspace(dh)), dtype=torch.uint8, device="cuda")

    def small_batched():
        ae.model_lu_compose_batch(*st, cnt, dh, sa)
        ae.model_lu_backward_batch(gs, *st, cnt, dh, sl, su, ss)
        ae.model_lu_inverse_batch(*st, cnt, dh, si)

    def small_looped():
        for m in range(cnt):
            pm = [t[m] for t in st]
            ae.model_lu_compose(*pm, dh, sa[m], wsm)
            ae.model_lu_backward(gs[m], *pm, dh, sl[m], su[m], ss[m], wsm)
            ae.model_lu_inverse(*pm, dh, si[m], wsm)

    small_ms = {}
    for name, fn, reps in (("batched", small_batched, 20), ("looped_full_size", small_looped, 3)):
        fn()
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        small_ms[name] = (time.perf_counter() - c0) / reps * 1e3
    flops = 2.0 * d ** 3                     # 3 x (2/3) d^3
    ach = flops / 3.0 / avg_ms / 1e9
    es = a.element_size()
    from oracle import affine_oracle as ao
    c0 = time.perf_counter()
    reps = 0
    while time.perf_counter() - c0 < (1.0 if args.no_cpu_baseline else 12.0):
        ao.lu_compose(*params)
        ao.vol_penalty(params[2])
        ao.lu_gradients(g_h.astype(np.float64), *params)
        reps += 1
    ct = time.perf_counter() - c0
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = 1
    return {
        "metric": "matrices/sec, LU-parametrised %d x %d matrix: compose + regulariser + parameter gradients" % (d, d),
        "value": args.steps / dt, "unit": "matrices/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": "lu_param: A = P L (U + diag s), d = %d, block-Hadamard initialisation + noise" % d, "d": d,
                   "inverse_ms_beside_the_step": inv_ms,
                   "per_block_matrices_32x128_compose_gradients_inverse_ms": small_ms},
        # the three GEMM launches of a step (62 % of its kernel time; twelve element-wise kernels are the rest)
        "roofline": {"bound": "mfma", "kernel": "k_igemm (triangular K ranges)", "achieved": ach, "peak": PEAK[args.dtype],
                     "unit": "TFLOP/s", "frac": ach / PEAK[args.dtype], "achieved_whole_step": flops / step_ms / 1e9,
                     "traffic": LU_TRAFFIC_BYTES.get(args.dtype) if d == 4096 else None, "avg_ms": avg_ms, "launches_per_step": 3,
                     "flops_per_launch": flops / 3, "bytes_per_launch": 3.0 * d * d * es, "step_ms_under_events": step_ms},
        "cpu_baseline": {"value": reps / ct, "unit": "matrices/s", "cores": cores, "kind": "oracle",
                         "sample": "%d full steps (d = 4096, float64) in %.1f s" % (reps, ct)},
    }


# measured HBM bytes per launch of the folding products (profiles/fold_attention.md)
FOLD_TRAFFIC_BYTES = {"bf16": 1.29e8}     # average of the six product launches of a step


def bench_fold(torch, ae, args):
    """One step = folding T1 (residual stream, d = 4 096) and T2 (one 128 x 128 matrix shared by the heads) into the four
    projections of one attention block of an 8-billion-parameter-class model: Q [4096][4096] and K [1024][4096]
    (T1^-1 on the input), V [1024][4096] (T2 after, T1^-1 before), O [4096][4096] (A1 after, T2^-1 before).
    Algorithmic FLOPs: 2 * out * in * (side of each factor), summed over the factors."""
    d, dh, dkv = 4096, 128, 1024
    bf = args.dtype == "bf16"
    td = torch.bfloat16 if bf else torch.float32
    rng = np.random.default_rng(21)
    a1, v1, a1inv = wl.make_transform(d, seed=21, bf16=bf, kind="affine")
    a2, v2, a2inv = wl.make_transform(dh, seed=22, bf16=bf, kind="affine")
    dev = lambda a, t=td: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda().to(t).contiguous()
    f32 = torch.float32
    layers = []            # (name, out, in, a_left, v_left, a_right_inv, v_right)
    for name, out, inn, al, vl, ar, vr in (("q", d, d, None, None, a1inv, v1), ("k", dkv, d, None, None, a1inv, v1),
                                           ("v", dkv, d, a2, v2, a1inv, v1), ("o", d, d, a1, None, a2inv, v2)):
        W = (rng.standard_normal((out, inn)) / np.sqrt(inn)).astype(np.float32)
        b = rng.standard_normal(out).astype(np.float32)
        layers.append(dict(name=name, out=out, inn=inn, W_h=W, b_h=b, al_h=al, vl_h=vl, ar_h=ar, vr_h=vr,
                           W=dev(W), b=dev(b, f32), al=None if al is None else dev(al), vl=None if vl is None else dev(vl, f32),
                           ar=None if ar is None else dev(ar), vr=None if vr is None else dev(vr, f32),
                           w_out=torch.empty((out, inn), dtype=td, device="cuda"), b_out=torch.empty(out, device="cuda")))
    ws_bytes = max(ae.model_fold_workspace(l["out"], l["inn"], 0 if l["al"] is None else l["al"].shape[0],
                                           0 if l["ar"] is None else l["ar"].shape[0], ae.DTYPES[args.dtype]) for l in layers)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")

    def step():
        for l in layers:
            ae.model_fold_linear(l["W"], l["b"], l["out"], l["inn"], l["al"], l["vl"], l["ar"], l["vr"], l["w_out"], l["b_out"], ws)

    flops = 0.0
    for l in layers:
        if l["ar"] is not None:
            flops += 2.0 * l["out"] * l["inn"] * l["ar"].shape[0]
        if l["al"] is not None:
            flops += 2.0 * l["out"] * l["inn"] * l["al"].shape[0]
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    step_ms = e0.elapsed_time(e1) / args.steps
    ach = flops / step_ms / 1e9
    from oracle import fold_oracle as fo
    c0 = time.perf_counter()
    reps = 0
    while time.perf_counter() - c0 < (1.0 if args.no_cpu_baseline else 12.0):
        for l in layers:
            fo.fold_linear(l["W_h"], l["b_h"], l["al_h"], l["vl_h"], l["ar_h"], l["vr_h"])
        reps += 1
    ct = time.perf_counter() - c0
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = 1
    return {
        "metric": "attention blocks/sec, folding T1 and T2 into the Q, K, V, O projections (d = 4096, 8 KV heads of 128)",
        "value": args.steps / dt, "unit": "blocks/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": "fold_attention: W~ = A_l W A_r^-1, b~ = A_l b - W~ v_r + v_l for Q, K, V, O", "d": d, "d_head": dh,
                   "kv_features": dkv},
        # all kernels of the step under the events: six products, five transposes, four bias kernels
        "roofline": {"bound": "mfma", "kernel": "k_igemm (dense)", "achieved": ach, "peak": PEAK[args.dtype], "unit": "TFLOP/s",
                     "frac": ach / PEAK[args.dtype], "traffic": FOLD_TRAFFIC_BYTES.get(args.dtype), "avg_ms": step_ms / 6,
                     "launches_per_step": 6, "flops_per_launch": flops / 6, "step_ms_under_events": step_ms},
        "cpu_baseline": {"value": reps / ct, "unit": "blocks/s", "cores": cores, "kind": "oracle",
                         "sample": "%d full steps (float64) in %.1f s" % (reps, ct)},
    }


# measured HBM bytes per product launch of the QR parametrisation (profiles/qr_param.md)
QR_TRAFFIC_BYTES = {"f32": 8.56e8}


def bench_qr_param(torch, ae, args):
    """One step = the QR parametrisation A = exp((G - G^T)/2)(R + diag s) of Eq. (5) for one d x d matrix, d = 4 096:
    compose A (order-8 Taylor polynomial in powers of X^3, five squarings), the volume regulariser, and the parameter
    gradients from dLoss/dA through the stored chain: 10 + 20 dense binary32 products of 2 d^3 FLOPs each."""
    d, squarings = 4096, 5
    td = torch.bfloat16 if args.dtype == "bf16" else torch.float32
    params = wl.make_qr_params(d, seed=13, kind="bd_orthogonal", noise=1e-3)
    g, rp, ls, sg = [torch.from_numpy(a).cuda() for a in params]
    ga_h = np.random.default_rng(14).standard_normal((d, d)).astype(np.float32)
    ga = torch.from_numpy(ga_h).cuda().to(td).contiguous()
    a = torch.empty((d, d), dtype=td, device="cuda")
    dg, dr = torch.empty((d, d), device="cuda"), torch.empty((d, d), device="cuda")
    dls, vgrad, val = torch.empty(d, device="cuda"), torch.empty(d, device="cuda"), torch.empty(1, device="cuda")
    ws = torch.empty(ae.model_qr_workspace(d, squarings), dtype=torch.uint8, device="cuda")

    def step():
        ae.model_qr_compose(g, rp, ls, sg, d, a, ws, squarings)
        ae.model_vol_penalty(ls, d, val, vgrad)
        ae.model_qr_backward(ga, rp, ls, sg, d, dg, dr, dls, ws, squarings)

    steps, warmup = min(args.steps, 5), min(args.warmup, 2)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ae.model_lu_timing(True)                 # HIP events around every matrix-core product inside the library
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    gemm_ms, launches = ae.model_lu_timing(False)
    avg_ms = gemm_ms / max(launches, 1)
    per_step = launches // steps
    flops_per_launch = 2.0 * d ** 3
    ach = flops_per_launch / avg_ms / 1e9
    # beside the step: A^-1 = (R + diag s)^-1 Q^T from the workspace the last compose left
    ae.model_qr_compose(g, rp, ls, sg, d, a, ws, squarings)
    ainv = torch.empty((d, d), dtype=td, device="cuda")
    wsi = torch.empty(ae.model_lu_inverse_workspace(d), dtype=torch.uint8, device="cuda")
    for _ in range(2):
        ae.model_qr_inverse(rp, ls, sg, d, ws, ainv, wsi, squarings)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        ae.model_qr_inverse(rp, ls, sg, d, ws, ainv, wsi, squarings)
    e1.record()
    torch.cuda.synchronize()
    inv_ms = e0.elapsed_time(e1) / 5
    from oracle import affine_oracle as ao
    cpu = None
    if not args.no_cpu_baseline:
        c0 = time.perf_counter()
        ao.qr_compose(*params)
        ao.vol_penalty(params[2])
        ao.qr_gradients(ga_h.astype(np.float64), *params)
        ct = time.perf_counter() - c0
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = 1
        cpu = {"value": 1.0 / ct, "unit": "matrices/s", "cores": cores, "kind": "oracle",
               "sample": "one full step (d = 4096, float64, library expm and its Frechet derivative) in %.1f s" % ct}
    return {
        "metric": "matrices/sec, QR-parametrised 4096 x 4096 matrix: compose + regulariser + parameter gradients",
        "value": steps / dt, "unit": "matrices/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": dt / steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "qr_param: A = exp((G - G^T)/2)(R + diag s), d = 4096, block-orthogonal initialisation + noise",
                   "d": d, "squarings": squarings, "taylor_order": 8, "storage_of_A_and_dA": args.dtype,
                   "inverse_ms_beside_the_step": inv_ms},
        "roofline": {"bound": "mfma", "kernel": "k_igemm<float> (dense)", "achieved": ach, "peak": PEAK["f32"], "unit": "TFLOP/s",
                     "frac": ach / PEAK["f32"], "traffic": QR_TRAFFIC_BYTES.get("f32"), "avg_ms": avg_ms,
                     "launches_per_step": per_step, "flops_per_launch": flops_per_launch, "bytes_per_launch": 3.0 * d * d * 4},
        "cpu_baseline": cpu,
    }


def bench_monte_carlo(torch, ae, args):
    """cfg4 end to end: the error-rate estimate over ALL 1e8 samples at each of the four SNR points — 1 525 launches of
    65 536 samples and one of 57 600 (a second handle) per point through model_monte_carlo, the two 64-bit counters
    zeroed once before and read once after each point.  value = samples/s over the whole run."""
    cfg = wl.CONFIGS["cfg4"]
    B, total, K = cfg["batch"], int(args.mc_samples or cfg["total_samples"]), 64
    m = ae.Model(cfg["spec"], B)
    tail = ae.Model(cfg["spec"], total % B) if total % B else None
    params = torch.from_numpy(wl.make_params(cfg["spec"], cfg["seed"])).cuda()
    for h in (m, tail):
        if h is not None:
            h.model_set_params_static(True)           # the parameters do not change between the launches of a run
    x = torch.empty((B, K), device="cuda")
    y = torch.empty((B, K), device="cuda")
    be = torch.zeros(1, dtype=torch.int64, device="cuda")
    ke = torch.zeros(1, dtype=torch.int64, device="cuda")
    ae.model_monte_carlo(m, tail, params, 0.0, cfg["seed"], 0, min(total, 2 * B + total % B), x, y, be, ke)   # warm-up
    torch.cuda.synchronize()
    per_snr, t_all = [], 0.0
    for snr in cfg["snr_db"]:
        be.zero_()
        ke.zero_()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ae.model_monte_carlo(m, tail, params, snr, cfg["seed"], 0, total, x, y, be, ke)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        t_all += dt
        nb, nk = int(be.item()), int(ke.item())      # the one read-back of the point
        per_snr.append(dict(snr_db=snr, seconds=round(dt, 4), samples_per_s=total / dt, bit_errors=nb, block_errors=nk,
                            ber=nb / (K * total), bler=nk / total))
    launches = total // B + (1 if total % B else 0)
    # per-kernel durations of the launch (HIP events on the stream the kernels run on): a separate short pass
    st = build_case("cfg4", torch, ae)
    st["m"].model_set_params_static(True)
    run_timed(st, ae, torch, 3, 2)
    run_timed(st, ae, torch, args.steps, 0, timing=True)
    rows = kernel_table(st, args.steps)
    st["m"].close()
    out = {
        "metric": "samples/sec, forward (Monte-Carlo error-rate estimate, all launches)", "value": len(per_snr) * total / t_all,
        "unit": "samples/s", "n_gpus": 1, "steps": launches * len(per_snr), "warmup": 3,
        "ms_per_step": t_all / (launches * len(per_snr)) * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "cfg4 full run: %s" % cfg["spec"], "batch": B, "total_samples_per_snr": total,
                   "launches_per_snr": launches, "tail_launch": total % B, "snr_db": cfg["snr_db"], "seed": cfg["seed"],
                   "pass": "message bits + forward + error count"},
        "per_snr": per_snr,
        "roofline": roofline_of(rows, "f32", "cfg4", ae),
    }
    if not args.no_cpu_baseline:
        cb = cpu_baseline("cfg4")
        cb["extrapolated_seconds_per_1e8_samples"] = total / cb["value"]
        out["cpu_baseline"] = cb
    return out


def cpu_baseline(name, threads=None, sample=None):
    """The oracle as it stands, on a bounded sample of the same workload (same layer list and
    resolution, smaller batch), timed on this machine's host cores (threads: limit its OpenMP threads)."""
    import oracle.ae_oracle as orc
    cfg = wl.CONFIGS[name]
    sample = sample or {"cfg1": 8192, "cfg2": 256, "cfg3": 16, "cfg4": 131072, "cfg5": 8}[name]   # 10-30 s of host work
    all_threads = orc.num_threads()
    if threads:
        orc.set_num_threads(threads)
    spec = cfg["spec"]
    bf = cfg["dtype"] == "bf16"
    params = wl.make_params(spec, cfg["seed"], bf16=bf)
    if name == "cfg4":
        x = orc.gen_bits(cfg["seed"], 0, sample, 64).reshape(sample, 64, 1, 1)
    else:
        x = wl.make_input(spec, sample, cfg["seed"], bf16=bf)
    net = orc.Net(spec, sample)
    t0 = time.perf_counter()
    y = net.forward(params, x, snr_db=cfg["snr_db"][0], seed=cfg["seed"])
    if cfg["backward"]:
        _, dy = orc.loss_mse(y, x.astype(np.float64))
        net.backward(params, dy)
    elif name == "cfg4":
        orc.count_errors(y.reshape(sample, 64), x.reshape(sample, 64))
    dt = time.perf_counter() - t0
    used = orc.num_threads()
    if threads:
        orc.set_num_threads(all_threads)
    return dict(value=sample / dt, unit="samples/s", cores=used, kind="oracle",
                sample="batch %d of %s (%s), one step in %.1f s" % (
                    sample, name, "forward+loss+backward" if cfg["backward"] else "forward", dt))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="cfg5", choices=sorted(wl.CONFIGS))
    ap.add_argument("--spec", default=None, help="benchmark an arbitrary layer spec instead of a named configuration")
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--dtype", default="bf16", choices=["f32", "bf16"])
    ap.add_argument("--forward-only", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true")
    ap.add_argument("--kernels", action="store_true", help="also print the per-kernel table to stderr")
    ap.add_argument("--full-run", action="store_true",
                    help="with --config cfg4: the whole Monte-Carlo estimate (1e8 samples at each SNR point: 1 525 launches "
                         "of 65 536 and one of 57 600), BER / BLER and samples/s per SNR point")
    ap.add_argument("--mc-samples", type=int, default=0, help="--full-run: samples per SNR point (default: the configuration's 1e8)")
    ap.add_argument("--no-overlap", action="store_true",
                    help="keep every kernel of the backward pass on one stream (for per-kernel profiles: with the "
                         "default two streams the weight-gradient kernels share the chip with other kernels)")
    ap.add_argument("--no-recompute", action="store_true",
                    help="store the first layer's convolution output instead of recomputing it in every pass that needs it "
                         "(model_set_recompute(0)): the library's behaviour for layers that have no recomputing path")
    ap.add_argument("--no-fused-backward", action="store_true",
                    help="run the ReLU backward / batch-norm backward sums as passes of their own instead of in the epilogue "
                         "of the kernel that produces the gradient (model_set_fused_backward(0))")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MIB",
                    help="only run a plain device-to-device copy of MIB MiB five times (reference for the "
                         "FETCH_SIZE / WRITE_SIZE counters of rocprofv3) and exit")
    ap.add_argument("--mx-quant", action="store_true",
                    help="benchmark the MX block quantiser Q(x) (blocks of 32, FP4 E2M1 elements) on 65 536 tokens x 4 096 "
                         "channels of synthetic activations instead of a network: one JSON line with roofline and cpu_baseline")
    ap.add_argument("--transform-mse", action="store_true",
                    help="benchmark the transformation error E(T) of Eq. (2) (dense affine map, MX quantiser) on 16 384 tokens x "
                         "4 096 channels instead of a network: one JSON line with roofline and cpu_baseline")
    ap.add_argument("--lu-param", action="store_true",
                    help="benchmark the LU parametrisation of Eq. (4) (compose, regulariser, parameter gradients; d = 4096) "
                         "instead of a network: one JSON line with roofline and cpu_baseline")
    ap.add_argument("--width", type=int, default=4096, metavar="D",
                    help="--lu-param: the matrix size d (a multiple of 32; the inverse is timed beside the step for multiples of 128)")
    ap.add_argument("--qr-param", action="store_true",
                    help="benchmark the QR parametrisation of Eq. (5) (matrix exponential by scaling and squaring, d = 4096; "
                         "at most 5 timed steps) instead of a network: one JSON line with roofline and cpu_baseline")
    ap.add_argument("--fold", action="store_true",
                    help="benchmark the folding of two affine transformations into the four projections of one attention block "
                         "(d = 4096) instead of a network: one JSON line with roofline and cpu_baseline")
    ap.add_argument("--mx-elem", default="fp4", choices=["fp4", "fp8", "int4"],
                    help="element format of --mx-quant (FP4 E2M1, FP8 E4M3, or the 4-bit integer reading)")
    ap.add_argument("--calibrate-mfma", action="store_true",
                    help="only run the library's plain matrix-core loop (with and without LDS fragment reads) and exit")
    ap.add_argument("--channel-sweep", action="store_true",
                    help="only time the stand-alone power-normalisation + noise kernel on 2^28 elements "
                         "(latent lengths of the configurations) against the HBM roofline and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no sharding, no collectives): use --gpus 1")

    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP library is the only implementation (no CPU fallback)")
    if args.calibrate_copy:
        src = torch.ones(args.calibrate_copy << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_mib": args.calibrate_copy, "launches": 5}))
        return
    from paper_2602_17681_amd import binding as ae

    if args.mx_quant:
        print(json.dumps(bench_mx_quant(torch, ae, args)))
        return
    if args.transform_mse:
        print(json.dumps(bench_transform_mse(torch, ae, args)))
        return
    if args.lu_param:
        print(json.dumps(bench_lu_param(torch, ae, args)))
        return
    if args.fold:
        print(json.dumps(bench_fold(torch, ae, args)))
        return
    if args.qr_param:
        print(json.dumps(bench_qr_param(torch, ae, args)))
        return
    if args.calibrate_mfma:
        res = {"kernel": "k_calib_mfma", "nominal_peak_tflops": PEAK["bf16"]}
        for key, reads, rnd in (("mfma_only_ones", 0, 0), ("mfma_6_lds_reads_per_8_ones", 6, 0),
                                ("mfma_only_random", 0, 1), ("mfma_6_lds_reads_per_8_random", 6, 1)):
            tf, mhz = max(ae.model_calibrate_mfma(reads, rnd, iters=40000) for _ in range(3))
            res[key] = {"tflops": round(tf, 1), "shader_mhz": round(mhz), "frac_of_nominal": round(tf / PEAK["bf16"], 3)}
        print(json.dumps(res))
        return
    if args.channel_sweep:
        # the channel step moves 2 elements per latent element (read z, write y; the noise is generated, never
        # read): inside the networks it handles 16 KB per sample, too little to show its bandwidth
        rows = []
        for dtype in (torch.float32, torch.bfloat16):
            for n in (64, 128, 512, 1024, 4096):
                batch = (1 << 28) // n
                z = torch.randn(batch * n, device="cuda").to(dtype)
                y = torch.empty_like(z)
                for _ in range(3):
                    ae.model_pnorm_awgn(z, y, batch, n, 10.0, 1, 0)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(10):
                    ae.model_pnorm_awgn(z, y, batch, n, 10.0, 1, 0)
                e1.record()
                torch.cuda.synchronize()
                ms = e0.elapsed_time(e1) / 10
                gbs = 2.0 * batch * n * z.element_size() / ms / 1e6
                rows.append(dict(dtype="bf16" if dtype == torch.bfloat16 else "f32", n=n, batch=batch, ms=round(ms, 4),
                                 gbs=round(gbs, 1), frac_hbm_peak=round(gbs / HBM_PEAK_GBS, 3)))
                del z, y
        print(json.dumps({"kernel": "k_pnorm_awgn", "elements": 1 << 28, "peak_gbs": HBM_PEAK_GBS, "rows": rows}))
        return

    name = args.config
    if args.full_run:
        if name != "cfg4" or args.spec:
            sys.exit("bench.py: --full-run is the Monte-Carlo run of --config cfg4")
        print(json.dumps(bench_monte_carlo(torch, ae, args)))
        return
    if args.spec:
        name = "custom"
        wl.CONFIGS[name] = dict(spec=args.spec, batch=args.batch, dtype=args.dtype, seed=7, snr_db=[10.0],
                                backward=not args.forward_only)
        args.no_per_config = True
        args.no_cpu_baseline = True
    cfg = wl.CONFIGS[name]
    st = build_case(name, torch, ae)
    if args.no_overlap:
        st["m"].model_set_overlap(False)
    if args.no_recompute:
        st["m"].model_set_recompute(False)
    if args.no_fused_backward:
        st["m"].model_set_fused_backward(False)
    # timed region: exactly `steps` steps, no instrumentation.  A configuration with several SNR points (cfg2, cfg4)
    # runs them as separate blocks of `steps` steps each: every point is reported, `value` is the rate over all of them.
    per_snr, dt = [], 0.0
    for snr in cfg["snr_db"]:
        st["snr"] = snr
        d1 = run_timed(st, ae, torch, args.steps, args.warmup if not per_snr else 1, timing=False)
        per_snr.append(dict(snr_db=snr, samples_per_s=st["B"] * args.steps / d1, ms_per_step=d1 / args.steps * 1e3))
        dt += d1
    dt /= len(per_snr)                                   # seconds per block of `steps` steps, averaged over the points
    st["snr"] = cfg["snr_db"][0]
    value = st["B"] * args.steps / dt
    # the same `steps` steps again with a pair of HIP events around every launch, recorded on the
    # stream the kernels run on (the event records cost about 15 % of the step time, so the
    # throughput above is measured without them): per-kernel durations for the roofline.  While timing is
    # enabled the library keeps every kernel on this one stream, so each duration is one kernel's own.
    dt_events = run_timed(st, ae, torch, args.steps, 0, timing=True)
    rows = kernel_table(st, args.steps)
    if args.kernels:
        for r in sorted(rows, key=lambda r: -r["ms_per_step"]):
            print("%-34s %9.4f ms/step  avg %9.4f ms  %s  %s" % (
                r["name"], r["ms_per_step"], r["avg_ms"],
                ("%8.1f TFLOP/s" % r["tflops"]) if r["tflops"] else " " * 15,
                ("%8.1f GB/s" % r["gbs"]) if r["gbs"] else ""), file=sys.stderr)
    out = {
        "metric": "samples/sec, forward%s" % ("+loss+backward" if cfg["backward"] else ""),
        "value": value, "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3, "ms_per_step_with_events": dt_events / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": "%s: %s" % (name, cfg["spec"]), "batch": st["B"], "snr_db": cfg["snr_db"],
                   "seed": cfg["seed"], "pass": "forward+loss+backward" if cfg["backward"] else "forward",
                   "backward_streams": 1 if args.no_overlap else 2,
                   "first_layer_conv_output": "stored" if args.no_recompute else "recomputed where the layer allows",
                   "inference_mode_and_static_params": not cfg["backward"]},
        "per_snr": per_snr,
        "roofline": roofline_of(rows, cfg["dtype"], name, ae),
        "kernels": [dict(name=r["name"], ms_per_step=round(r["ms_per_step"], 5),
                         tflops=None if r["tflops"] is None else round(r["tflops"], 2),
                         gbs=None if r["gbs"] is None else round(r["gbs"], 1))
                    for r in sorted(rows, key=lambda r: -r["ms_per_step"])[:12]],
    }
    st["m"].close()
    del st
    if not args.no_per_config:
        per = {}
        for other in sorted(wl.CONFIGS):
            if other == name:
                per[other] = dict(samples_per_s=value, ms_per_step=dt / args.steps * 1e3)
                continue
            torch.cuda.empty_cache()
            s2 = build_case(other, torch, ae)
            k2 = max(3, min(args.steps, 10))
            d2 = run_timed(s2, ae, torch, k2, 2)
            per[other] = dict(samples_per_s=s2["B"] * k2 / d2, ms_per_step=d2 / k2 * 1e3)
            s2["m"].close()
            del s2
        if not args.no_cpu_baseline:
            # the smallest configuration also against the oracle on ONE host thread (bounded sample)
            per["cfg1"]["cpu_oracle_one_thread"] = cpu_baseline("cfg1", threads=1, sample=1024)
        out["per_config"] = per
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(name)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
