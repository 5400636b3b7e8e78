"""GPU parity tests: the HIP library, called through its C boundary, against the CPU
oracle on the same seeded inputs.  Integer / bit work must match exactly; floating
point within 1e-4 (fp32) or 2e-2 (bf16) in relative L2 and relative max norm."""
import numpy as np
import pytest

import oracle.ae_oracle as orc
import workloads as wl
from parity_util import TOL, assert_close, rel_errors, run_case, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ae():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2602_17681_amd import binding
    return binding


# ------------------------------------------------------------------ noise: bit exact
@pytest.mark.parametrize("seed,first,batch,n", [
    (0, 0, 64, 64), (3, 65536 * 7, 1024, 128), (0x123456789ABCDEF, (1 << 32) - 5, 11, 37),
    (4, 0, 32, 4096), (99, 1 << 40, 3, 1), (7, 12345, 257, 1026), (11, 0, 1, 4_000_000)])
def test_noise_bit_exact(ae, seed, first, batch, n):
    import torch
    out = torch.empty((batch, n), dtype=torch.float32, device="cuda")
    ae.model_noise(seed, first, batch, n, out)
    torch.cuda.synchronize()
    ref = orc.noise(seed, first, batch, n)
    got = out.cpu().numpy()
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))


def test_gen_bits_bit_exact_and_count_errors(ae):
    import torch
    seed, first, B, K = 3, 65536 * 3 + 17, 4099, 64
    x = torch.empty((B, K), dtype=torch.float32, device="cuda")
    ae.model_gen_bits(seed, first, B, K, x)
    ref = orc.gen_bits(seed, first, B, K)
    assert np.array_equal(x.cpu().numpy(), ref)
    K2 = 200
    x2 = torch.empty((33, K2), dtype=torch.float32, device="cuda")
    ae.model_gen_bits(seed, 5, 33, K2, x2)
    assert np.array_equal(x2.cpu().numpy(), orc.gen_bits(seed, 5, 33, K2))
    rng = np.random.default_rng(0)
    y = np.clip((ref > 0) * 1.0 + 0.45 * rng.standard_normal((B, K)), 0, 1).astype(np.float32)
    y[0, 0] = 0.5
    be = torch.zeros(1, dtype=torch.int64, device="cuda")
    ke = torch.zeros(1, dtype=torch.int64, device="cuda")
    yd = torch.from_numpy(y).cuda()
    ae.model_count_errors(yd, x, B, K, be, ke)
    ae.model_count_errors(yd, x, B, K, be, ke)      # counters accumulate
    rb, rk = orc.count_errors(y, ref)
    assert (int(be.item()), int(ke.item())) == (2 * rb, 2 * rk)


# ------------------------------------------------------------------ channel kernel alone
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("batch,n", [(1000, 128), (64, 64), (7, 4096), (5, 1024), (3, 36), (513, 8), (33, 4), (70001, 32), (9, 256),
                                     (11, 192)])
def test_pnorm_awgn_standalone(ae, dtype, batch, n):
    import torch
    rng = np.random.default_rng(n)
    z = rng.standard_normal((batch, n)).astype(np.float32) * 3.0
    z[1] = 0.0          # all-zero sample: output is pure noise
    if dtype == "bf16":
        z = wl.round_to_bf16(z)
    zd = to_dev(z, dtype, torch)
    yd = torch.empty_like(zd)
    ae.model_pnorm_awgn(zd, yd, batch, n, 5.0, 42, 1000)
    zi = zd.clone()
    ae.model_pnorm_awgn(zi, zi, batch, n, 5.0, 42, 1000)        # in place: the header allows y to be z
    assert torch.equal(zi, yd)
    net = orc.Net("in:%dx1x1,pnorm,awgn" % n, batch)
    ref = net.forward(np.zeros(0, np.float32), z.reshape(batch, n, 1, 1), snr_db=5.0, seed=42, first_sample=1000)
    got = yd.float().cpu().numpy()
    assert_close(got, ref.reshape(batch, n), TOL[dtype] if dtype == "bf16" else 2e-6, "pnorm_awgn")
    if dtype == "f32":
        sig = np.float32(orc.sigma(5.0))
        assert np.array_equal(got[1], sig * orc.noise(42, 1000, batch, n)[1])
        pw = ((got - (sig * orc.noise(42, 1000, batch, n)).astype(np.float64)) ** 2).mean(axis=1)
        np.testing.assert_allclose(np.delete(pw, 1), 1.0, atol=1e-5)


# ------------------------------------------------------------------ small networks, every op pattern
SMALL = [
    # conv+bn+relu+pool encoder, fc latent, fc + upsampling conv decoder (several tiles, ragged sizes)
    ("in:3x12x20,conv3:8,bn,relu,pool2,conv3:12,bn,relu,pool2,flatten,fc:24,pnorm,awgn,fc:180,reshape:12x3x5,"
     "up2,conv3:8,relu,up2,conv3:3,sigmoid", 5),
    # single-channel image, conv1 latent map
    ("in:1x8x8,conv3:4,bn,relu,pool2,conv1:6,pnorm,awgn,conv1:4,up2,conv3:1,sigmoid", 7),
    # fully connected chain
    ("in:10x1x1,fc:33,relu,fc:16,pnorm,awgn,fc:20,relu,fc:10,sigmoid", 67),
    # patterns outside the benchmark configs: bn without pool, pool without bn, sigmoid+bn, awgn alone
    ("in:2x8x8,conv3:5,bn,sigmoid,conv3:4,relu,pool2,conv1:3,bn,awgn,up2,conv3:2", 3),
    # channel counts that are multiples of the vector widths
    ("in:4x8x8,conv3:16,bn,relu,pool2,conv3:32,bn,relu,pool2,flatten,fc:64,pnorm,awgn,fc:128,reshape:32x2x2,"
     "up2,conv3:16,relu,up2,conv3:8,sigmoid", 6),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", range(len(SMALL)))
def test_small_networks_forward_backward(ae, case, dtype):
    spec, batch = SMALL[case]
    # bf16: a 4-element bias gradient upstream of a batch-stat BN is a sum that cancels almost
    # completely (the BN input gradient sums to zero per channel), so its relative error is a
    # few times the bf16 rounding of its terms
    run_case(spec, batch, dtype=dtype, seed=100 + case, snr_db=7.0, first_sample=3,
             grad_tol=5e-2 if dtype == "bf16" else None)


THIN_RAGGED = [
    # the matrix-core kernels of the thin layers (first layer, last layer and its input gradient) on patches that
    # stick out of the image, widths that rule out 16-byte loads, 32 and 64 wide channels, through an upsample and not
    ("in:3x12x20,conv3:32,relu,conv3:3,sigmoid", 3),
    ("in:2x10x12,conv3:64,bn,relu,pool2,up2,conv3:2,sigmoid", 4),
    ("in:4x16x24,conv3:64,relu,conv3:4", 2),
]


@pytest.mark.parametrize("case", range(len(THIN_RAGGED)))
def test_thin_layers_on_ragged_images_binary32(ae, case):
    import torch
    spec, batch = THIN_RAGGED[case]
    run_case(spec, batch, dtype="f32", seed=120 + case, snr_db=7.0)
    # ... and those kernels are the ones that ran
    m = ae.Model(spec, batch, ae.AE_F32, 0)
    p = torch.from_numpy(wl.make_params(spec, 120 + case, perturb=True)).cuda()
    x = torch.from_numpy(wl.make_input(spec, batch, 120 + case)).cuda()
    y = torch.empty((batch,) + m.out_shape, device="cuda")
    g = torch.empty((m.n_params,), device="cuda")
    m.model_timing_reset()
    m.model_timing_enable(True)
    m.model_forward(p, x, 7.0, 120 + case, y)
    m.model_backward(p, x, torch.ones_like(y), g)
    m.model_timing_enable(False)
    names = {t["name"].split(".", 1)[1] for t in m.model_timing_read() if t["launches"]}
    m.close()
    assert {"fwd.conv_thin_in_mfma", "fwd.conv_thin_out_mfma", "bwd.dgrad_thin_mfma"} <= names, sorted(names)
    if case != 1:   # (images at least 16 wide: the thin weight gradients as well)
        assert "bwd.wgrad_thin_mfma" in names and "bwd.wgrad_thin" not in names, sorted(names)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_stored_statistics_batch_norm(ae, dtype):
    run_case("in:3x8x8,conv3:8,bn,relu,pool2,conv1:4,sigmoid", 4, dtype=dtype, seed=5, bn_mode=1)


def test_batch_norm_statistics_of_channels_far_from_zero(ae):
    """Conv biases of 30-50 standard deviations of the conv result put every channel mean far from zero, where a
    variance formed as E[x^2] - mean^2 from binary32 partial sums would lose the 1e-4 bar; the kernels take their
    partial sums about the bias.  First layer through the thin kernel, second through the implicit-GEMM epilogue."""
    spec = "in:3x16x16,conv3:64,bn,relu,pool2,conv3:64,bn,relu,pool2,conv1:4,sigmoid"
    params = wl.make_params(spec, 21, perturb=True)
    ent, _, _, _ = wl.param_layout(spec)
    rng = np.random.default_rng(21)
    for e in ent:
        if e["kind"] == "b" and e["name"].startswith("conv3"):
            params[e["offset"]:e["offset"] + e["shape"][0]] = (40.0 + 10.0 * rng.standard_normal(e["shape"][0])).astype(np.float32)
    run_case(spec, 8, dtype="f32", seed=21, snr_db=10.0, params=params)


def test_sample_offset_partition_invariance(ae):
    """Two launches of B/2 with offsets give the same outputs as one launch of B (no batch-norm here)."""
    import torch
    spec = "in:6x1x1,fc:16,relu,fc:8,pnorm,awgn,fc:16,relu,fc:6,sigmoid"
    B = 64
    params = wl.make_params(spec, 1, perturb=True)
    x = wl.make_input(spec, B, 1)
    pd = torch.from_numpy(params).cuda()
    full = ae.Model(spec, B)
    yf = torch.empty((B, 6, 1, 1), device="cuda")
    full.model_set_sample_offset(1000)
    full.model_forward(pd, torch.from_numpy(x).cuda(), 3.0, 9, yf)
    half = ae.Model(spec, B // 2)
    ys = []
    for i in range(2):
        yh = torch.empty((B // 2, 6, 1, 1), device="cuda")
        half.model_set_sample_offset(1000 + i * (B // 2))
        half.model_forward(pd, torch.from_numpy(x[i * (B // 2):(i + 1) * (B // 2)]).cuda(), 3.0, 9, yh)
        ys.append(yh)
    assert torch.equal(torch.cat(ys), yf)


# ------------------------------------------------------------------ loss
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n", [1, 1000, 3 * 32 * 32 * 17 + 5])
def test_loss_mse(ae, dtype, n):
    import torch
    rng = np.random.default_rng(n)
    y = rng.random(n).astype(np.float32)
    t = rng.random(n).astype(np.float32)
    if dtype == "bf16":
        y, t = wl.round_to_bf16(y), wl.round_to_bf16(t)
    yd, td = to_dev(y, dtype, torch), to_dev(t, dtype, torch)
    loss = torch.full((1,), 123.0, device="cuda")
    dy = torch.empty_like(yd)
    ae.model_loss_mse(yd, td, loss, dy)
    ref, dref = orc.loss_mse(y, t)
    assert abs(loss.item() - ref) <= 1e-5 * ref + 1e-12
    assert_close(dy.float().cpu().numpy(), dref, 1e-6 if dtype == "f32" else 5e-3, "dy")
    ae.model_loss_mse(yd, td, loss, None)      # overwrites, does not accumulate
    assert abs(loss.item() - ref) <= 1e-5 * ref + 1e-12


# ------------------------------------------------------------------ benchmark configurations
def test_cfg1_full_forward(ae):
    cfg = wl.CONFIGS["cfg1"]
    run_case(cfg["spec"], cfg["batch"], dtype="f32", seed=cfg["seed"], snr_db=10.0, backward=False, perturb=False)


def test_cfg1_forward_backward_perturbed(ae):
    cfg = wl.CONFIGS["cfg1"]
    run_case(cfg["spec"], 16, dtype="f32", seed=cfg["seed"], snr_db=10.0, backward=True, perturb=True)


SMALL_IMAGE = [
    (None, 64),                       # cfg1 itself
    ("in:3x16x24,conv3:16,bn,relu,pool2,conv3:48,bn,relu,pool2,flatten,fc:22,pnorm,awgn,fc:768,reshape:32x4x6,"
     "up2,conv3:32,relu,up2,conv3:3,sigmoid", 9),
    ("in:4x32x32,conv3:32,bn,relu,pool2,conv3:16,bn,relu,pool2,flatten,fc:256,pnorm,awgn,fc:1024,reshape:16x8x8,"
     "up2,conv3:32,relu,up2,conv3:4,sigmoid", 300),
]


@pytest.mark.parametrize("case", range(len(SMALL_IMAGE)))
def test_inference_mode_small_image_path(ae, case):
    """A model in inference mode runs small-image networks of cfg1's shape in three launches (one workgroup per
    sample, tensors in LDS): y against the oracle at 1e-4 and against the layer-by-layer path of the same library;
    nothing is kept for a backward pass."""
    import torch
    spec, batch = SMALL_IMAGE[case]
    spec = spec or wl.CONFIGS["cfg1"]["spec"]
    params = wl.make_params(spec, 50 + case, perturb=True)
    x = wl.make_input(spec, batch, 50 + case)
    first = (1 << 32) - 3
    y_ref = orc.Net(spec, batch).forward(params, x, snr_db=7.0, seed=50 + case, first_sample=first)
    m = ae.Model(spec, batch)
    pd, xd = torch.from_numpy(params).cuda(), torch.from_numpy(x).cuda()
    ys = []
    for k, inference in enumerate((False, True, True)):
        m.model_set_inference(inference)
        m.model_timing_reset()
        m.model_timing_enable(k == 1)
        y = torch.full((batch,) + m.out_shape, float("nan"), device="cuda")
        m.model_set_sample_offset(first)
        m.model_forward(pd, xd, 7.0, 50 + case, y)
        ys.append(y.cpu().numpy())
        assert_close(ys[-1], y_ref, 1e-4, "y (inference=%s)" % inference)
        if k == 1:      # the pass really took the three-launch path: its one timing slot saw the launch
            assert [t["name"] for t in m.model_timing_read() if t["launches"]] == ["step00.fwd.fused_small"]
    m.model_timing_enable(False)
    assert np.array_equal(ys[1], ys[2])
    assert_close(ys[1], ys[0], 2e-5, "three-launch path against the layer-by-layer path")
    g = torch.zeros(m.n_params, device="cuda")
    with pytest.raises(ae.AeError) as e:
        m.model_backward(pd, xd, torch.zeros_like(y), g)
    assert e.value.code == -4
    with pytest.raises(ae.AeError) as e:
        m.model_get_activation(0, torch.zeros((batch,) + m.model_step_info(0)[1], device="cuda"))
    assert e.value.code == -4
    m.model_set_inference(False)
    m.model_forward(pd, xd, 7.0, 50 + case, y)
    m.model_backward(pd, xd, torch.zeros_like(y), g)        # training mode again: backward works
    m.close()


FIRST_LAYER_RECOMPUTED = [
    # (spec, batch): first layer conv3 of <= 4 channels into 32 / 64 channels + bn + relu + pool2 in bf16, image a
    # whole number of 256-pixel patches (patch widths 16, 32, 64; two patch columns; one or two MFMA column tiles)
    ("in:3x16x16,conv3:32,bn,relu,pool2,conv3:32,relu,up2,conv3:3,sigmoid", 5),
    ("in:1x32x32,conv3:64,bn,relu,pool2,conv3:32,bn,relu,pool2,conv1:8,pnorm,awgn,conv1:32,up2,conv3:32,relu,up2,conv3:1,sigmoid", 3),
    ("in:4x8x128,conv3:64,bn,relu,pool2,conv3:32,relu,up2,conv3:4,sigmoid", 2),
    ("in:2x64x64,conv3:32,bn,relu,pool2,conv3:32,relu,up2,conv3:2,sigmoid", 9),
    # 128 channels on the wide side (two workgroup columns), first and last layer
    ("in:3x32x32,conv3:128,bn,relu,pool2,conv3:128,relu,up2,conv3:3,sigmoid", 7),
]


@pytest.mark.parametrize("case", range(len(FIRST_LAYER_RECOMPUTED)))
@pytest.mark.parametrize("bn_mode", [0, 1])
def test_first_layer_conv_output_recomputed_not_stored(ae, case, bn_mode):
    """A first layer conv3 + bn + relu + pool2 in bf16 never writes its convolution output: statistics, pooled
    activation, batch-norm backward sums and weight gradient each recompute it from the input.  Parity of the whole
    network against the oracle at the usual bars (the counted-decisions bar for the gradients), the timing slots
    show the path was taken, and the stored-output path of the same library (model_set_recompute(0)) gives the same
    pooled activation up to the rounding of statistics summed in another order, and gradients to 1e-2."""
    import torch
    spec, batch = FIRST_LAYER_RECOMPUTED[case]
    run_case(spec, batch, dtype="bf16", seed=70 + case, snr_db=9.0, bn_mode=bn_mode, backward=True, perturb=True,
             flips=True, tag="first-layer recompute %d" % case)
    m = ae.Model(spec, batch, ae.AE_BF16, bn_mode)
    p = torch.from_numpy(wl.make_params(spec, 70 + case, perturb=True, bf16=True, bn_mode=bn_mode)).cuda()
    x = torch.from_numpy(wl.make_input(spec, batch, 70 + case, bf16=True)).cuda().to(torch.bfloat16)
    y = torch.empty((batch,) + m.out_shape, dtype=torch.bfloat16, device="cuda")
    dy, loss = torch.empty_like(y), torch.zeros(1, device="cuda")
    res = []
    for on in (1, 0, 1):
        m.model_set_recompute(on)
        m.model_timing_reset()
        m.model_timing_enable(True)
        m.model_forward(p, x, 9.0, 70 + case, y)
        ae.model_loss_mse(y, x, loss, dy)
        g = torch.full((m.n_params,), float("nan"), device="cuda")
        m.model_backward(p, x, dy, g)
        m.model_timing_enable(False)
        names = [t["name"] for t in m.model_timing_read() if t["launches"] and t["name"].startswith("step00.")]
        assert ("step00.fwd.thin_first_bn_act_pool" in names) == bool(on), names
        assert ("step00.bwd.thin_first_wgrad" in names) == bool(on), names
        assert ("step00.fwd.thin_first_stats" in names) == bool(on and bn_mode == 0), names
        a0 = torch.empty((batch,) + m.model_step_info(0)[1], device="cuda")
        m.model_get_activation(0, a0)
        c0 = torch.empty((batch,) + m.model_get_conv_output(0), device="cuda")
        m.model_get_conv_output(0, c0)
        res.append((y.float().cpu().numpy().copy(), a0.cpu().numpy(), c0.cpu().numpy(), g.cpu().numpy()))
    m.close()
    for k in range(4):                                     # deterministic (the 32-channel layers of these networks
        assert np.array_equal(res[0][k], res[2][k])        # take the generic fallback kernels: they are, too)
    assert np.array_equal(res[0][2], res[1][2])            # the convolution output itself: same bits either way
    assert_close(res[0][1], res[1][1], 4e-3, "pooled activation, recomputed against stored", tol_max=8e-3)
    assert_close(res[0][0], res[1][0], 1e-2, "y, recomputed against stored", tol_max=3e-2)
    assert_close(res[0][3], res[1][3], 1e-2, "gradients, recomputed against stored", tol_max=5e-2)


def test_changing_the_recompute_setting_between_forward_and_backward_is_refused(ae):
    """A backward pass needs a forward pass taken with the same setting (the stored-output path keeps a tensor the
    recomputing one does not): AE_ESTATE, no kernel runs; after a new forward pass it works."""
    import torch
    spec, batch = FIRST_LAYER_RECOMPUTED[0]
    m = ae.Model(spec, batch, ae.AE_BF16)
    p = torch.from_numpy(wl.make_params(spec, 5, perturb=True, bf16=True)).cuda()
    x = torch.from_numpy(wl.make_input(spec, batch, 5, bf16=True)).cuda().to(torch.bfloat16)
    y = torch.empty((batch,) + m.out_shape, dtype=torch.bfloat16, device="cuda")
    g = torch.zeros(m.n_params, device="cuda")
    m.model_forward(p, x, 9.0, 5, y)
    m.model_set_recompute(0)
    with pytest.raises(ae.AeError) as e:
        m.model_backward(p, x, torch.ones_like(y), g)
    assert e.value.code == -4
    m.model_forward(p, x, 9.0, 5, y)
    m.model_backward(p, x, torch.ones_like(y), g)
    torch.cuda.synchronize()
    assert torch.isfinite(g).all()
    m.close()


FUSED_BACKWARD = [
    # (spec, batch, dtype, (bn_reduce passes, act_colsum passes) the epilogues replace)
    # conv + relu and conv + bn + relu (+ pool2) layers whose backward sums / masks are taken by the epilogue of the
    # input-gradient kernel of the layer above: LDS-patch kernel (256 tiles at 32 x 32), 1x1 layer, stride-2 forms
    ("in:3x32x32,conv3:64,relu,conv3:64,relu,conv3:64,bn,relu,conv3:64,bn,relu,pool2,conv1:64,pnorm,awgn,conv1:64,relu,"
     "up2,conv3:3,sigmoid", 64, "bf16", (2, 2)),
    ("in:3x32x32,conv3:64,bn,relu,pool2,conv3:128,bn,relu,pool2,conv3:128,bn,relu,pool2,conv1:64,pnorm,awgn,conv1:128,relu,"
     "up2,conv3:128,relu,up2,conv3:64,relu,up2,conv3:3,sigmoid", 32, "bf16", (2, 3)),
    # 128-wide images: the input-gradient kernels with the epilogues are the LDS-patch kernel on column strips
    ("in:64x128x128,conv3:64,relu,conv3:64,bn,relu,conv3:64", 4, "bf16", (1, 1)),
    # a stride-2 input gradient with 64 output channels and 512 tiles of 256 x 64
    ("in:64x64x64,conv3:64,relu,up2,conv3:64", 32, "bf16", (0, 1)),
    # binary32 has no such epilogues (measured on cfg2: 1.76 ms with them against 1.70 ms with the separate passes —
    # twice the bytes per element in the epilogue, few tiles per layer): nothing changes there
    ("in:3x16x16,conv3:64,bn,relu,pool2,conv3:128,bn,relu,pool2,conv1:64,pnorm,awgn,conv1:128,relu,up2,conv3:64,relu,"
     "up2,conv3:3,sigmoid", 32, "f32", (0, 0)),
]


def _with_dead_bn_channels(spec, params, bn_mode=0):
    """gamma = 0 (and a positive, resp. negative beta) in two channels of every batch-norm layer."""
    ent, _, _, _ = wl.param_layout(spec, bn_mode)
    p = params.copy()
    for e in ent:
        if e["kind"] == "gamma":
            p[e["offset"] + 1] = 0.0
            p[e["offset"] + 5] = 0.0
        if e["kind"] == "beta":
            p[e["offset"] + 1] = 0.75
            p[e["offset"] + 5] = -0.5
    return p


@pytest.mark.parametrize("case", range(len(FUSED_BACKWARD)))
@pytest.mark.parametrize("dead", [False, True])
def test_fused_backward_epilogues(ae, case, dead):
    """The ReLU backward + bias sums of conv + relu layers and the two batch-norm backward sums of conv + bn + relu
    (+ pool2) layers come out of the epilogue of the kernel that writes the layer's output gradient: parity of every
    gradient against the oracle (counted-decisions bar), the separate passes are gone from the timing slots, and
    with model_set_fused_backward(0) the same library gives the same gradients up to the order of the sums.
    dead = True: batch-norm channels with gamma = 0, whose normalised input cannot be derived from the saved
    activation (the finalize kernel takes their sums from the definition)."""
    import torch
    spec, batch, dtype, want = FUSED_BACKWARD[case]
    bf = dtype == "bf16"
    params = wl.make_params(spec, 80 + case, perturb=True, bf16=bf)
    if dead:
        params = _with_dead_bn_channels(spec, params)
    run_case(spec, batch, dtype=dtype, seed=80 + case, snr_db=9.0, backward=True, params=params, flips=bf,
             tag="fused backward %d dead=%s" % (case, dead))
    m = ae.Model(spec, batch, ae.DTYPES[dtype])
    p = torch.from_numpy(params).cuda()
    x = to_dev(wl.make_input(spec, batch, 80 + case, bf16=bf), dtype, torch)
    y = torch.empty((batch,) + m.out_shape, dtype=x.dtype, device="cuda")
    dy = to_dev(wl.make_cotangent((batch,) + m.out_shape, 80 + case), dtype, torch)
    res, slots = [], []
    for on in (1, 0, 1):
        m.model_set_fused_backward(on)
        m.model_timing_reset()
        m.model_timing_enable(True)
        m.model_forward(p, x, 9.0, 80 + case, y)
        g = torch.full((m.n_params,), float("nan"), device="cuda")
        m.model_backward(p, x, dy, g)
        m.model_timing_enable(False)
        slots.append(sorted(t["name"].split(".", 1)[1] for t in m.model_timing_read() if t["launches"] and ".bwd." in t["name"]))
        res.append(g.cpu().numpy())
    m.close()
    assert np.array_equal(res[0], res[2])
    # (sums taken in another order move the batch-norm means in the last bit, which flips single bf16 roundings of the
    # stored gradients further down: far below the parity bar, which run_case holds against the oracle above)
    assert_close(res[0], res[1], 2e-3 if bf else 1e-5, "gradients, fused epilogues against separate passes",
                 tol_max=1e-2 if bf else 1e-4)
    import collections
    gone = collections.Counter(slots[1]) - collections.Counter(slots[0])
    assert gone["bwd.bn_reduce"] == want[0] and gone["bwd.act_colsum"] == want[1], (gone, slots)


def test_inference_mode_of_a_network_without_a_fused_path(ae):
    """Inference mode changes nothing for a network that has no special path: same bits as the default mode."""
    import torch
    spec = "in:10x1x1,fc:33,relu,fc:16,pnorm,awgn,fc:20,relu,fc:10,sigmoid"
    m = ae.Model(spec, 67)
    pd = torch.from_numpy(wl.make_params(spec, 3, perturb=True)).cuda()
    xd = torch.from_numpy(wl.make_input(spec, 67, 3)).cuda()
    y0, y1 = torch.empty((67, 10, 1, 1), device="cuda"), torch.empty((67, 10, 1, 1), device="cuda")
    m.model_forward(pd, xd, 3.0, 3, y0)
    m.model_set_inference(True)
    m.model_forward(pd, xd, 3.0, 3, y1)
    assert torch.equal(y0, y1)
    m.close()


@pytest.mark.parametrize("snr_db", [0.0, 20.0])
def test_cfg2_reduced_resolution(ae, snr_db):
    spec = wl.scaled_spec("cfg2", 16)
    run_case(spec, 12, dtype="f32", seed=1, snr_db=snr_db)


def test_cfg3_reduced_resolution_bf16(ae):
    spec = wl.scaled_spec("cfg3", 16)
    run_case(spec, 6, dtype="bf16", seed=2, snr_db=5.0, flips=True)


@pytest.mark.parametrize("first,B,snr_db", [
    (0, 65536, -2.0),                    # launch 0
    (65536 * 5, 65536, 2.0), (65536 * 700, 65536, 0.0),      # two launches from the middle of the run
    (65536 * 1525, 57600, 4.0)])         # the last, shorter launch of the 1e8-sample run
def test_cfg4_launch_and_error_counts(ae, first, B, snr_db):
    import torch
    cfg = wl.CONFIGS["cfg4"]
    K = 64
    spec = cfg["spec"]
    params = wl.make_params(spec, cfg["seed"])
    m = ae.Model(spec, B)
    pd = torch.from_numpy(params).cuda()
    x = torch.empty((B, K, 1, 1), device="cuda")
    y = torch.empty((B, K, 1, 1), device="cuda")
    be = torch.zeros(1, dtype=torch.int64, device="cuda")
    ke = torch.zeros(1, dtype=torch.int64, device="cuda")
    ae.model_gen_bits(cfg["seed"], first, B, K, x)
    m.model_set_sample_offset(first)
    m.model_forward(pd, x, snr_db, cfg["seed"], y)
    ae.model_count_errors(y, x, B, K, be, ke)
    xr = orc.gen_bits(cfg["seed"], first, B, K)
    assert np.array_equal(x.cpu().numpy().reshape(B, K), xr)
    net = orc.Net(spec, B)
    yr = net.forward(params, xr.reshape(B, K, 1, 1), snr_db=snr_db, seed=cfg["seed"], first_sample=first)
    assert_close(y.cpu().numpy(), yr, 1e-4, "cfg4 y")
    # decisions agree except where the reference output sits within rounding of the threshold
    yg = y.cpu().numpy().reshape(B, K)
    yo = yr.reshape(B, K)
    near = np.abs(yo - 0.5) < 1e-4
    assert near.mean() < 1e-3
    assert np.array_equal((yg > 0.5)[~near], (yo > 0.5)[~near])
    rb, rk = orc.count_errors(yg.astype(np.float64), xr)     # counting itself is exact
    assert (int(be.item()), int(ke.item())) == (rb, rk)
    ob, _ = orc.count_errors(yo, xr)
    assert abs(rb - ob) <= int(near.sum())
    m.close()


def test_monte_carlo_run_in_launches_with_a_shorter_last_one(ae):
    """model_monte_carlo over a sample range that is not a multiple of the launch size (three launches of 4 096 and one
    of 1 000 on a second handle, starting across the 2^32 sample boundary): the two counters, read once, against the
    oracle run over the whole range as one batch, and against the same range done call by call."""
    import torch
    cfg = wl.CONFIGS["cfg4"]
    spec, seed, K = cfg["spec"], cfg["seed"], 64
    B, rest = 4096, 1000
    total, first = 3 * B + rest, (1 << 32) - 5000
    params = wl.make_params(spec, seed)
    pd = torch.from_numpy(params).cuda()
    m, tail = ae.Model(spec, B), ae.Model(spec, rest)
    for h in (m, tail):
        h.model_set_params_static(True)
    x, y = torch.empty((B, K), device="cuda"), torch.empty((B, K), device="cuda")
    be = torch.zeros(1, dtype=torch.int64, device="cuda")
    ke = torch.zeros(1, dtype=torch.int64, device="cuda")
    ae.model_monte_carlo(m, tail, pd, 1.0, seed, first, total, x, y, be, ke)
    got = (int(be.item()), int(ke.item()))
    # the same range call by call
    be2, ke2 = torch.zeros_like(be), torch.zeros_like(ke)
    ys = []
    for l in range(4):
        h, nb = (m, B) if l < 3 else (tail, rest)
        f = first + l * B
        ae.model_gen_bits(seed, f, nb, K, x[:nb])
        h.model_set_sample_offset(f)
        h.model_forward(pd, x[:nb], 1.0, seed, y[:nb])
        ae.model_count_errors(y[:nb], x[:nb], nb, K, be2, ke2)
        ys.append(y[:nb].cpu().numpy().copy())
    assert got == (int(be2.item()), int(ke2.item()))
    # the oracle over the whole range at once (no batch coupling in this network)
    xr = orc.gen_bits(seed, first, total, K)
    yo = orc.Net(spec, total).forward(params, xr.reshape(total, K, 1, 1), snr_db=1.0, seed=seed, first_sample=first).reshape(total, K)
    yg = np.concatenate(ys)
    assert_close(yg, yo, 1e-4, "monte-carlo y")
    near = np.abs(yo - 0.5) < 1e-4
    assert got == orc.count_errors(yg.astype(np.float64), xr)
    ob, ok = orc.count_errors(yo, xr)
    assert abs(got[0] - ob) <= int(near.sum()) and abs(got[1] - ok) <= int(near.any(axis=1).sum())
    # argument checks: a remainder without a second handle, a second handle of the wrong batch
    with pytest.raises(ae.AeError):
        ae.model_monte_carlo(m, None, pd, 1.0, seed, 0, total, x, y, be, ke)
    with pytest.raises(ae.AeError):
        ae.model_monte_carlo(m, m, pd, 1.0, seed, 0, total, x, y, be, ke)
    ae.model_monte_carlo(m, None, pd, 1.0, seed, 0, 2 * B, x, y, be, ke)      # a multiple needs none
    m.close()
    tail.close()


def test_cfg5_reduced_resolution_bf16(ae):
    spec = wl.scaled_spec("cfg5", 64)     # 2x2 pixels after the fifth pool: batch-norm still sees 16 values per channel
    run_case(spec, 4, dtype="bf16", seed=4, snr_db=10.0, flips=True)


# ------------------------------------------------------------------ single layers in bf16: gradients at 2e-2
LAYERS_BF16 = [
    ("in:64x16x16,conv3:128,bn,relu,pool2", 4),
    ("in:128x8x8,up2,conv3:64,relu", 4),
    ("in:64x8x8,conv3:64", 3),
    ("in:256x1x1,fc:512,relu", 64),
    ("in:128x4x4,conv1:64,pnorm,awgn", 8),
    ("in:64x4x4,conv1:128,sigmoid", 8),
    ("in:3x16x16,conv3:64,bn,relu,pool2", 4),
    ("in:64x8x8,up2,conv3:3,sigmoid", 4),
    ("in:64x6x10,conv3:128,relu,up2,conv3:64", 3),      # sides that are not powers of two, ragged tiles
    # enough tiles for the four-phase form of the upsampled conv (and the 4x4 stride-2 form of its input gradient).
    # No ReLU behind the upsampled conv: its summed weights are rounded to bf16 once more, which moves the stored
    # bf16 outputs by an ulp here and there (2.5e-3 in relative L2, inside the 2e-2 bar), and a ReLU mask taken on
    # them would then differ from the oracle's in ~0.2 % of the elements: sqrt(0.002) = 4 % in every gradient,
    # whatever the kernels do (see FLIP_C in parity_util.py); without it the gradients test the two forms themselves.
    ("in:64x16x16,conv3:64,relu,up2,conv3:64", 32),
]


@pytest.mark.parametrize("case", range(len(LAYERS_BF16)))
def test_single_layers_bf16_gradients(ae, case):
    spec, batch = LAYERS_BF16[case]
    run_case(spec, batch, dtype="bf16", seed=300 + case, snr_db=10.0)


# ------------------------------------------------------------------ backward pass on two streams
@pytest.mark.parametrize("dtype,spec,batch", [
    ("bf16", None, 8),                                                        # the largest configuration, scaled down
    ("f32", "in:6x1x1,fc:64,relu,fc:32,pnorm,awgn,fc:64,relu,fc:6,sigmoid", 512),
    # layers without activation run their weight gradient in order, between layers that use the second stream
    ("bf16", "in:64x32x32,conv3:128,relu,conv3:64,conv3:128,relu,conv3:64,relu,conv3:64", 16),
])
def test_backward_two_streams_same_bits(ae, dtype, spec, batch):
    """The weight gradients run on a second stream by default; with that switched off, and on
    repeated calls, every gradient must come out bit for bit the same (the kernels are
    deterministic, so any difference is a missing ordering between the two streams)."""
    import torch
    if spec is None:
        spec = wl.scaled_spec("cfg5", 32)
    bf = dtype == "bf16"
    m = ae.Model(spec, batch, ae.DTYPES[dtype])
    params = torch.from_numpy(wl.make_params(spec, 11, bf16=bf)).cuda()
    x = torch.from_numpy(wl.make_input(spec, batch, 11, bf16=bf)).cuda().to(m.tdtype).contiguous()
    y = torch.empty((batch,) + m.out_shape, dtype=m.tdtype, device="cuda")
    dy = torch.from_numpy(wl.make_cotangent((batch,) + m.out_shape, 11, bf16=bf)).cuda().to(m.tdtype).contiguous()
    got = []
    for overlap in (False, True, True, False, True):
        m.model_set_overlap(overlap)
        g = torch.full((m.n_params,), float("nan"), dtype=torch.float32, device="cuda")
        m.model_forward(params, x, 10.0, 11, y)
        m.model_backward(params, x, dy, g)
        # no synchronisation here: the copy below is enqueued on the same stream as the call
        got.append(g.cpu().numpy())
    m.close()
    assert np.all(np.isfinite(got[0]))
    for k in range(1, len(got)):
        assert np.array_equal(got[0], got[k]), "call %d differs from the single-stream result" % k


@pytest.mark.parametrize("name,dtype,batch", [("cfg2", "f32", 32), ("cfg5", "bf16", 4)])
def test_forward_and_backward_replay_from_a_captured_graph(ae, name, dtype, batch):
    """The calls make no allocation and no host synchronisation, and the library's second stream is forked from and
    joined into the caller's by events, so a caller may capture them into a HIP graph: four replays, with eager calls
    (same handle, other buffers) and synchronisations between them, each bit for bit the eager result.  The bf16
    case takes the recomputing first layer and the fused backward epilogues."""
    import torch
    spec = wl.CONFIGS[name]["spec"]
    bf = dtype == "bf16"
    m = ae.Model(spec, batch, ae.DTYPES[dtype])
    params = torch.from_numpy(wl.make_params(spec, 11, bf16=bf)).cuda()
    x = to_dev(wl.make_input(spec, batch, 11, bf16=bf), dtype, torch)
    y0 = torch.empty((batch,) + m.out_shape, device="cuda", dtype=x.dtype)
    y1 = torch.full_like(y0, float("nan"))
    dy = to_dev(wl.make_cotangent((batch,) + m.out_shape, 11), dtype, torch)
    g0 = torch.empty(m.n_params, device="cuda")
    g1 = torch.full_like(g0, float("nan"))

    def run(y, g):
        m.model_forward(params, x, 10.0, 11, y)
        m.model_backward(params, x, dy, g)

    run(y0, g0)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=s):
        run(y1, g1)
    for _ in range(4):
        y1.fill_(float("nan"))
        g1.fill_(float("nan"))
        run(y0, g0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y0, y1) and torch.equal(g0, g1)
    del graph
    m.close()


# ------------------------------------------------------------------ error handling (host side, no kernel faults)
def test_error_codes(ae):
    import torch
    with pytest.raises(ae.AeError) as e:
        ae.Model("in:3x4x4,relu", 2)
    assert e.value.code == -2
    with pytest.raises(ae.AeError) as e:
        ae.Model("in:3x5x5,conv3:4,pool2", 2)
    assert e.value.code == -3
    with pytest.raises(ae.AeError) as e:
        ae.Model("in:3x4x4,conv3:4", 0)
    assert e.value.code == -1
    m = ae.Model("in:3x4x4,conv3:4", 2)
    p = torch.zeros(m.n_params, device="cuda")
    x = torch.zeros((2, 3, 4, 4), device="cuda")
    g = torch.zeros(m.n_params, device="cuda")
    with pytest.raises(ae.AeError) as e:
        m.model_backward(p, x, torch.zeros((2, 4, 4, 4), device="cuda"), g)
    assert e.value.code == -4
    assert ae.lib.model_forward(m._h, None, None, 1.0, 0, None, None) == -1
    assert "null" in ae.model_last_error()


def test_calibration_loop_and_its_argument_checks(ae):
    """The plain matrix-core loop (a measurement aid) runs, reports a rate in the range of the
    hardware (above the fp32 vector peak, not above the datasheet's bf16 peak), and rejects bad arguments."""
    import ctypes as C
    import torch
    plain, mhz = ae.model_calibrate_mfma(0, 0, iters=500)
    with_lds, _ = ae.model_calibrate_mfma(6, 0, iters=500)
    rnd, mhz_rnd = ae.model_calibrate_mfma(0, 1, iters=500)
    assert 160.0 < with_lds <= plain * 1.05 and plain < 2500.0 * 1.02, (plain, with_lds)
    assert 160.0 < rnd <= plain * 1.05 and 500.0 < mhz_rnd < 2600.0 and 500.0 < mhz < 2600.0, (rnd, mhz, mhz_rnd)
    out = C.c_double()
    scratch = torch.zeros(512, device="cuda")
    sp = C.c_void_p(scratch.data_ptr())
    assert ae.lib.model_calibrate_mfma(3, 0, 100, sp, C.byref(out), None, None) == -1
    assert ae.lib.model_calibrate_mfma(0, 0, 0, sp, C.byref(out), None, None) == -1
    assert ae.lib.model_calibrate_mfma(0, 0, 100, None, C.byref(out), None, None) == -1
    assert ae.lib.model_calibrate_mfma(0, 0, 100, C.c_void_p(scratch.data_ptr() + 4), C.byref(out), None, None) == -1


# ------------------------------------------------------------------ full benchmark sizes
@pytest.mark.parametrize("snr_db", wl.CONFIGS["cfg2"]["snr_db"])
def test_cfg2_full_size_forward_backward(ae, snr_db):
    """cfg2 exactly as bench.py runs it (batch 256, 3x32x32, fp32) at each SNR point of its sweep: every activation
    and every gradient of the training step."""
    cfg = wl.CONFIGS["cfg2"]
    run_case(cfg["spec"], cfg["batch"], dtype="f32", seed=cfg["seed"], snr_db=snr_db, perturb=False, flips=True, cot="mse")


FULL_SIZE_LINEAR = [
    # decision-free layers at the sizes bench.py runs: conv forward, input gradient and weight gradient
    # (cfg2: 64->128 at 16x16, batch 256, fp32; cfg5: 64->128 at 128x128 and up2+128->64, bf16, batch 8)
    ("in:64x16x16,conv3:64,conv3:128", 256, "f32"),
    ("in:64x32x32,up2,conv3:64,conv1:32", 8, "f32"),
    ("in:64x128x128,conv3:64,conv3:128", 8, "bf16"),
    ("in:128x64x64,conv3:128,up2,conv3:64", 8, "bf16"),
    # both forms of an upsampled conv at a size where the forward takes the four-phase form without
    # split-K (4 phases x 128 tiles) and the input gradient runs as one launch of 256 tiles
    ("in:64x32x32,conv3:256,up2,conv3:64", 32, "bf16"),
    # images wider than the 64-pixel tile of the LDS-patch kernel: column strips with halo columns from the neighbour
    # (fp32; 128 and 256 wide, a height that is not a power of two)
    ("in:16x128x128,conv3:64,conv3:64", 4, "f32"),
    ("in:32x12x256,conv3:64,relu,conv3:128", 24, "bf16"),
    # the patch kernel with an odd number of channel slabs (96 bf16 / 48 fp32 channels = 3 slabs of 64 bytes) and three
    # 64-wide column tiles (192 output channels), 32- and 16-pixel-wide images; weights in fragment order throughout
    ("in:96x32x32,conv3:192,conv3:64", 64, "bf16"),
    ("in:48x16x16,conv3:64,conv3:128", 256, "f32"),
]


@pytest.mark.parametrize("case", range(len(FULL_SIZE_LINEAR)))
def test_full_size_linear_layers(ae, case):
    spec, batch, dtype = FULL_SIZE_LINEAR[case]
    run_case(spec, batch, dtype=dtype, seed=400 + case, snr_db=10.0)


def test_network_with_more_layers_than_one_packing_launch_holds(ae):
    """35 convolution layers: the weights of a pass are then repacked layer by layer instead of by one launch for all
    (the other packing kernel) — among them two 3x3 layers that run with the input patch in LDS and take their weights
    in MFMA fragment order, forward and input gradient."""
    spec = "in:16x16x16,conv3:64,relu," + "conv1:32,relu,conv1:64,relu," * 16 + "conv3:64,relu,conv1:16"
    run_case(spec, 256, dtype="f32", seed=77, snr_db=10.0, flips=True, tag="35 layers")


def test_cfg3_full_size_forward_backward(ae):
    """cfg3 at its full size (batch 128, 3x64x64, bf16) as bench.py runs it: y and every saved activation against both
    oracles, every gradient of the training step (the upstream gradient is the MSE gradient) against the oracle."""
    cfg = wl.CONFIGS["cfg3"]
    run_case(cfg["spec"], cfg["batch"], dtype="bf16", seed=cfg["seed"], snr_db=5.0, perturb=False, flips=True, cot="mse")


def test_cfg5_full_size_forward_backward(ae):
    """cfg5 at its full size (batch 32, 3x256x256, bf16), the launch configuration bench.py times: y and every saved
    activation against the plain and the bf16-storage oracle, and every gradient of the training step (forward,
    MSE gradient, backward) against the oracle — with the bar that follows from the counted decision flips, and at
    2e-2 under the same decisions."""
    cfg = wl.CONFIGS["cfg5"]
    run_case(cfg["spec"], cfg["batch"], dtype="bf16", seed=cfg["seed"], snr_db=10.0, perturb=False, flips=True, cot="mse")


def test_cfg5_full_resolution_backward_small_batch(ae):
    """Backward of cfg5 at full 256x256 resolution with a generic (random) upstream gradient, batch 2."""
    cfg = wl.CONFIGS["cfg5"]
    run_case(cfg["spec"], 2, dtype="bf16", seed=cfg["seed"], snr_db=10.0, perturb=False, check_acts=False, flips=True)


def test_cfg5_full_size_backward_properties(ae):
    """Properties of the full-size cfg5 backward that hold at any size: run-to-run determinism (the
    first run keeps every kernel on one stream, the others use the second stream for the weight
    gradients), exact linearity in dy for a power-of-two factor, zero bias gradient in front of
    batch-stat BN."""
    import torch
    cfg = wl.CONFIGS["cfg5"]
    B = cfg["batch"]
    m = ae.Model(cfg["spec"], B, ae.AE_BF16)
    p = torch.from_numpy(wl.make_params(cfg["spec"], cfg["seed"], bf16=True)).cuda()
    x = torch.from_numpy(wl.make_input(cfg["spec"], B, cfg["seed"], bf16=True)).cuda().to(torch.bfloat16)
    y = torch.empty((B,) + m.out_shape, dtype=torch.bfloat16, device="cuda")
    dy = torch.empty_like(y)
    loss = torch.zeros(1, device="cuda")
    grads = []
    for k, scale in enumerate((1.0, 1.0, 4.0)):
        m.model_set_overlap(k > 0)
        m.model_forward(p, x, 10.0, cfg["seed"], y)
        ae.model_loss_mse(y, x, loss, dy)
        g = torch.full((m.n_params,), float("nan"), device="cuda")
        m.model_backward(p, x, (dy * scale).contiguous(), g)
        torch.cuda.synchronize()
        assert torch.isfinite(g).all()
        grads.append(g)
    assert torch.equal(grads[0], grads[1])                 # deterministic
    # dy*4 is exact in bf16, and every stage is linear in the incoming gradient up to bf16 rounding of
    # the stored gradients, which commutes with a power-of-two scale: bit-exact linearity
    assert torch.equal(grads[2], grads[0] * 4.0)
    ent, _, _, _ = wl.param_layout(cfg["spec"])
    toks = cfg["spec"].split(",")[1:]
    for e in ent:
        if e["kind"] == "b" and e["op"] + 1 < len(toks) and toks[e["op"] + 1] == "bn":
            sl = slice(e["offset"], e["offset"] + e["shape"][0])
            assert float(grads[0][sl].abs().max()) == 0.0
    m.close()
