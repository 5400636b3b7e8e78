"""Pins of the CPU oracle to things other than itself: published known-answer vectors,
closed forms, invariants, library routines on special cases, brute force, finite
differences.  A plausible mistake anywhere in the oracle (dropped term, wrong sign or
index, transposed operand) should fail at least one test here.  CPU only."""
import os

import numpy as np
import pytest
from scipy import signal, stats

import oracle.ae_oracle as orc
import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ Philox
def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(GOLD, "philox4x32_10_kat.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) == 3
    for r in rows:
        v = [int(t, 16) for t in r]
        out = orc.philox4x32_10(v[0:4], v[4:6])
        assert [int(o) for o in out] == v[6:10]


def _philox_py(ctr, key):
    """Second, independent transcription in Python integers (10 rounds, 9 key bumps)."""
    c = list(ctr)
    k = list(key)
    for r in range(10):
        if r:
            k[0] = (k[0] + 0x9E3779B9) & 0xFFFFFFFF
            k[1] = (k[1] + 0xBB67AE85) & 0xFFFFFFFF
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & 0xFFFFFFFF, (p0 >> 32) ^ c[3] ^ k[1], p0 & 0xFFFFFFFF]
    return c


def test_philox_random_counters_against_python_ints():
    rng = np.random.default_rng(11)
    for _ in range(200):
        ctr = [int(v) for v in rng.integers(0, 2**32, 4)]
        key = [int(v) for v in rng.integers(0, 2**32, 2)]
        assert [int(o) for o in orc.philox4x32_10(ctr, key)] == _philox_py(ctr, key)


# ------------------------------------------------------------------ u32 -> normal
def test_gauss_matches_double_precision_box_muller():
    rng = np.random.default_rng(5)
    w = rng.integers(0, 2**32, size=(1_000_000, 2), dtype=np.uint64).astype(np.uint32)
    edge = np.array([[0, 0], [1, 1], [0xFFFFFFFF, 0xFFFFFFFF], [0xFFFFFF00, 0x40000000], [0x80000000, 0x80000000],
                     [2, 0xC0000000], [0xFFFFFFFF, 0x3FFFFFFF], [0, 0x7FFFFFC0], [3, 0x20000000], [0x7FFFFFFF, 0x1FFFFFC0]],
                    dtype=np.uint32)
    w = np.concatenate([edge, w])
    # also many small w0 (deep tail) and w0 near the top (rho near 0)
    tail = np.stack([np.arange(0, 4096, dtype=np.uint32), rng.integers(0, 2**32, 4096, dtype=np.uint64).astype(np.uint32)], 1)
    top = np.stack([np.uint32(0xFFFFFFFF) - np.arange(0, 4096, dtype=np.uint32) * 64,
                    rng.integers(0, 2**32, 4096, dtype=np.uint64).astype(np.uint32)], 1)
    w = np.concatenate([w, tail, top])
    g32, g64 = orc.gauss_many(w)
    assert np.all(np.isfinite(g32))
    err = np.abs(g32.astype(np.float64) - g64)
    # Two error sources.  (1) polynomial + rounding error of the float32 op sequence:
    # a few 1e-7 relative, bounded here by 4e-6*max(1,|g|).  (2) u itself is a float32:
    # |u32 - u| <= 2^-24, so |ln u32 - ln u| <= 2^-23 for u >= 1/2 and the radius
    # rho = sqrt(-2 ln u) moves by at most min(sqrt(2 * 2^-23), 2^-23 / rho).  (2) only
    # matters for |g| < ~1e-2 (u within 1e-4 of 1), where the density is flat.
    rho = np.hypot(g64[:, 0], g64[:, 1])[:, None]
    quant = np.minimum(np.sqrt(2.0 ** -22), 2.0 ** -23 / np.maximum(rho, 1e-300))
    bound = 4e-6 * np.maximum(1.0, np.abs(g64)) + quant
    assert np.all(err <= bound), float((err / bound).max())
    # away from the centre the plain bound holds on its own
    far = (rho > 0.05).ravel()
    assert np.all(err[far] <= 4e-6 * np.maximum(1.0, np.abs(g64[far])))
    assert far.mean() > 0.99
    # largest magnitude possible: sqrt(2*33*ln 2)
    assert np.abs(g32).max() <= np.sqrt(2 * 33 * np.log(2)) * (1 + 1e-6)


def test_gauss_moments_and_ks():
    n = 4_000_000
    g = orc.noise(seed=77, first_sample=0, batch=1, n=n).astype(np.float64).ravel()
    assert abs(g.mean()) < 4.0 / np.sqrt(n)
    assert abs(g.var() - 1.0) < 4.0 * np.sqrt(2.0 / n)
    assert abs(stats.skew(g)) < 4.0 * np.sqrt(6.0 / n)
    assert abs(stats.kurtosis(g)) < 4.0 * np.sqrt(24.0 / n)
    assert stats.kstest(g[:1_000_000], "norm").pvalue > 1e-3
    # pairs from one word pair are uncorrelated, as are neighbours
    assert abs(np.corrcoef(g[0::2], g[1::2])[0, 1]) < 4.0 / np.sqrt(n / 2)


def test_noise_counter_layout_and_partition_invariance():
    seed, first, B, n = 0x123456789ABCDEF, (1 << 32) - 3, 7, 37   # crosses the 32-bit sample boundary, ragged n
    full = orc.noise(seed, first, B, n)
    # layout: element i of global sample g uses Philox(ctr=(g_lo,g_hi,i>>2,0), key=(seed_lo,seed_hi)), word pair (i&3)>>1
    for b in (0, 3, 6):
        g = first + b
        for i in (0, 1, 2, 3, 4, 17, 36):
            wds = orc.philox4x32_10([g & 0xFFFFFFFF, g >> 32, i >> 2, 0], [seed & 0xFFFFFFFF, seed >> 32])
            pair = (i & 3) >> 1
            g32, _ = orc.gauss_many(np.array([[wds[2 * pair], wds[2 * pair + 1]]], dtype=np.uint32))
            assert full[b, i] == g32[0, i & 1]
    a = orc.noise(seed, first, 3, n)
    b_ = orc.noise(seed, first + 3, 4, n)
    assert np.array_equal(full, np.concatenate([a, b_]))
    assert not np.array_equal(orc.noise(seed + 1, first, B, n), full)


# ------------------------------------------------------------------ layers, forward
def _run(spec, batch, params, x, **kw):
    net = orc.Net(spec, batch, kw.pop("bn_mode", 0))
    y = net.forward(params, x, **kw)
    return net, y


def test_conv_identity_and_single_tap_shift():
    rng = np.random.default_rng(0)
    B, C, H, W = 2, 3, 5, 6
    x = rng.standard_normal((B, C, H, W)).astype(np.float32)
    spec = "in:%dx%dx%d,conv3:%d" % (C, H, W, C)
    wgt = np.zeros((C, C, 3, 3), np.float32)
    for c in range(C):
        wgt[c, c, 1, 1] = 1.0
    p = np.concatenate([wgt.ravel(), np.zeros(C, np.float32)])
    _, y = _run(spec, B, p, x)
    assert np.array_equal(y, x.astype(np.float64))
    # single tap at (r,s)=(0,0): y[h,w] = x[h-1,w-1], zero filled (cross-correlation, pad 1)
    wgt[:] = 0
    for c in range(C):
        wgt[c, c, 0, 0] = 1.0
    p = np.concatenate([wgt.ravel(), np.zeros(C, np.float32)])
    _, y = _run(spec, B, p, x)
    exp = np.zeros_like(y)
    exp[:, :, 1:, 1:] = x[:, :, :-1, :-1]
    assert np.array_equal(y, exp)
    # tap at (2,1): y[h,w] = x[h+1,w]
    wgt[:] = 0
    for c in range(C):
        wgt[c, c, 2, 1] = 1.0
    p = np.concatenate([wgt.ravel(), np.zeros(C, np.float32)])
    _, y = _run(spec, B, p, x)
    exp = np.zeros_like(y)
    exp[:, :, :-1, :] = x[:, :, 1:, :]
    assert np.array_equal(y, exp)


@pytest.mark.parametrize("k", [1, 3])
def test_conv_against_scipy_correlate(k):
    rng = np.random.default_rng(1)
    B, Ci, Co, H, W = 2, 3, 4, 6, 5
    x = rng.standard_normal((B, Ci, H, W)).astype(np.float32)
    wgt = rng.standard_normal((Co, Ci, k, k)).astype(np.float32)
    b = rng.standard_normal(Co).astype(np.float32)
    _, y = _run("in:%dx%dx%d,conv%d:%d" % (Ci, H, W, k, Co), B, np.concatenate([wgt.ravel(), b]), x)
    exp = np.zeros((B, Co, H, W))
    for n in range(B):
        for co in range(Co):
            acc = np.full((H, W), float(b[co]))
            for ci in range(Ci):
                acc += signal.correlate2d(x[n, ci].astype(np.float64), wgt[co, ci].astype(np.float64), mode="same")
            exp[n, co] = acc
    np.testing.assert_allclose(y, exp, rtol=1e-12, atol=1e-12)


def test_fc_against_matmul_and_flatten_order():
    rng = np.random.default_rng(2)
    B, C, H, W, O = 3, 2, 3, 4, 5
    x = rng.standard_normal((B, C, H, W)).astype(np.float32)
    wgt = rng.standard_normal((O, C * H * W)).astype(np.float32)
    b = rng.standard_normal(O).astype(np.float32)
    _, y = _run("in:%dx%dx%d,flatten,fc:%d" % (C, H, W, O), B, np.concatenate([wgt.ravel(), b]), x)
    exp = x.reshape(B, -1).astype(np.float64) @ wgt.astype(np.float64).T + b
    np.testing.assert_allclose(y.reshape(B, O), exp, rtol=1e-13, atol=1e-13)
    # reshape restores (c,h,w) order
    net = orc.Net("in:%dx%dx%d,flatten,reshape:%dx%dx%d" % (C, H, W, C, H, W), B)
    assert np.array_equal(net.forward(np.zeros(0, np.float32), x), x.astype(np.float64))


def test_bn_batch_statistics_invariants():
    rng = np.random.default_rng(3)
    B, C, H, W = 4, 3, 5, 4
    x = (rng.standard_normal((B, C, H, W)) * np.array([1.0, 5.0, 0.2]).reshape(1, C, 1, 1) + 3.0).astype(np.float32)
    gamma = np.array([1.5, -0.5, 2.0], np.float32)
    beta = np.array([0.1, 0.2, -0.3], np.float32)
    spec = "in:%dx%dx%d,bn" % (C, H, W)
    _, y = _run(spec, B, np.concatenate([gamma, beta]), x)
    xd = x.astype(np.float64)
    var = xd.var(axis=(0, 2, 3))          # biased
    m = y.mean(axis=(0, 2, 3))
    v = y.var(axis=(0, 2, 3))
    np.testing.assert_allclose(m, beta, atol=1e-12)
    np.testing.assert_allclose(v, gamma.astype(np.float64) ** 2 * var / (var + 1e-5), rtol=1e-12)
    # numpy definition
    exp = gamma.reshape(1, C, 1, 1) * (xd - xd.mean(axis=(0, 2, 3), keepdims=True)) / np.sqrt(
        xd.var(axis=(0, 2, 3), keepdims=True) + 1e-5) + beta.reshape(1, C, 1, 1)
    np.testing.assert_allclose(y, exp, rtol=1e-12, atol=1e-12)
    # invariance to x -> a x + c (a power of two keeps float32 inputs exact), up to eps
    _, y2 = _run(spec, B, np.concatenate([gamma, beta]), (x * 4.0).astype(np.float32))
    bsh = beta.reshape(1, C, 1, 1).astype(np.float64)
    ratio = np.sqrt((var + 1e-5) / (var + 1e-5 / 16.0)).reshape(1, C, 1, 1)   # only eps breaks the invariance
    np.testing.assert_allclose(y2 - bsh, (y - bsh) * ratio, rtol=1e-9, atol=1e-9)
    # shift invariance (the float32 shift rounds the inputs, hence the looser tolerance)
    _, y3 = _run(spec, B, np.concatenate([gamma, beta]), (x + 8.0).astype(np.float32))
    np.testing.assert_allclose(y3, y, atol=2e-5)


def test_bn_stored_statistics_is_affine():
    rng = np.random.default_rng(4)
    B, C, H, W = 2, 3, 2, 2
    x = rng.standard_normal((B, C, H, W)).astype(np.float32)
    g, b, m, v = (rng.standard_normal(C).astype(np.float32) for _ in range(4))
    v = np.abs(v) + 0.5
    _, y = _run("in:%dx%dx%d,bn" % (C, H, W), B, np.concatenate([g, b, m, v]), x, bn_mode=1)
    sh = (1, C, 1, 1)
    exp = g.reshape(sh).astype(np.float64) * (x - m.reshape(sh).astype(np.float64)) / np.sqrt(
        v.reshape(sh).astype(np.float64) + 1e-5) + b.reshape(sh)
    np.testing.assert_allclose(y, exp, rtol=1e-12, atol=1e-12)


def test_relu_sigmoid_pool_up_against_numpy():
    rng = np.random.default_rng(5)
    B, C, H, W = 2, 3, 6, 4
    x = rng.standard_normal((B, C, H, W)).astype(np.float32)
    x[0, 0, 0, 0] = 0.0
    e = np.zeros(0, np.float32)
    xd = x.astype(np.float64)
    assert np.array_equal(_run("in:3x6x4,relu", B, e, x)[1], np.maximum(xd, 0))
    np.testing.assert_allclose(_run("in:3x6x4,sigmoid", B, e, x)[1], 1 / (1 + np.exp(-xd)), rtol=1e-15)
    assert np.array_equal(_run("in:3x6x4,pool2", B, e, x)[1], xd.reshape(B, C, 3, 2, 2, 2).max(axis=(3, 5)))
    assert np.array_equal(_run("in:3x6x4,up2", B, e, x)[1], xd.repeat(2, axis=2).repeat(2, axis=3))
    # pool(relu(x)) == relu(pool(x)) exactly
    assert np.array_equal(_run("in:3x6x4,relu,pool2", B, e, x)[1], _run("in:3x6x4,pool2,relu", B, e, x)[1])


def test_pnorm_unit_power_scale_invariance_zero():
    rng = np.random.default_rng(6)
    B, C, H, W = 5, 4, 3, 3
    z = rng.standard_normal((B, C, H, W)).astype(np.float32)
    z[2] = 0.0
    e = np.zeros(0, np.float32)
    _, x = _run("in:4x3x3,pnorm", B, e, z)
    pw = (x.reshape(B, -1) ** 2).mean(axis=1)
    np.testing.assert_allclose(pw[[0, 1, 3, 4]], 1.0, atol=1e-12)
    assert np.all(x[2] == 0.0)
    _, x2 = _run("in:4x3x3,pnorm", B, e, (z * 8.0).astype(np.float32))
    np.testing.assert_allclose(x2, x, rtol=1e-13, atol=0)
    zd = z.astype(np.float64).reshape(B, -1)
    exp = zd[0] / np.sqrt((zd[0] ** 2).mean())
    np.testing.assert_allclose(x[0].ravel(), exp, rtol=1e-14)


@pytest.mark.parametrize("snr_db", [-2.0, 0.0, 10.0, 20.0])
def test_awgn_noise_statistics_match_snr(snr_db):
    B, n = 64, 16384
    x = np.zeros((B, n, 1, 1), np.float32)
    x[:, ::2] = 1.0
    x[:, 1::2] = -1.0      # unit power already
    net = orc.Net("in:%dx1x1,pnorm,awgn" % n, B)
    y = net.forward(np.zeros(0, np.float32), x, snr_db=snr_db, seed=9, first_sample=100)
    d = (y - x.astype(np.float64)).ravel()
    N = d.size
    sig2 = 10.0 ** (-snr_db / 10.0)
    assert abs(d.mean()) < 4.0 * np.sqrt(sig2 / N)
    assert abs(d.var() / sig2 - 1.0) < 4.0 * np.sqrt(2.0 / N) + 1e-6
    if snr_db == 0.0:
        assert orc.sigma(0.0) == 1.0
        assert np.array_equal(d.reshape(B, n).astype(np.float32), orc.noise(9, 100, B, n))
    # the noise added is exactly float32(sigma) * g (float32 product)
    g = orc.noise(9, 100, B, n)
    ns = (np.float32(orc.sigma(snr_db)) * g).astype(np.float64)
    np.testing.assert_allclose(d.reshape(B, n), ns, atol=1e-15 + 1e-16 * 0, rtol=0)


def test_mse_closed_form():
    y = np.full((2, 3, 4, 4), 0.75)
    t = np.full((2, 3, 4, 4), 0.25)
    v, dy = orc.loss_mse(y, t)
    assert v == 0.25
    np.testing.assert_allclose(dy, 2 * 0.5 / y.size, rtol=1e-15)
    rng = np.random.default_rng(7)
    y = rng.random((3, 5))
    t = rng.random((3, 5))
    v, dy = orc.loss_mse(y, t)
    np.testing.assert_allclose(v, ((y - t) ** 2).mean(), rtol=1e-14)
    np.testing.assert_allclose(dy, 2 * (y - t) / y.size, rtol=1e-14)


# ------------------------------------------------------------------ adjoints / backward
def test_upsample_and_pool_adjoints():
    rng = np.random.default_rng(8)
    B, C, H, W = 2, 2, 3, 4
    x = rng.standard_normal((B, C, H, W)).astype(np.float32)
    e = np.zeros(0, np.float32)
    net = orc.Net("in:2x3x4,up2", B)
    ux = net.forward(e, x)
    gy = rng.standard_normal(ux.shape)
    _, dx = net.backward(e, gy)
    np.testing.assert_allclose((ux * gy).sum(), (x.astype(np.float64) * dx).sum(), rtol=1e-12)
    np.testing.assert_allclose(dx, gy.reshape(B, C, H, 2, W, 2).sum(axis=(3, 5)), rtol=1e-13)
    # pool backward routes to the first maximum in scan order
    xp = np.zeros((1, 1, 2, 4), np.float32)
    xp[0, 0] = [[1, 1, 0, 3], [1, 1, 3, 3]]
    net = orc.Net("in:1x2x4,pool2", 1)
    net.forward(e, xp)
    _, dx = net.backward(e, np.array([[[[5.0, 7.0]]]]))
    assert np.array_equal(dx[0, 0], np.array([[5.0, 0, 0, 7.0], [0, 0, 0, 0]]))


def _fd_check(spec, B, seed, bn_mode=0, snr_db=7.0):
    """Central finite differences of L = <forward(params,x), cot> in double precision
    against the analytic backward, for every parameter and every input element."""
    params = wl.make_params(spec, seed, bn_mode=bn_mode, perturb=True)
    x = wl.make_input(spec, B, seed)
    x = (x - 0.3).astype(np.float32)     # both signs so ReLU / pool choices vary
    net = orc.Net(spec, B, bn_mode)
    y = net.forward(params, x, snr_db=snr_db, seed=seed, first_sample=5)
    rng = np.random.default_rng(seed + 100)
    cot = rng.standard_normal(y.shape)
    grads, dx = net.backward(params, cot)

    def L(p, xx):
        return float((orc.Net(spec, B, bn_mode).forward(p, xx, snr_db=snr_db, seed=seed, first_sample=5) * cot).sum())

    def fd(vec, i, h, is_param):
        vp = vec.copy(); vm = vec.copy()
        flat_p = vp.reshape(-1); flat_m = vm.reshape(-1)
        flat_p[i] = np.float32(flat_p[i] + np.float32(h)); flat_m[i] = np.float32(flat_m[i] - np.float32(h))
        delta = float(flat_p[i]) - float(flat_m[i])
        if is_param:
            return (L(vp, x) - L(vm, x)) / delta
        return (L(params, vp) - L(params, vm)) / delta

    def compare(vec, analytic, is_param, idxs):
        scale = np.abs(analytic).max() + 1e-30
        skipped = 0
        for i in idxs:
            d1 = fd(vec, i, 2.0 ** -9, is_param)
            d2 = fd(vec, i, 2.0 ** -11, is_param)
            if abs(d1 - d2) > 2e-4 * scale:      # a ReLU / max-pool kink lies inside the stencil
                skipped += 1
                continue
            assert abs(d2 - analytic.reshape(-1)[i]) <= 1e-4 * scale, (spec, is_param, i, d2, analytic.reshape(-1)[i])
        assert skipped <= max(2, len(idxs) // 5), (skipped, len(idxs))

    n_p = params.size
    pidx = np.unique(np.concatenate([rng.choice(n_p, size=min(n_p, 60), replace=False),
                                     [e["offset"] for e in wl.param_layout(spec, bn_mode)[0]]])).astype(int)
    # stored BN statistics are buffers, not trainable: their gradient slots are defined as 0
    frozen = np.zeros(n_p, bool)
    for e in wl.param_layout(spec, bn_mode)[0]:
        if e["kind"] in ("rmean", "rvar"):
            frozen[e["offset"]:e["offset"] + int(np.prod(e["shape"]))] = True
    assert np.all(grads[frozen] == 0.0)
    pidx = pidx[~frozen[pidx]]
    compare(params, grads, True, pidx)
    xidx = rng.choice(x.size, size=min(x.size, 25), replace=False)
    compare(x, dx, False, xidx)


def test_finite_differences_conv_autoencoder():
    spec = ("in:2x4x4,conv3:3,bn,relu,pool2,flatten,fc:6,pnorm,awgn,fc:12,reshape:3x2x2,"
            "up2,conv3:2,relu,up2,conv3:1,sigmoid")
    _fd_check(spec, B=3, seed=21)


def test_finite_differences_conv1x1_latent_map_and_fc_chain():
    _fd_check("in:2x4x4,conv3:4,bn,relu,pool2,conv1:2,pnorm,awgn,conv1:3,up2,conv3:2,sigmoid", B=2, seed=22)
    _fd_check("in:5x1x1,fc:7,relu,fc:4,pnorm,awgn,fc:6,relu,fc:5,sigmoid", B=4, seed=23)


def test_finite_differences_bn_stored_statistics():
    _fd_check("in:2x4x4,conv3:3,bn,relu,pool2,conv1:2,sigmoid", B=2, seed=24, bn_mode=1)


def test_backward_structural_identities():
    """Facts that hold exactly: a bias feeding batch-stat BN has zero gradient; BN input
    gradients sum to zero per channel and are orthogonal to x-hat; the pnorm input
    gradient is orthogonal to z."""
    spec = "in:2x4x4,conv3:3,bn"
    B = 3
    params = wl.make_params(spec, 31, perturb=True)
    x = wl.make_input(spec, B, 31)
    net = orc.Net(spec, B)
    y = net.forward(params, x)
    cot = np.random.default_rng(31).standard_normal(y.shape)
    grads, _ = net.backward(params, cot)
    ent = {(e["name"], e["kind"]): e for e in wl.param_layout(spec)[0]}
    boff = ent[("conv3:3", "b")]["offset"]
    goff = ent[("bn", "gamma")]["offset"]
    assert np.abs(grads[boff:boff + 3]).max() <= 1e-12 * np.abs(grads[goff:goff + 3]).max()
    # BN alone
    xb = net.activation(0)                              # conv output = BN input
    nb = orc.Net("in:3x4x4,bn", B)
    nb.forward(params[goff:goff + 6], xb.astype(np.float32))
    _, dxb = nb.backward(params[goff:goff + 6], cot)
    xb = xb.astype(np.float32).astype(np.float64)
    var = xb.var(axis=(0, 2, 3))
    xh = (xb - xb.mean(axis=(0, 2, 3), keepdims=True)) / np.sqrt(var.reshape(1, 3, 1, 1) + 1e-5)
    assert np.abs(dxb.sum(axis=(0, 2, 3))).max() < 1e-10
    # sum dx*xh = gamma*invstd*dgamma*(1 - mean(xh^2)) and mean(xh^2) = var/(var+eps): zero up to eps
    dgamma = (cot * xh).sum(axis=(0, 2, 3))
    gam = params[goff:goff + 3].astype(np.float64)
    exp = gam / np.sqrt(var + 1e-5) * dgamma * 1e-5 / (var + 1e-5)
    np.testing.assert_allclose((dxb * xh).sum(axis=(0, 2, 3)), exp, rtol=1e-6, atol=1e-10)
    # pnorm
    z = np.random.default_rng(32).standard_normal((B, 8, 1, 1)).astype(np.float32)
    npn = orc.Net("in:8x1x1,pnorm", B)
    out = npn.forward(np.zeros(0, np.float32), z)
    g = np.random.default_rng(33).standard_normal(out.shape)
    _, dz = npn.backward(np.zeros(0, np.float32), g)
    assert np.abs((dz * z).sum(axis=(1, 2, 3))).max() < 1e-12


# ------------------------------------------------------------------ Monte-Carlo bookkeeping
def test_gen_bits_layout_and_balance():
    seed, first, B, K = 3, 1000, 512, 200      # K > 128 spans two quads
    x = orc.gen_bits(seed, first, B, K)
    assert set(np.unique(x)) == {-1.0, 1.0}
    assert abs(x.mean()) < 4.0 / np.sqrt(x.size)
    for b in (0, 77, 511):
        for j in (0, 31, 32, 127, 128, 199):
            wds = orc.philox4x32_10([first + b, 0, j >> 7, 1], [seed, 0])
            bit = (int(wds[(j >> 5) & 3]) >> (j & 31)) & 1
            assert x[b, j] == (1.0 if bit else -1.0)
    assert np.array_equal(orc.gen_bits(seed, first + 100, 50, K), x[100:150])


def test_count_errors_brute_force():
    rng = np.random.default_rng(9)
    B, K = 300, 64
    x = np.where(rng.random((B, K)) < 0.5, 1.0, -1.0).astype(np.float32)
    y = np.clip((x > 0) * 1.0 + 0.45 * rng.standard_normal((B, K)), 0, 1)
    y[0, 0] = 0.5          # exactly at the threshold decodes as 0
    be, ke = orc.count_errors(y, x)
    wrong = (y > 0.5) != (x > 0)
    assert be == int(wrong.sum()) and ke == int(wrong.any(axis=1).sum())


# ------------------------------------------------------------------ spec handling
def test_spec_shapes_and_param_counts():
    # weights-only counts follow from the layer lists: 210 208 / 4 935 040 / 70 064 896 / 720 896 / 7 884 160
    weights_only = {"cfg1": 210_208, "cfg2": 4_935_040, "cfg3": 70_064_896, "cfg4": 720_896, "cfg5": 7_884_160}
    latent = {"cfg1": 64, "cfg2": 512, "cfg3": 1024, "cfg4": 128, "cfg5": 4096}
    for name, cfg in wl.CONFIGS.items():
        net = orc.Net(cfg["spec"], 2)
        ent, n, ishape, oshape = wl.param_layout(cfg["spec"])
        assert net.n_params == n
        assert net.in_shape == ishape and net.out_shape == oshape == ishape
        assert sum(int(np.prod(e["shape"])) for e in ent if e["kind"] == "w") == weights_only[name]
        pn = [i for i, o in enumerate(net.ops) if o["kind"] == "pnorm"][0]
        assert int(np.prod(net.ops[pn]["shape"])) == latent[name]
        offs = [o["param_off"] for o in net.ops[1:] if o["kind"] in ("conv", "fc", "bn")]
        assert offs == [e["offset"] for e in ent if e["kind"] in ("w", "gamma")]


@pytest.mark.parametrize("bad", ["", "conv3:4", "in:3x4", "in:3x4x4,conv5:2", "in:3x5x5,pool2", "in:3x4x4,fc:5",
                                 "in:3x4x4,reshape:3x4x5", "in:3x4x4,conv3:0", "in:3x4x4,,relu", "in:3x4x4,foo"])
def test_bad_specs_rejected(bad):
    with pytest.raises(ValueError):
        orc.Net(bad, 2)


# ------------------------------------------------------------------ bfloat16 storage emulation
def test_store_bf16_rounding_points_and_values():
    """With store_bf16 the stored tensors are bfloat16-representable and equal to the rounded
    plain results; tensors the format never stores (inside a bn/relu/pool run) are not rounded."""
    spec = "in:3x8x8,conv3:4,bn,relu,pool2,conv1:2,sigmoid"
    B = 3
    params = wl.make_params(spec, 40, perturb=True, bf16=True)
    x = wl.make_input(spec, B, 40, bf16=True)
    plain = orc.Net(spec, B)
    plain.forward(params, x)
    emu = orc.Net(spec, B, store_bf16=True)
    emu.forward(params, x)

    def is_bf16(a):
        a32 = a.astype(np.float32)
        return np.array_equal(a32.astype(np.float64), a) and np.array_equal(wl.round_to_bf16(a32), a32)

    conv = emu.activation(0)
    assert is_bf16(conv)
    np.testing.assert_array_equal(conv, wl.round_to_bf16(plain.activation(0).astype(np.float32)).astype(np.float64))
    assert not is_bf16(emu.activation(1))            # bn output lives in registers only
    assert is_bf16(emu.activation(3))                # end of the bn/relu/pool run
    assert is_bf16(emu.activation(4)) and is_bf16(emu.activation(5))
    # ties-to-even and sign handling of the rounding itself, against the integer recipe
    v = np.array([1.00390625, 1.01171875, -1.00390625, 3.0e-5, 65280.0, 0.0, 1.0 + 2 ** -8 + 2 ** -20], np.float32)
    n = orc.Net("in:%dx1x1,relu" % v.size, 1, store_bf16=True)     # relu output is stored
    out = n.forward(np.zeros(0, np.float32), np.abs(v).reshape(1, -1, 1, 1)).ravel()
    np.testing.assert_array_equal(out, wl.round_to_bf16(np.abs(v)).astype(np.float64))


def test_store_bf16_rounds_the_gradients_of_stored_tensors():
    """Backward under the storage emulation, recomputed by hand on a two-layer chain: the gradient handed from a layer
    to the one before it (the gradient of a stored tensor) is rounded to bfloat16, parameter gradients are not, and
    they are formed from the rounded gradients."""
    spec = "in:5x1x1,fc:4,relu,fc:3"
    B = 6
    params = wl.make_params(spec, 41, perturb=True, bf16=True)
    x = wl.make_input(spec, B, 41, bf16=True)
    ent, _, _, _ = wl.param_layout(spec)
    w1, b1, w2, b2 = (params[e["offset"]:e["offset"] + int(np.prod(e["shape"]))].reshape(e["shape"]).astype(np.float64) for e in ent)
    rb = lambda a: wl.round_to_bf16(np.asarray(a, np.float32)).astype(np.float64)
    emu = orc.Net(spec, B, store_bf16=True)
    emu.forward(params, x)
    dy = rb(np.random.default_rng(41).standard_normal((B, 3, 1, 1)))
    g, dx = emu.backward(params, dy)
    xx = x.reshape(B, 5).astype(np.float64)
    h1 = rb(xx @ w1.T + b1)                              # stored fc output
    a1 = rb(np.maximum(h1, 0.0))                         # stored relu output
    d2 = dy.reshape(B, 3)
    da1 = rb(d2 @ w2)                                    # gradient of the stored relu output: rounded
    assert not np.array_equal(da1, d2 @ w2)
    dh1 = rb(da1 * (h1 > 0))                             # gradient of the stored fc output (rounding changes nothing here)
    ref = np.concatenate([(dh1.T @ xx).ravel(), dh1.sum(0), (d2.T @ a1).ravel(), d2.sum(0)])
    np.testing.assert_allclose(g, ref, rtol=1e-12, atol=1e-15)
    np.testing.assert_array_equal(dx.reshape(B, 5), rb(dh1 @ w1))
    plain = orc.Net(spec, B)
    plain.forward(params, x)
    assert not np.allclose(plain.backward(params, dy)[0], g, rtol=1e-9, atol=0)   # the plain oracle rounds nothing


# ------------------------------------------------------------------ backward with stated decisions
def test_backward_with_given_decisions_by_hand_and_against_its_own():
    """The oracle's backward can be told the ReLU pass bits and the max-pool winners instead of taking them from its
    forward values (used to compare the arithmetic of two backward passes whose forward values differ by rounding).
    By hand on one 2x2 window; and on a network: its own decisions, stated, reproduce the ordinary gradients exactly,
    while a changed winner moves the gradient where the definition says."""
    z = np.zeros(0, np.float32)
    n = orc.Net("in:1x2x2,relu,pool2", 1)
    n.forward(z, np.array([[[[1, 2], [3, -1]]]], np.float32))
    one = np.ones((1, 1, 1, 1))
    assert np.array_equal(n.backward(z, one)[1].ravel(), [0, 0, 1, 0])            # own decisions: winner (1,0)
    n.set_decisions(1, np.array([1], np.uint8))                                   # winner := (0,1)
    assert np.array_equal(n.backward(z, one)[1].ravel(), [0, 1, 0, 0])
    n.set_decisions(0, np.array([1, 0, 1, 1], np.uint8))                          # and the ReLU blocks that element
    assert np.array_equal(n.backward(z, one)[1].ravel(), [0, 0, 0, 0])
    n.set_decisions(0, None)
    n.set_decisions(1, None)
    assert np.array_equal(n.backward(z, one)[1].ravel(), [0, 0, 1, 0])
    with pytest.raises(ValueError):
        n.set_decisions(1, np.zeros(4, np.uint8))                                 # wrong size
    with pytest.raises(ValueError):
        n.set_decisions(5, np.zeros(1, np.uint8))
    spec = "in:2x6x8,conv3:5,bn,relu,pool2,conv3:4,relu,flatten,fc:6,pnorm,awgn,fc:48,reshape:4x3x4,up2,conv3:2,sigmoid"
    B = 3
    net = orc.Net(spec, B)
    params = wl.make_params(spec, 5, perturb=True)
    x = wl.make_input(spec, B, 5)
    y = net.forward(params, x, snr_db=8.0, seed=5)
    cot = np.random.default_rng(5).standard_normal(y.shape)
    g0, dx0 = net.backward(params, cot)
    kinds = [o["kind"] for o in net.ops[1:]]
    for i, k in enumerate(kinds):
        if k == "relu":
            net.set_decisions(i, (net.activation(i - 1) > 0).astype(np.uint8))
        elif k == "pool2":
            a = net.activation(i - 1)
            b, c, h, w = a.shape
            win = a.reshape(b, c, h // 2, 2, w // 2, 2).transpose(0, 1, 2, 4, 3, 5).reshape(b, c, h // 2, w // 2, 4).argmax(-1)
            net.set_decisions(i, win.astype(np.uint8))
    g1, dx1 = net.backward(params, cot)
    assert np.array_equal(g0, g1) and np.array_equal(dx0, dx1)
    ipool = kinds.index("pool2")
    win[0, 0, 0, 0] = (win[0, 0, 0, 0] + 1) % 4
    net.set_decisions(ipool, win.astype(np.uint8))
    g2, _ = net.backward(params, cot)
    assert not np.array_equal(g0, g2)
