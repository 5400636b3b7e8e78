"""GPU parity of the LU parametrisation (model_lu_compose / model_lu_backward / model_vol_penalty) against
oracle/affine_oracle.py, element by element, through the C boundary."""
import ctypes as C

import numpy as np
import pytest

import workloads as wl
from oracle import affine_oracle as ao

pytestmark = pytest.mark.gpu

# binary32 products against float64: 1e-4; bf16 operands and results (2^-9 relative each): 2e-2 — relative to the entry
# plus the same fraction of the matrix's root mean square (entries are sums of d products of mixed sign)
TOL = {"f32": 1e-4, "bf16": 2e-2}


@pytest.fixture(scope="module")
def ae():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2602_17681_amd import binding
    return binding


def _close(got, ref, tol):
    rms = float(np.sqrt(np.mean(ref ** 2))) + 1e-30
    err = np.abs(got - ref) - tol * np.abs(ref)
    return float(err.max()) <= tol * rms


def _dev(ae, params):
    import torch
    lp, up, ls, sg, perm = params
    return [torch.from_numpy(a).cuda() for a in (lp, up, ls, sg)] + [torch.from_numpy(perm).cuda()]


def _round(a, dtype):
    return wl.round_to_bf16(a.astype(np.float32)) if dtype == "bf16" else a.astype(np.float32)


def _compose(ae, params, d, dtype):
    import torch
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    a = torch.full((d, d), float("nan"), dtype=td, device="cuda")
    ws = torch.empty(ae.model_lu_workspace(d, ae.DTYPES[dtype]), dtype=torch.uint8, device="cuda")
    ae.model_lu_compose(*_dev(ae, params), d, a, ws)
    torch.cuda.synchronize()
    return a.float().cpu().numpy().astype(np.float64)


def _backward(ae, g, params, d, dtype):
    import torch
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    gt = torch.from_numpy(g.astype(np.float32)).cuda().to(td).contiguous()
    dlp = torch.full((d, d), float("nan"), device="cuda")
    dup = torch.full((d, d), float("nan"), device="cuda")
    dls = torch.full((d,), float("nan"), device="cuda")
    ws = torch.empty(ae.model_lu_workspace(d, ae.DTYPES[dtype]), dtype=torch.uint8, device="cuda")
    ae.model_lu_backward(gt, *_dev(ae, params), d, dlp, dup, dls, ws)
    torch.cuda.synchronize()
    return [t.cpu().numpy().astype(np.float64) for t in (dlp, dup, dls)]


CASES = [(32, "random"), (160, "random"), (512, "random"), (256, "bd_hadamard"), (1056, "random")]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("d,kind", CASES)
def test_compose_matches_oracle(ae, d, kind, dtype):
    params = wl.make_lu_params(d, seed=d, kind=kind, noise=1e-3 if kind == "bd_hadamard" else 0.0)
    a = _compose(ae, params, d, dtype)
    ref = ao.lu_compose(*params)
    assert _close(a, ref, TOL[dtype]), np.abs(a - ref).max()
    if kind == "bd_hadamard":                                         # the initialisation: block orthogonal up to the noise
        assert np.abs(a @ a.T - np.eye(d)).max() < (0.05 if dtype == "bf16" else 0.02)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("d,kind", CASES)
def test_backward_matches_oracle(ae, d, kind, dtype):
    params = wl.make_lu_params(d, seed=d + 1, kind=kind, noise=1e-3 if kind == "bd_hadamard" else 0.0)
    g = _round(np.random.default_rng(d).standard_normal((d, d)), dtype).astype(np.float64)
    dlp, dup, dls = _backward(ae, g, params, d, dtype)
    r_lp, r_up, r_ls = ao.lu_gradients(g, *params)
    tol = TOL[dtype]
    assert _close(dlp, r_lp, tol) and _close(dup, r_up, tol) and _close(dls, r_ls, tol)
    assert np.array_equal(np.triu(dlp), np.zeros((d, d))) and np.array_equal(np.tril(dup), np.zeros((d, d)))


def test_volume_penalty_matches_oracle(ae):
    import torch
    for d in (1, 32, 1000, 4096):
        ls = (0.05 * np.random.default_rng(d).standard_normal(d)).astype(np.float32)
        t = torch.from_numpy(ls).cuda()
        val = torch.full((1,), float("nan"), device="cuda")
        grad = torch.full((d,), float("nan"), device="cuda")
        ae.model_vol_penalty(t, d, val, grad)
        ae.model_vol_penalty(t, d, val)                                # the gradient is optional
        v_o, g_o = ao.vol_penalty(ls)
        assert abs(val.item() - v_o) <= 1e-6 * v_o + 1e-12
        assert np.allclose(grad.cpu().numpy(), g_o, rtol=1e-6, atol=1e-9)
    z = torch.zeros(64, device="cuda")
    val = torch.ones(1, device="cuda")
    ae.model_vol_penalty(z, 64, val)
    assert val.item() == 0.0                                           # |s| = 1: no penalty


def test_argument_checks(ae):
    import torch
    t = torch.zeros(64 * 64, device="cuda")
    p = C.c_void_p(t.data_ptr())
    n = C.c_int64()
    assert ae.lib.model_lu_workspace(48, 0, C.byref(n)) == -1          # d not a multiple of 32
    assert ae.lib.model_lu_workspace(64, 7, C.byref(n)) == -1          # dtype
    assert ae.lib.model_lu_workspace(32768, 0, C.byref(n)) == -1       # too large
    assert ae.lib.model_lu_workspace(64, 1, C.byref(n)) == 0 and n.value == 6 * 64 * 64 * 2 + 256
    assert ae.lib.model_lu_compose(p, p, p, p, p, 48, 0, p, p, None) == -1
    assert ae.lib.model_lu_compose(None, p, p, p, p, 64, 0, p, p, None) == -1
    assert ae.lib.model_lu_backward(p, p, p, p, p, p, 64, 0, p, p, None, p, None) == -1
    assert ae.lib.model_vol_penalty(p, 0, p, None, None) == -1
    assert "model_vol_penalty" in ae.model_last_error()


def test_product_timing_counts_launches_and_changes_nothing(ae):
    d = 256
    params = wl.make_lu_params(d, seed=3)
    a0 = _compose(ae, params, d, "bf16")
    ae.model_lu_timing(True)
    a1 = _compose(ae, params, d, "bf16")
    g = wl.round_to_bf16(np.random.default_rng(1).standard_normal((d, d)).astype(np.float32)).astype(np.float64)
    _backward(ae, g, params, d, "bf16")
    ms, n = ae.model_lu_timing(False)
    assert n == 3 and 0.0 < ms < 100.0 and np.array_equal(a0, a1)
    assert ae.model_lu_timing(False) == (0.0, 0)


def test_backward_on_two_streams_back_to_back_same_bits(ae):
    """model_lu_backward runs its two branches on two streams.  Eight calls in a row on one workspace with changing
    gradients, no synchronisation between them, against the same calls made one product at a time on one stream
    (the timing mode): identical bits."""
    import torch
    d = 1024
    params = wl.make_lu_params(d, seed=5)
    dev = _dev(ae, params)
    rng = np.random.default_rng(2)
    gs = [torch.from_numpy(rng.standard_normal((d, d)).astype(np.float32)).cuda().to(torch.bfloat16) for _ in range(8)]
    ws = torch.empty(ae.model_lu_workspace(d, ae.DTYPES["bf16"]), dtype=torch.uint8, device="cuda")

    def run():
        outs = [[torch.full((d, d), float("nan"), device="cuda"), torch.full((d, d), float("nan"), device="cuda"),
                 torch.full((d,), float("nan"), device="cuda")] for _ in gs]
        for g, o in zip(gs, outs):
            ae.model_lu_backward(g, *dev, d, o[0], o[1], o[2], ws)
        torch.cuda.synchronize()
        return outs

    two = run()
    ae.model_lu_timing(True)
    one = run()
    ae.model_lu_timing(False)
    for a, b in zip(two, one):
        for x, y in zip(a, b):
            assert torch.equal(x, y)
    assert not torch.equal(two[0][0], two[1][0])


def test_full_size_compose_and_backward(ae):
    """d = 4 096 in bf16, the launch bench.py times, every element against the oracle."""
    d = 4096
    params = wl.make_lu_params(d, seed=11, kind="bd_hadamard", noise=1e-3)
    a = _compose(ae, params, d, "bf16")
    assert _close(a, ao.lu_compose(*params), TOL["bf16"])
    g = wl.round_to_bf16(np.random.default_rng(12).standard_normal((d, d)).astype(np.float32)).astype(np.float64)
    dlp, dup, dls = _backward(ae, g, params, d, "bf16")
    r_lp, r_up, r_ls = ao.lu_gradients(g, *params)
    assert _close(dlp, r_lp, TOL["bf16"]) and _close(dup, r_up, TOL["bf16"]) and _close(dls, r_ls, TOL["bf16"])


# ------------------------------------------------------------------ the inverse of the parametrised matrix
def _inverse(ae, params, d, dtype):
    import torch
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    out = torch.full((d, d), float("nan"), dtype=td, device="cuda")
    ws = torch.empty(ae.model_lu_inverse_workspace(d), dtype=torch.uint8, device="cuda")
    ae.model_lu_inverse(*_dev(ae, params), d, out, ws)
    torch.cuda.synchronize()
    return out.float().cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("d,kind", [(128, "random"), (256, "random"), (384, "random"), (512, "bd_hadamard"), (640, "bd_hadamard"),
                                    (1024, "random"), (1408, "random"), (2048, "bd_hadamard")])
def test_inverse_matches_the_inverse_of_the_composed_matrix(ae, d, kind, dtype):
    """A^-1 from the triangular factors against numpy's inverse of the oracle's A (float64).  The blocked recursion
    runs in binary32: its error is a few 1e-7 times the condition number of the factors (below 1e2 here), so the
    binary32 result is held to 1e-4 and the bf16 result to the rounding of the output.  Sizes that are not 128 times a
    power of two (3, 5 and 11 blocks of 128) run the recursion padded with an identity block."""
    params = wl.make_lu_params(d, seed=d + 7, kind=kind, noise=1e-3 if kind == "bd_hadamard" else 0.0)
    a = ao.lu_compose(*params)
    ref = np.linalg.inv(a)
    got = _inverse(ae, params, d, dtype)
    assert _close(got, ref, TOL[dtype]), (np.abs(got - ref).max(), np.linalg.cond(a))
    if dtype == "f32":
        assert np.abs(a @ got - np.eye(d)).max() < 1e-4


def test_inverse_full_size(ae):
    """d = 4 096, bf16 output: the size bench.py times beside the parametrisation step."""
    d = 4096
    params = wl.make_lu_params(d, seed=11, kind="bd_hadamard", noise=1e-3)
    a = ao.lu_compose(*params)
    got = _inverse(ae, params, d, "bf16")
    assert _close(got, np.linalg.inv(a), TOL["bf16"])
    got32 = _inverse(ae, params, d, "f32")
    assert np.abs(a @ got32 - np.eye(d)).max() < 1e-4


def test_inverse_at_a_width_of_three_blocks_of_1024(ae):
    """d = 3 072 (a residual width of the paper's model family that is not 128 times a power of two)."""
    d = 3072
    params = wl.make_lu_params(d, seed=13, kind="bd_hadamard", noise=1e-3)
    a = ao.lu_compose(*params)
    got32 = _inverse(ae, params, d, "f32")
    assert _close(got32, np.linalg.inv(a), TOL["f32"])
    assert np.abs(a @ got32 - np.eye(d)).max() < 1e-4


def test_largest_size_exercised(ae):
    """d = 8 192 (the widest residual stream of the model family the paper evaluates): A in full against the oracle, and
    the inverse through the residual A A^-1 = I on sampled columns."""
    d = 8192
    params = wl.make_lu_params(d, seed=17, kind="bd_hadamard", noise=5e-4)
    a_ref = ao.lu_compose(*params)
    a = _compose(ae, params, d, "bf16")
    assert _close(a, a_ref, TOL["bf16"])
    del a
    inv = _inverse(ae, params, d, "f32")
    cols = np.arange(0, d, 127)
    resid = a_ref @ inv[:, cols]
    resid[cols, np.arange(len(cols))] -= 1.0
    assert np.abs(resid).max() < 1e-4
    del inv, resid, a_ref
    # the gradients at this size (the triangular products switch to 256 x 256 tiles here)
    g = wl.round_to_bf16(np.random.default_rng(18).standard_normal((d, d)).astype(np.float32)).astype(np.float64)
    dlp, dup, dls = _backward(ae, g, params, d, "bf16")
    r_lp, r_up, r_ls = ao.lu_gradients(g, *params)
    assert _close(dlp, r_lp, TOL["bf16"]) and _close(dup, r_up, TOL["bf16"]) and _close(dls, r_ls, TOL["bf16"])


def test_inverse_feeds_the_transformation_error(ae):
    """The whole chain on the GPU: parameters -> A and A^-1 -> E(T), against the oracle chain with numpy's inverse."""
    import torch
    from oracle import mx_oracle as mxo
    d, rows = 512, 512
    params = wl.make_lu_params(d, seed=21, kind="bd_hadamard", noise=2e-3)
    dp = _dev(ae, params)
    a = torch.empty((d, d), dtype=torch.bfloat16, device="cuda")
    ainv = torch.empty((d, d), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(max(ae.model_lu_workspace(d, ae.DTYPES["bf16"]), ae.model_lu_inverse_workspace(d)), dtype=torch.uint8, device="cuda")
    ae.model_lu_compose(*dp, d, a, ws)
    ae.model_lu_inverse(*dp, d, ainv, ws)
    x = wl.make_activations(rows, d, seed=5, bf16=True)
    xt = torch.from_numpy(x).cuda().to(torch.bfloat16)
    zeros = torch.zeros(d, device="cuda")
    yq = torch.empty_like(xt)
    w2 = torch.empty(ae.model_transform_mse_workspace(rows, d, ae.DTYPES["bf16"]) // 4, dtype=torch.float32, device="cuda")
    eb, et = torch.empty(d // 32, device="cuda"), torch.empty(1, device="cuda")
    ae.model_transform_mse(xt, a, zeros, ainv, zeros, rows, d, 32, yq, w2, eb, et)
    a_ref = wl.round_to_bf16(ao.lu_compose(*params).astype(np.float32))
    ainv_ref = wl.round_to_bf16(np.linalg.inv(ao.lu_compose(*params)).astype(np.float32))
    e_o, _, _ = mxo.transform_mse(x, a_ref, np.zeros(d, np.float32), ainv_ref, 32, storage="bf16")
    assert abs(et.item() - e_o) <= 2e-2 * e_o, (et.item(), e_o)


def test_inverse_argument_checks(ae):
    import torch
    t = torch.zeros(128 * 128, device="cuda")
    p = C.c_void_p(t.data_ptr())
    n = C.c_int64()
    assert ae.lib.model_lu_inverse_workspace(192, C.byref(n)) == -1        # not a multiple of 128
    assert ae.lib.model_lu_inverse_workspace(64, C.byref(n)) == -1
    assert ae.lib.model_lu_inverse_workspace(16384 + 128, C.byref(n)) == -1
    assert ae.lib.model_lu_inverse_workspace(256, C.byref(n)) == 0 and n.value == 8 * 256 * 256 * 4 + 1024
    assert ae.lib.model_lu_inverse_workspace(384, C.byref(n)) == 0 and n.value == 8 * 512 * 512 * 4 + 1024   # padded to 4 blocks
    assert ae.lib.model_lu_inverse(p, p, p, p, p, 192, 0, p, p, None) == -1
    assert ae.lib.model_lu_inverse(p, p, p, p, p, 128, 3, p, p, None) == -1
    assert ae.lib.model_lu_inverse(None, p, p, p, p, 128, 0, p, p, None) == -1


# ------------------------------------------------------------------ QR parametrisation (Eq. 5)
def _qr_run(ae, params, d, dtype, g_a=None, squarings=5):
    import torch
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    dp = [torch.from_numpy(a).cuda() for a in params]
    a = torch.full((d, d), float("nan"), dtype=td, device="cuda")
    ws = torch.empty(ae.model_qr_workspace(d, squarings), dtype=torch.uint8, device="cuda")
    ae.model_qr_compose(*dp, d, a, ws, squarings)
    out = [a.float().cpu().numpy().astype(np.float64)]
    if g_a is not None:
        gt = torch.from_numpy(g_a.astype(np.float32)).cuda().to(td).contiguous()
        dg = torch.full((d, d), float("nan"), device="cuda")
        dr = torch.full((d, d), float("nan"), device="cuda")
        dls = torch.full((d,), float("nan"), device="cuda")
        ae.model_qr_backward(gt, dp[1], dp[2], dp[3], d, dg, dr, dls, ws, squarings)
        out += [t.cpu().numpy().astype(np.float64) for t in (dg, dr, dls)]
    torch.cuda.synchronize()
    return out


QR_CASES = [(32, "random"), (96, "random"), (256, "bd_orthogonal"), (512, "random")]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("d,kind", QR_CASES)
def test_qr_compose_and_backward_match_oracle(ae, d, kind, dtype):
    """The exponential runs in binary32 whatever the storage type; bf16 only rounds dA on the way in and A on the way out."""
    params = wl.make_qr_params(d, seed=d + 3, kind=kind, noise=1e-3 if kind == "bd_orthogonal" else 0.0)
    if kind == "random":
        params = (params[0] * 2.0,) + tuple(params[1:])      # a rotation well away from the identity
    g_a = _round(np.random.default_rng(d).standard_normal((d, d)), dtype).astype(np.float64)
    a, dg, dr, dls = _qr_run(ae, params, d, dtype, g_a)
    ref = ao.qr_compose(*params)
    assert _close(a, ref, TOL[dtype]), np.abs(a - ref).max()
    r_g, r_r, r_ls = ao.qr_gradients(g_a, *params)
    tol = TOL["f32"]                                          # the gradients come out in binary32 in both cases
    assert _close(dg, r_g, tol), np.abs(dg - r_g).max()
    assert _close(dr, r_r, tol) and _close(dls, r_ls, tol)
    assert np.array_equal(dg, -dg.T) and np.array_equal(np.tril(dr), np.zeros((d, d)))
    if kind == "bd_orthogonal" and dtype == "f32":
        assert np.abs(a @ a.T - np.eye(d)).max() < 0.02      # the initialisation: orthogonal up to the noise


def test_qr_full_size(ae):
    """d = 4 096, the size bench.py times (bf16 storage of A and dA): A in full against the oracle; the gradients of
    the launch configuration at d = 1 024, where the oracle's Frechet derivative takes seconds."""
    d = 4096
    params = wl.make_qr_params(d, seed=13, kind="bd_orthogonal", noise=1e-3)
    a, = _qr_run(ae, params, d, "bf16")
    assert _close(a, ao.qr_compose(*params), TOL["bf16"])
    d = 1024
    params = wl.make_qr_params(d, seed=14, kind="bd_orthogonal", noise=1e-3)
    g_a = _round(np.random.default_rng(1).standard_normal((d, d)), "bf16").astype(np.float64)
    a, dg, dr, dls = _qr_run(ae, params, d, "bf16", g_a)
    r_g, r_r, r_ls = ao.qr_gradients(g_a, *params)
    assert _close(a, ao.qr_compose(*params), TOL["bf16"])
    assert _close(dg, r_g, TOL["f32"]) and _close(dr, r_r, TOL["f32"]) and _close(dls, r_ls, TOL["f32"])


@pytest.mark.parametrize("d", [512, 384])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_qr_inverse_matches_the_inverse_of_the_composed_matrix(ae, dtype, d):
    import torch
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    params = wl.make_qr_params(d, seed=31)
    params = (params[0] * 2.0,) + tuple(params[1:])
    dp = [torch.from_numpy(a).cuda() for a in params]
    a = torch.empty((d, d), dtype=td, device="cuda")
    ws = torch.empty(ae.model_qr_workspace(d, 5), dtype=torch.uint8, device="cuda")
    ae.model_qr_compose(*dp, d, a, ws, 5)
    ainv = torch.full((d, d), float("nan"), dtype=td, device="cuda")
    ws2 = torch.empty(ae.model_lu_inverse_workspace(d), dtype=torch.uint8, device="cuda")
    ae.model_qr_inverse(dp[1], dp[2], dp[3], d, ws, ainv, ws2, 5)
    ref = np.linalg.inv(ao.qr_compose(*params))
    assert _close(ainv.float().cpu().numpy().astype(np.float64), ref, TOL[dtype])
    assert ae.lib.model_qr_inverse(None, None, None, 512, 0, 5, None, None, None, None) == -1
    p = C.c_void_p(ws.data_ptr())
    assert ae.lib.model_qr_inverse(p, p, p, 192, 0, 5, p, p, p, None) == -1       # not a multiple of 128


def test_qr_more_squarings_for_a_large_generator(ae):
    """||S|| around 40: five squarings leave X too large for the polynomial, eight are enough."""
    d = 64
    params = wl.make_qr_params(d, seed=9)
    params = (params[0] * 40.0,) + tuple(params[1:])
    ref = ao.qr_compose(*params)
    a8, = _qr_run(ae, params, d, "f32", squarings=8)
    assert _close(a8, ref, 1e-3), np.abs(a8 - ref).max()


def test_qr_polynomial_order_at_the_documented_limit(ae):
    """||S||_2 = 16 with five squarings, the largest generator the header promises for that setting: X = S / 32 has
    norm 0.5, where the order-8 polynomial's remainder (0.5^9 / 9! = 5e-9, times 2^5 through the squarings) is at the
    level of binary32 rounding; held to 1e-4 like every binary32 result here."""
    d = 128
    params = wl.make_qr_params(d, seed=19)
    g = params[0].astype(np.float64)
    norm = np.linalg.norm((g - g.T) / 2.0, 2)
    params = ((params[0] * (16.0 / norm)).astype(np.float32),) + tuple(params[1:])
    ref = ao.qr_compose(*params)
    a5, = _qr_run(ae, params, d, "f32", squarings=5)
    assert _close(a5, ref, TOL["f32"]), np.abs(a5 - ref).max()


def test_qr_squarings_from_the_generator_norm(ae):
    """model_qr_squarings gives the smallest J with 2^J >= 2 ||S||_inf (a bound of the spectral norm); composing a
    generator of unknown size with that J meets the binary32 bar, and a NaN in the generator is refused."""
    import torch
    d = 128
    for scale in (0.01, 1.0, 40.0):
        params = wl.make_qr_params(d, seed=23)
        params = ((params[0] * scale).astype(np.float32),) + tuple(params[1:])
        g = params[0].astype(np.float64)
        s = (g - g.T) / 2.0
        ninf = np.abs(s).sum(axis=1).max()
        want = 0
        while 2.0 ** want < 2.0 * ninf:
            want += 1
        ws = torch.empty(ae.model_qr_workspace(d, 0), dtype=torch.uint8, device="cuda")
        j = ae.model_qr_squarings(torch.from_numpy(params[0]).cuda(), d, ws)
        assert abs(j - want) <= (1 if abs(np.log2(2.0 * ninf) - round(np.log2(2.0 * ninf))) < 1e-4 else 0), (j, want)
        assert 2.0 ** j >= 2.0 * np.linalg.norm(s, 2)
        a, = _qr_run(ae, params, d, "f32", squarings=j)
        ref = ao.qr_compose(*params)
        assert _close(a, ref, 1e-3 if scale > 10 else TOL["f32"]), np.abs(a - ref).max()
    bad = torch.zeros((d, d), device="cuda")
    bad[3, 5] = float("nan")
    with pytest.raises(ae.AeError):
        ae.model_qr_squarings(bad, d, ws)
    huge = torch.zeros((d, d), device="cuda")
    huge[0, 1] = 1e6
    with pytest.raises(ae.AeError):
        ae.model_qr_squarings(huge, d, ws)


def test_qr_argument_checks(ae):
    import torch
    t = torch.zeros(64 * 64, device="cuda")
    p = C.c_void_p(t.data_ptr())
    n = C.c_int64()
    assert ae.lib.model_qr_workspace(48, 5, C.byref(n)) == -1
    assert ae.lib.model_qr_workspace(64, 17, C.byref(n)) == -1
    assert ae.lib.model_qr_workspace(64, 5, C.byref(n)) == 0 and n.value == 26 * 64 * 64 * 4 + 1024
    assert ae.lib.model_qr_compose(p, p, p, p, 64, 0, -1, p, p, None) == -1
    assert ae.lib.model_qr_compose(None, p, p, p, 64, 0, 5, p, p, None) == -1
    assert ae.lib.model_qr_backward(p, p, p, p, 64, 9, 5, p, p, p, p, None) == -1


# ------------------------------------------------------------------ many small matrices in one launch (the per-block transformations)
def _small_sets(count, d, seed, kind="random"):
    sets = [wl.make_lu_params(d, seed=seed + 31 * m, kind=kind, noise=1e-3 if kind == "bd_hadamard" else 0.0,
                              block=min(32, d)) for m in range(count)]
    return sets, [np.stack([s[i] for s in sets]) for i in range(5)]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("count,d,kind", [(1, 128, "random"), (33, 128, "bd_hadamard"), (5, 64, "random"), (7, 96, "random"),
                                          (3, 20, "random"), (4, 1, "random"), (300, 32, "bd_hadamard")])
def test_small_batch_matches_oracle_matrix_by_matrix(ae, count, d, kind, dtype):
    """model_lu_{compose,backward,inverse}_batch against the oracle applied to each parameter set on its own
    (and numpy's inverse of the oracle's A); sizes below, at and not a divisor of the 128 x 128 LDS tile."""
    import torch
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    sets, stacked = _small_sets(count, d, seed=1000 + count + d, kind=kind)
    dev = [torch.from_numpy(np.ascontiguousarray(a)).cuda() for a in stacked]
    rng = np.random.default_rng(count * 131 + d)
    g = _round(rng.standard_normal((count, d, d)), dtype).astype(np.float64)
    gt = torch.from_numpy(g.astype(np.float32)).cuda().to(td).contiguous()
    a = torch.full((count, d, d), float("nan"), dtype=td, device="cuda")
    ainv = torch.full((count, d, d), float("nan"), dtype=td, device="cuda")
    dlp = torch.full((count, d, d), float("nan"), device="cuda")
    dup = torch.full((count, d, d), float("nan"), device="cuda")
    dls = torch.full((count, d), float("nan"), device="cuda")
    ae.model_lu_compose_batch(*dev, count, d, a)
    ae.model_lu_backward_batch(gt, *dev, count, d, dlp, dup, dls)
    ae.model_lu_inverse_batch(*dev, count, d, ainv)
    torch.cuda.synchronize()
    a, ainv = a.float().cpu().numpy().astype(np.float64), ainv.float().cpu().numpy().astype(np.float64)
    dlp, dup, dls = [t.cpu().numpy().astype(np.float64) for t in (dlp, dup, dls)]
    for m, p in enumerate(sets):
        a_ref = ao.lu_compose(*p)
        assert _close(a[m], a_ref, TOL[dtype]), (m, np.abs(a[m] - a_ref).max())
        r_lp, r_up, r_ls = ao.lu_gradients(g[m], *p)
        assert _close(dlp[m], r_lp, TOL["f32"]) and _close(dup[m], r_up, TOL["f32"]) and _close(dls[m], r_ls, TOL["f32"]), m
        assert np.all(np.triu(dlp[m]) == 0.0) and np.all(np.tril(dup[m]) == 0.0)
        assert _close(ainv[m], np.linalg.inv(a_ref), TOL[dtype]), (m, np.abs(ainv[m] - np.linalg.inv(a_ref)).max())


def test_small_batch_agrees_with_the_full_size_calls(ae):
    """d = 128 is served by both paths: same A and A^-1 to binary32 rounding."""
    d, count = 128, 3
    sets, stacked = _small_sets(count, d, seed=77)
    import torch
    dev = [torch.from_numpy(np.ascontiguousarray(a)).cuda() for a in stacked]
    a = torch.empty((count, d, d), device="cuda")
    ainv = torch.empty((count, d, d), device="cuda")
    ae.model_lu_compose_batch(*dev, count, d, a)
    ae.model_lu_inverse_batch(*dev, count, d, ainv)
    torch.cuda.synchronize()
    for m, p in enumerate(sets):
        assert _close(a[m].cpu().numpy().astype(np.float64), _compose(ae, p, d, "f32"), 1e-5)
        assert _close(ainv[m].cpu().numpy().astype(np.float64), _inverse(ae, p, d, "f32"), 1e-4)


def test_small_batch_argument_checks(ae):
    import torch
    t = torch.zeros(128 * 128, device="cuda")
    p = C.c_void_p(t.data_ptr())
    assert ae.lib.model_lu_compose_batch(p, p, p, p, p, 1, 129, 0, p, None) == -1 and "1 .. 128" in ae.model_last_error()
    assert ae.lib.model_lu_compose_batch(p, p, p, p, p, 0, 64, 0, p, None) == -1
    assert ae.lib.model_lu_compose_batch(p, p, p, p, p, 1, 64, 2, p, None) == -1
    assert ae.lib.model_lu_compose_batch(None, p, p, p, p, 1, 64, 0, p, None) == -1
    assert ae.lib.model_lu_backward_batch(p, p, p, p, p, p, 1, 0, 0, p, p, p, None) == -1
    assert ae.lib.model_lu_inverse_batch(p, p, p, p, None, 1, 64, 0, p, None) == -1


def test_index_vector_that_is_not_a_permutation_stays_inside_the_arrays(ae):
    """perm is not trusted: an entry outside 0..d-1 is treated as its own position (every kernel that indexes with it
    checks the range), so A is still defined row by row; the gradient and inverse calls must complete with finite
    results (which rows they produce is unspecified for such input)."""
    import torch
    d = 128
    lp, up, ls, sg, perm = wl.make_lu_params(d, seed=41)
    bad = perm.copy()
    bad[[3, 50, 127]] = [-1, d, 1 << 30]
    fixed = bad.copy()
    fixed[[3, 50, 127]] = [3, 50, 127]
    ref = ao.lu_compose(lp, up, ls, sg, fixed)
    assert _close(_compose(ae, (lp, up, ls, sg, bad), d, "f32"), ref, TOL["f32"])
    dev = [torch.from_numpy(np.ascontiguousarray(a[None])).cuda() for a in (lp, up, ls, sg, bad)]
    a = torch.full((1, d, d), float("nan"), device="cuda")
    ae.model_lu_compose_batch(*dev, 1, d, a)
    assert _close(a[0].cpu().numpy().astype(np.float64), ref, TOL["f32"])
    g = np.random.default_rng(3).standard_normal((d, d))
    for out in _backward(ae, g, (lp, up, ls, sg, bad), d, "f32") + [_inverse(ae, (lp, up, ls, sg, bad), d, "f32")]:
        assert np.all(np.isfinite(out))
    gt = torch.from_numpy(g.astype(np.float32)[None]).cuda()
    dlp, dup, dls = torch.empty((1, d, d), device="cuda"), torch.empty((1, d, d), device="cuda"), torch.empty((1, d), device="cuda")
    ainv = torch.empty((1, d, d), device="cuda")
    ae.model_lu_backward_batch(gt, *dev, 1, d, dlp, dup, dls)
    ae.model_lu_inverse_batch(*dev, 1, d, ainv)
    torch.cuda.synchronize()
    for t in (dlp, dup, dls, ainv):
        assert bool(torch.isfinite(t).all())
