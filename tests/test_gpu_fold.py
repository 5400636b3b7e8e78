"""GPU parity of the folding entry points (model_fold_linear / model_fold_embedding) against oracle/fold_oracle.py,
element by element, through the C boundary."""
import ctypes as C

import numpy as np
import pytest

import workloads as wl
from oracle import fold_oracle as fo

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}      # of the entry plus the same fraction of the result's root mean square


@pytest.fixture(scope="module")
def ae():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2602_17681_amd import binding
    return binding


def _close(got, ref, tol):
    rms = float(np.sqrt(np.mean(ref ** 2))) + 1e-30
    return float((np.abs(got - ref) - tol * np.abs(ref)).max()) <= tol * rms


def _rt(a, dtype):
    """The value as stored (float64 of the bf16 / fp32 rounding)."""
    a = np.asarray(a, dtype=np.float32)
    return (wl.round_to_bf16(a) if dtype == "bf16" else a).astype(np.float64)


def _side(n, seed, dtype):
    """A well-conditioned n x n matrix, its inverse (of the stored matrix, then stored) and a shift."""
    a, v, ainv = wl.make_transform(n, seed=seed, bf16=(dtype == "bf16"), kind="affine")
    return a.astype(np.float64), ainv.astype(np.float64), v.astype(np.float64)


def _fold(ae, W, b, a_left, v_left, a_right_inv, v_right, dtype):
    import torch
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    out, inn = W.shape
    dev = lambda a, t=td: None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda().to(t).contiguous()
    f32 = torch.float32
    w_out = torch.full((out, inn), float("nan"), dtype=td, device="cuda")
    b_out = torch.full((out,), float("nan"), device="cuda")
    p = 0 if a_left is None else a_left.shape[0]
    q = 0 if a_right_inv is None else a_right_inv.shape[0]
    ws = torch.empty(ae.model_fold_workspace(out, inn, p, q, ae.DTYPES[dtype]), dtype=torch.uint8, device="cuda")
    ae.model_fold_linear(dev(W), dev(b, f32), out, inn, dev(a_left), dev(v_left, f32), dev(a_right_inv), dev(v_right, f32),
                         w_out, b_out, ws)
    torch.cuda.synchronize()
    return w_out.float().cpu().numpy().astype(np.float64), b_out.cpu().numpy().astype(np.float64)


# (out, in, p, q): 0 = that side absent; shapes of K/Q (right only), FFN out (left only), V (both, shared head matrix on
# the left), O (left full, shared head matrix on the right); sizes that are and are not multiples of the 64-wide tiles
CASES = [(96, 160, 0, 160), (160, 96, 160, 0), (128, 256, 32, 256), (256, 128, 256, 32), (224, 352, 32, 32), (512, 1024, 128, 1024)]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("out,inn,p,q", CASES)
def test_fold_linear_matches_oracle(ae, out, inn, p, q, dtype):
    rng = np.random.default_rng(out + inn)
    W = _rt(rng.standard_normal((out, inn)) / np.sqrt(inn), dtype)
    b = rng.standard_normal(out).astype(np.float32).astype(np.float64)
    al, _, vl = _side(p, 1, dtype) if p else (None, None, None)
    _, arinv, vr = _side(q, 2, dtype) if q else (None, None, None)
    if out == 256:
        vl = None                                           # the output projection: the left matrix without a shift
    wt, bt = _fold(ae, W, b, al, vl, arinv, vr, dtype)
    r_w, r_b = fo.fold_linear(W, b, al, vl, arinv, vr)
    assert _close(wt, r_w, TOL[dtype]), np.abs(wt - r_w).max()
    assert _close(bt, r_b, TOL[dtype]), np.abs(bt - r_b).max()
    # what folding is for: the folded layer on transformed inputs gives the transformed output of the original layer
    x = rng.standard_normal((8, inn))
    xt = x if not q else (x.reshape(8, inn // q, q) @ np.linalg.inv(arinv).T + vr).reshape(8, inn)
    y = x @ W.T + b
    yt = y if not p else (y.reshape(8, out // p, p) @ al.T + (0.0 if vl is None else vl)).reshape(8, out)
    got = xt @ wt.T + bt
    assert _close(got, yt, 5 * TOL[dtype] if dtype == "bf16" else 2e-3), np.abs(got - yt).max()


def test_no_transformation_copies_the_layer(ae):
    W = _rt(np.random.default_rng(0).standard_normal((64, 96)), "bf16")
    wt, bt = _fold(ae, W, None, None, None, None, None, "bf16")
    assert np.array_equal(wt, W) and np.array_equal(bt, np.zeros(64))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_fold_embedding_matches_oracle(ae, dtype):
    import torch
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    vocab, d = 1000, 192
    rng = np.random.default_rng(5)
    E = _rt(rng.standard_normal((vocab, d)), dtype)
    a, _, v = _side(d, 3, dtype)
    dev = lambda x, t=td: torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda().to(t).contiguous()
    e_out = torch.full((vocab, d), float("nan"), dtype=td, device="cuda")
    ae.model_fold_embedding(dev(E), vocab, d, dev(a), dev(v, torch.float32), e_out)
    assert _close(e_out.float().cpu().numpy().astype(np.float64), fo.fold_embedding(E, a, v), TOL[dtype])
    ae.model_fold_embedding(dev(E), vocab, d, dev(a), None, e_out)
    assert _close(e_out.float().cpu().numpy().astype(np.float64), fo.fold_embedding(E, a, np.zeros(d)), TOL[dtype])


def test_argument_checks(ae):
    import torch
    t = torch.zeros(256 * 256, device="cuda")
    p = C.c_void_p(t.data_ptr())
    t2 = torch.zeros(256 * 256, device="cuda")
    o = C.c_void_p(t2.data_ptr())
    n = C.c_int64()
    assert ae.lib.model_fold_workspace(0, 64, 0, 0, 0, C.byref(n)) == -1
    assert ae.lib.model_fold_workspace(64, 64, 32, 64, 1, C.byref(n)) == 0 and n.value == (64 * 64 + 3 * 64 * 64) * 2 + 1024
    call = lambda out, inn, al, pp, vl, ar, qq, vr, wo=o: ae.lib.model_fold_linear(p, p, out, inn, al, pp, vl, ar, qq, vr, 0, wo, p, p, None)
    assert call(64, 64, p, 48, None, None, 0, None) == -1          # p does not divide out
    assert call(64, 64, p, 16, None, None, 0, None) == -1          # p below 32
    assert call(64, 64, None, 0, p, None, 0, None) == -1           # a shift without its matrix
    assert call(64, 64, None, 0, None, p, 24, None) == -1          # q not a multiple of 16
    assert call(64, 64, None, 0, None, None, 0, None, wo=p) == -1  # in place
    assert "w_out" in ae.model_last_error()
    assert ae.lib.model_fold_embedding(p, 16, 40, p, None, 0, o, None) == -1     # d not a multiple of 16


def test_full_size_values_projection(ae):
    """The values projection of an 8-billion-parameter-class model (1 024 x 4 096: eight key/value heads of 128) with the
    shared head transformation on the left and the residual-stream inverse on the right, bf16: the largest doubly
    folded layer of the launch configuration bench.py times."""
    out, inn, p, q = 1024, 4096, 128, 4096
    rng = np.random.default_rng(9)
    W = _rt(rng.standard_normal((out, inn)) / np.sqrt(inn), "bf16")
    b = rng.standard_normal(out).astype(np.float32).astype(np.float64)
    al, _, vl = _side(p, 1, "bf16")
    _, arinv, vr = _side(q, 2, "bf16")
    wt, bt = _fold(ae, W, b, al, vl, arinv, vr, "bf16")
    r_w, r_b = fo.fold_linear(W, b, al, vl, arinv, vr)
    assert _close(wt, r_w, TOL["bf16"]) and _close(bt, r_b, TOL["bf16"])
