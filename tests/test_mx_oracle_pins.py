"""Pins of the MX block-quantiser oracle (oracle/mx_oracle.py) against what the paper and the
arithmetic fix: the paper's worked example, the format's value set, invariants of Eq. (1), the
error bound of a round-to-nearest quantiser, and an independent nearest-value search."""
import itertools
import os

import numpy as np
import pytest

import oracle.mx_oracle as mx

HERE = os.path.dirname(os.path.abspath(__file__))
GRID = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]      # FP4 E2M1 magnitudes (OCP microscaling formats)


def _golden():
    rows = {}
    for line in open(os.path.join(HERE, "golden", "mx_hadamard_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        rows[k] = np.array([float(t) for t in v])
    return rows


def test_paper_example_rotation_and_block_errors():
    """The rotated vector the paper prints, and its claim about the two blocks' errors (B = 2)."""
    g = _golden()
    x, hx = g["x"], g["H4x"]
    h4 = 0.5 * np.array([[1, 1, 1, 1], [1, -1, 1, -1], [1, 1, -1, -1], [1, -1, -1, 1]], dtype=np.float64)
    assert np.array_equal(h4 @ x, hx)                       # the printed rotation
    assert np.allclose(h4 @ h4.T, np.eye(4))
    err = lambda v: ((v - mx.mx_quantize(v[None, :], block=2)[0]) ** 2).reshape(2, 2).sum(axis=1)
    e_x, e_hx = err(x), err(hx)
    assert e_hx[0] < e_x[0] and e_hx[1] > e_x[1]            # "reduces the first block's error, increases the second's"
    # and the values by hand: [10, 1]: floor(log2 10) = 3, s = 2, 10/2 = 5 ties between 4 and 6 -> 4 (even) -> 8;
    # [0.5, 0.5]: s = 2^-3, 0.5/s = 4 exactly; [6, 4.5]: s = 1 -> [6, 4]; [5, 4.5]: s = 1 -> [4, 4]
    assert np.array_equal(mx.mx_quantize(x[None, :], block=2)[0], [8.0, 1.0, 0.5, 0.5])
    assert np.array_equal(mx.mx_quantize(hx[None, :], block=2)[0], [6.0, 4.0, 4.0, 4.0])


def test_scale_is_the_power_of_two_of_eq1():
    for amax, want in ((1.0, 2.0 ** -2), (1.999, 2.0 ** -2), (2.0, 2.0 ** -1), (6.0, 1.0), (7.99, 1.0), (8.0, 2.0),
                       (0.75, 2.0 ** -3), (3e-5, 2.0 ** (-16 - 2))):
        x = np.zeros((1, 32))
        x[0, 7] = -amax
        assert mx.block_scales(x)[0, 0] == want, amax
        # the scaled maximum lies in [4, 8): the top binade of the format, or clipped
        assert 4.0 <= amax / want < 8.0


def test_values_on_the_scaled_grid_are_fixed_points():
    rng = np.random.default_rng(1)
    for k in (-20, -3, 0, 5, 40):
        s = 2.0 ** k
        x = s * rng.choice(GRID, size=(64, 32)) * rng.choice([-1.0, 1.0], size=(64, 32))
        x[:, 0] = 6.0 * s * rng.choice([-1.0, 1.0], size=64)            # block maximum 6 s: scale exactly s
        assert np.array_equal(mx.mx_quantize(x), x)
    assert sorted(set(np.abs(mx.quantize_element_e2m1(np.linspace(-8, 8, 100001))))) == GRID


def test_idempotent_odd_and_scale_equivariant():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((128, 256)) * np.exp(rng.standard_normal((128, 256)))   # heavy tails
    q = mx.mx_quantize(x)
    assert np.array_equal(mx.mx_quantize(q), q)                                      # Q(Q(x)) = Q(x)
    assert np.array_equal(mx.mx_quantize(-x), -q)                                    # odd
    for k in (-30, -1, 7, 60):
        assert np.array_equal(mx.mx_quantize(x * 2.0 ** k), q * 2.0 ** k)            # powers of two pass through
    assert np.array_equal(mx.mx_quantize(np.zeros((3, 64))), np.zeros((3, 64)))      # all-zero blocks
    # blocks do not see each other: permuting whole blocks permutes the result
    perm = rng.permutation(8)
    xb = x.reshape(128, 8, 32)
    assert np.array_equal(mx.mx_quantize(xb[:, perm].reshape(128, 256)).reshape(128, 8, 32), q.reshape(128, 8, 32)[:, perm])


def test_error_bound_of_round_to_nearest():
    """|x - Q(x)| <= s * (half the grid step at that magnitude); only scaled values in (6, 8) clip, by < 2 s."""
    rng = np.random.default_rng(3)
    x = rng.standard_normal((256, 128)) * np.exp(2 * rng.standard_normal((256, 128)))
    q = mx.mx_quantize(x)
    s = np.repeat(mx.block_scales(x), 32, axis=1)
    a = np.abs(x) / s
    half_step = np.where(a < 2.0, 0.25, np.where(a < 4.0, 0.5, 1.0))
    bound = np.where(a <= 6.0, half_step, a - 6.0)
    assert np.all(np.abs(x - q) / s <= bound + 1e-12)
    assert np.all(a < 8.0) and np.all(np.abs(x - q) / s < 2.0)
    assert np.all(np.sign(q) * np.sign(x) >= 0)
    # monotone: sorting a block's scaled values sorts their quantised values
    y = np.sort(rng.uniform(-8, 8, 20001))
    assert np.all(np.diff(mx.quantize_element_e2m1(y)) >= 0)


def test_ties_go_to_the_even_code():
    ties = {0.25: 0.0, 0.75: 1.0, 1.25: 1.0, 1.75: 2.0, 2.5: 2.0, 3.5: 4.0, 5.0: 4.0}
    for y, want in ties.items():
        assert mx.quantize_element_e2m1(np.array([y]))[0] == want
        assert mx.quantize_element_e2m1(np.array([-y]))[0] == -want
    assert mx.quantize_element_e2m1(np.array([6.0001, 7.9, 100.0])).tolist() == [6.0, 6.0, 6.0]


def test_against_exhaustive_search_on_tiny_inputs():
    """Independent of the oracle's code: for blocks of two elements on a coarse lattice, the result is the
    nearest element of {+-s*g} with s recomputed from log2 by hand, ties resolved by the even-code rule."""
    vals = [0.0, 0.3, 0.5, 0.8, 1.0, 1.3, 2.2, 2.5, 3.1, 4.9, 5.0, 5.1, 7.0, 9.0, 12.0]
    for a, b in itertools.product(vals, repeat=2):
        for sa, sb in ((1, 1), (-1, 1)):
            x = np.array([[sa * a, sb * b]])
            q = mx.mx_quantize(x, block=2)[0]
            m = max(a, b)
            if m == 0.0:
                assert np.array_equal(q, [0.0, 0.0])
                continue
            s = 2.0 ** (int(np.floor(np.log2(m))) - 2)
            for xv, qv in zip(x[0], q):
                cands = sorted((abs(abs(xv) - s * g), i % 2, s * g) for i, g in enumerate(GRID))   # distance, then even code first
                assert abs(qv) == cands[0][2], (a, b, xv, qv)


def test_scale_exponent_clamps_to_e8m0():
    x = np.zeros((1, 32))
    x[0, 0] = 2.0 ** -140                                    # floor(log2) - 2 = -142 < -127
    assert mx.block_scales(x)[0, 0] == 2.0 ** -127
    assert mx.mx_quantize(x)[0, 0] == 0.0                    # 2^-140 / 2^-127 = 2^-13 rounds to zero
    x[0, 0] = 3.0e38                                         # floor(log2) = 127 -> exponent 125: inside the range
    assert mx.block_scales(x)[0, 0] == 2.0 ** 125


# ------------------------------------------------------------------ transformation mean squared error (Eq. 2)
def _hadamard(n):
    h = np.array([[1.0]])
    while h.shape[0] < n:
        h = np.block([[h, h], [h, -h]])
    return h / np.sqrt(n)


def test_transform_mse_identity_is_plain_quantisation_error():
    x = np.random.default_rng(5).standard_normal((64, 128)) * 3.0
    e, eb, yq = mx.transform_mse(x, np.eye(128), np.zeros(128), np.eye(128))
    q = mx.mx_quantize(x)
    assert np.array_equal(yq, q)
    assert np.isclose(e, ((x - q) ** 2).mean(), rtol=1e-14)
    assert np.allclose(eb, ((x - q) ** 2).reshape(64, 4, 32).mean(axis=(0, 2)), rtol=1e-14)
    assert np.isclose(eb.mean(), e, rtol=1e-14)                       # E is the average of the block errors


def test_transform_mse_paper_example_blocks():
    """[10, 1, .5, .5] with H_4 and B = 2 (the paper's example): the first block's error falls, the second's rises."""
    x = np.array([[10.0, 1.0, 0.5, 0.5]])
    h4 = _hadamard(4)
    _, eb_id, _ = mx.transform_mse(x, np.eye(4), np.zeros(4), np.eye(4), block=2)
    _, eb_h, yq = mx.transform_mse(x, h4, np.zeros(4), h4.T, block=2)
    assert np.array_equal(yq, [[6.0, 4.0, 4.0, 4.0]])
    # in the ROTATED coordinates the paper's statement holds block by block ...
    y = x @ h4.T
    ey = ((y - yq) ** 2).reshape(2, 2).sum(axis=1)
    ex = ((x - mx.mx_quantize(x, 2)) ** 2).reshape(2, 2).sum(axis=1)
    assert ey[0] < ex[0] and ey[1] > ex[1]
    # ... and back in the original coordinates an orthogonal map keeps the total (by hand: 4 vs 0.25 + 1.25 = 1.5)
    assert np.isclose(eb_id.sum() * 2, 4.0) and np.isclose(eb_h.sum() * 2, 1.5)


def test_transform_mse_orthogonal_map_preserves_the_error_norm_and_the_bound_holds():
    rng = np.random.default_rng(6)
    d = 64
    x = rng.standard_normal((256, d)) * np.exp(rng.standard_normal(d))
    h = _hadamard(d)
    e, _, yq = mx.transform_mse(x, h, np.zeros(d), h.T)
    y = x @ h.T
    assert np.isclose(e, ((y - yq) ** 2).mean(), rtol=1e-12)           # ||A^-1 r|| = ||r|| for orthogonal A
    # general invertible A and a shift: x - T^-1(Q(T x)) = A^-1 (T x - Q(T x))  (first step of the bound's proof) ...
    A = rng.standard_normal((d, d)) + 4.0 * np.eye(d)
    v = rng.standard_normal(d)
    Ainv = np.linalg.inv(A)
    e, eb, yq = mx.transform_mse(x, A, v, Ainv)
    y = x @ A.T + v
    resid = (y - yq) @ Ainv.T
    assert np.isclose(e, (resid ** 2).mean(), rtol=1e-9)
    # ... hence E(T) <= ||A^-1||_sigma^2 / d * E||y - Q(y)||^2
    assert e <= np.linalg.norm(Ainv, 2) ** 2 * ((y - yq) ** 2).mean() * (1 + 1e-12)
    assert np.isclose(eb.mean(), e, rtol=1e-12)
    # a shift that centres the transformed tokens changes nothing in the algebra: T^-1 undoes it
    e0, _, _ = mx.transform_mse(x, np.eye(d), v, np.eye(d))
    assert np.isclose(e0, (((x + v) - mx.mx_quantize(x + v)) ** 2).mean(), rtol=1e-12)


def test_transform_mse_power_of_two_gain_is_free():
    """Q commutes with powers of two, so T = 2^k A has the error of A exactly."""
    rng = np.random.default_rng(7)
    d = 64
    x = rng.standard_normal((128, d))
    A = rng.standard_normal((d, d)) + 3.0 * np.eye(d)
    Ainv = np.linalg.inv(A)
    v = rng.standard_normal(d)
    e1, eb1, _ = mx.transform_mse(x, A, v, Ainv)
    e2, eb2, _ = mx.transform_mse(x, 8.0 * A, 8.0 * v, Ainv / 8.0)
    assert np.isclose(e1, e2, rtol=1e-12) and np.allclose(eb1, eb2, rtol=1e-12)


# ------------------------------------------------------------------ other element formats
def test_fp8_e4m3_grid_is_the_ocp_format():
    g = mx.E4M3_GRID
    assert g.size == 127 and g[0] == 0.0 and np.all(np.diff(g) > 0)
    assert g[1] == 2.0 ** -9 and g[8] == 2.0 ** -6 and g[-1] == 448.0          # smallest subnormal, smallest normal, largest
    assert g[7] == 7 * 2.0 ** -9 and g[9] - g[8] == 2.0 ** -9                   # the subnormal spacing continues into the first binade
    assert np.all(np.diff(g)[8:] == 2.0 ** (np.floor(np.log2(g[8:-1])) - 3))    # eight steps per binade
    assert mx.FORMATS["fp8"][1] == 8 and 2.0 ** 8 <= g[-1] < 2.0 ** 9           # r_max: the largest binade


@pytest.mark.parametrize("fmt", ["fp8", "int4"])
def test_other_formats_fixed_points_idempotence_and_error_bound(fmt):
    grid, r_max = mx.FORMATS[fmt]
    rng = np.random.default_rng(11)
    # every grid value times a power of two, with the block maximum in the largest binade, is a fixed point
    blk = np.concatenate([[2.0 ** r_max], rng.choice(grid[grid < 2.0 ** (r_max + 1)], size=31) * rng.choice([-1.0, 1.0], size=31)])
    for k in (-3, 0, 5):
        x = (blk * 2.0 ** k)[None, :]
        assert np.array_equal(mx.mx_quantize(x, 32, fmt), x)
    x = rng.standard_normal((64, 64)) * np.exp(rng.standard_normal((64, 1)))
    q = mx.mx_quantize(x, 32, fmt)
    assert np.array_equal(mx.mx_quantize(q, 32, fmt), q)                        # idempotent
    assert np.array_equal(mx.mx_quantize(-x, 32, fmt), -q)                      # odd
    assert np.array_equal(mx.mx_quantize(8.0 * x, 32, fmt), 8.0 * q)            # commutes with powers of two
    # round to nearest: the error is at most half the local spacing, except where the largest binade clips
    s = np.repeat(mx.block_scales(x, 32) * 2.0 ** (mx.E2M1_RMAX - r_max), 32, axis=1)    # block_scales uses FP4's r_max
    y = np.abs(x) / s
    top = grid[-1]
    inside = y <= top
    idx = np.searchsorted(grid, y[inside], side="right") - 1
    gap = np.where(idx + 1 < grid.size, grid[np.minimum(idx + 1, grid.size - 1)] - grid[idx], 0.0)
    assert np.all(np.abs(np.abs(q[inside]) / s[inside] - y[inside]) <= gap / 2 + 1e-15)
    assert np.all(np.abs(q[~inside]) / s[~inside] == top)


def test_other_formats_against_exhaustive_search_and_ties():
    for fmt in ("fp8", "int4"):
        grid, r_max = mx.FORMATS[fmt]
        top = 2.0 ** r_max
        ys = np.linspace(-1.2 * grid[-1], 1.2 * grid[-1], 4001)
        for y in ys[::7]:
            x = np.array([[top * 1.0, y if abs(y) < 2 * top else 0.0]])          # block of two, maximum in the largest binade: s = 1
            q = mx.mx_quantize(x, 2, fmt)[0, 1]
            want = min(grid, key=lambda g: (abs(abs(x[0, 1]) - g), 0))           # nearest magnitude (ties checked below)
            assert abs(abs(q) - abs(x[0, 1])) <= abs(want - abs(x[0, 1])) + 1e-15
        mids = (grid[:-1] + grid[1:]) / 2                                         # every tie goes to the even code
        for i, m in enumerate(mids):
            got = mx.quantize_element(np.array([m]), fmt)[0]
            assert got == (grid[i] if i % 2 == 0 else grid[i + 1])
