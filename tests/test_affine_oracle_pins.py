"""Pins of oracle/affine_oracle.py (LU parametrisation, Eq. 4; volume regulariser, Eq. 6) against what the paper and
the mathematics fix: a 2 x 2 case by hand, |det A| = prod |s_i|, triangular structure, finite differences of a scalar
loss, the regulariser's zero set, and the block-orthogonal initialisation."""
import numpy as np

import workloads as wl
from oracle import affine_oracle as ao


def _params(d, seed, **kw):
    lp, up, ls, sg, perm = wl.make_lu_params(d, seed, **kw)
    return [a.astype(np.float64) for a in (lp, up, ls, sg)] + [perm]


def test_two_by_two_by_hand():
    # L = [[1,0],[3,1]], U + diag s = [[2,5],[0,-4]], P swaps the rows:  L(U+D) = [[2,5],[6,11]]  ->  A = [[6,11],[2,5]]
    lp = np.array([[9.0, 9.0], [3.0, 9.0]])            # entries on and above the diagonal are ignored
    up = np.array([[9.0, 5.0], [9.0, 9.0]])            # entries on and below the diagonal are ignored
    a = ao.lu_compose(lp, up, np.log([2.0, 4.0]), [1.0, -1.0], [1, 0])
    assert np.allclose(a, [[6.0, 11.0], [2.0, 5.0]], rtol=1e-15)
    # a cyclic permutation tells P from its inverse: (P M)[i] = M[perm[i]], so row 0 of A is row 2 of L(U+D)
    lp = np.array([[0.0, 0, 0], [2.0, 0, 0], [0.0, 3.0, 0]])
    up = np.array([[0.0, 1.0, 0], [0, 0, 1.0], [0, 0, 0]])                # L(U+I) = [[1,1,0],[2,3,1],[0,3,4]]
    a = ao.lu_compose(lp, up, np.zeros(3), np.ones(3), [2, 0, 1])
    assert np.array_equal(a, [[0.0, 3.0, 4.0], [1.0, 1.0, 0.0], [2.0, 3.0, 1.0]])


def test_determinant_is_the_product_of_the_diagonal_vector():
    lp, up, ls, sg, perm = _params(48, 1)
    a = ao.lu_compose(lp, up, ls, sg, perm)
    sign, logdet = np.linalg.slogdet(a)
    assert np.isclose(logdet, ls.sum(), rtol=1e-10, atol=1e-10)          # |det A| = prod |s_i|
    # the sign: that of the permutation times the signs of s
    inv = sum(1 for i in range(48) for j in range(i) if perm[j] > perm[i])
    assert sign == (-1.0) ** inv * np.prod(sg)


def test_factors_have_the_stated_structure_and_identity_parameters_give_the_permutation():
    lp, up, ls, sg, perm = _params(16, 2)
    L, UD, s = ao.lu_factors(lp, up, ls, sg)
    assert np.array_equal(np.diag(L), np.ones(16)) and np.array_equal(np.triu(L, 1), np.zeros((16, 16)))
    assert np.array_equal(np.tril(UD, -1), np.zeros((16, 16))) and np.allclose(np.diag(UD), s)
    a = ao.lu_compose(np.zeros((16, 16)), np.zeros((16, 16)), np.zeros(16), np.ones(16), perm)
    assert np.array_equal(a, np.eye(16)[perm])
    # undoing the permutation and factorising again without pivoting gives the factors back
    a = ao.lu_compose(lp, up, ls, sg, perm)
    b = np.empty_like(a)
    b[perm] = a
    assert np.allclose(b, L @ UD, rtol=1e-13)


def test_gradients_against_finite_differences():
    d = 6
    lp, up, ls, sg, perm = _params(d, 3)
    rng = np.random.default_rng(0)
    c = rng.standard_normal((d, d))
    loss = lambda lp_, up_, ls_: float(np.sum(c * np.tanh(ao.lu_compose(lp_, up_, ls_, sg, perm))))
    a = ao.lu_compose(lp, up, ls, sg, perm)
    g = c * (1.0 - np.tanh(a) ** 2)                                       # d loss / d A
    dl, du, dls = ao.lu_gradients(g, lp, up, ls, sg, perm)
    h = 1e-6
    for i in range(d):
        for j in range(d):
            e = np.zeros((d, d)); e[i, j] = h
            num_l = (loss(lp + e, up, ls) - loss(lp - e, up, ls)) / (2 * h)
            num_u = (loss(lp, up + e, ls) - loss(lp, up - e, ls)) / (2 * h)
            assert abs(num_l - dl[i, j]) < 1e-7 and abs(num_u - du[i, j]) < 1e-7      # zero outside the used triangles
        e = np.zeros(d); e[i] = h
        num_s = (loss(lp, up, ls + e) - loss(lp, up, ls - e)) / (2 * h)
        assert abs(num_s - dls[i]) < 1e-7
    assert np.array_equal(np.triu(dl), np.zeros((d, d))) and np.array_equal(np.tril(du), np.zeros((d, d)))


def test_volume_regulariser_and_its_log_form_share_their_minima():
    rng = np.random.default_rng(4)
    ls = rng.standard_normal(32) * 0.2
    s = np.exp(ls) * rng.choice([-1.0, 1.0], size=32)
    val, grad = ao.vol_penalty(ls)
    assert np.isclose(ao.vol_loss(s), (np.exp(ls.sum()) - 1.0) ** 2, rtol=1e-12)     # Eq. 6 through log|s|
    assert np.isclose(val, ls.sum() ** 2) and np.allclose(grad, 2.0 * ls.sum())
    ls0 = ls - ls.mean()                                                              # sum log|s| = 0: |det A| = 1
    assert ao.vol_penalty(ls0)[0] < 1e-28 and ao.vol_loss(np.exp(ls0)) < 1e-28
    assert ao.vol_loss(np.ones(8)) == 0.0 and ao.vol_penalty(np.zeros(8))[0] == 0.0
    assert (ao.vol_loss(s) > 0) == (val > 0)
    h = 1e-6
    e = np.zeros(32); e[5] = h
    assert abs((ao.vol_penalty(ls + e)[0] - ao.vol_penalty(ls - e)[0]) / (2 * h) - grad[5]) < 1e-8


def test_initialisation_is_block_diagonal_hadamard_and_noise_stays_small():
    d, b = 128, 32
    lp, up, ls, sg, perm = _params(d, 5, kind="bd_hadamard")
    a = ao.lu_compose(lp, up, ls, sg, perm)
    assert np.allclose(a @ a.T, np.eye(d), atol=1e-6)                                 # orthogonal (float32 parameters)
    off = np.kron(np.eye(d // b), np.ones((b, b))) == 0
    assert np.abs(a[off]).max() < 1e-6 and np.allclose(np.abs(a[~off]), 1.0 / np.sqrt(b), atol=1e-6)
    assert abs(ls.sum()) < 1e-5 and ao.vol_penalty(ls)[0] < 1e-9                      # volume preserving at the start
    lp2, up2, ls2, sg2, perm2 = _params(d, 5, kind="bd_hadamard", noise=1e-3)
    a2 = ao.lu_compose(lp2, up2, ls2, sg2, perm2)
    assert np.array_equal(perm, perm2) and np.array_equal(ls, ls2)
    assert 0 < np.abs(a2 - a).max() < 0.05 and np.allclose(a2[~off], a[~off], atol=2e-3)


# ------------------------------------------------------------------ QR parametrisation (Eq. 5)
def _qr_params(d, seed, **kw):
    return [a.astype(np.float64) for a in wl.make_qr_params(d, seed, **kw)]


def test_qr_two_by_two_is_a_plane_rotation():
    th = 0.7
    g = np.array([[5.0, 2 * th], [0.0, -3.0]])               # the symmetric part of G does not matter: S = [[0, th], [-th, 0]]
    a = ao.qr_compose(g, np.array([[9.0, 0.5], [9.0, 9.0]]), np.log([2.0, 3.0]), [1.0, -1.0])
    q = np.array([[np.cos(th), np.sin(th)], [-np.sin(th), np.cos(th)]])
    assert np.allclose(a, q @ np.array([[2.0, 0.5], [0.0, -3.0]]), rtol=1e-13)


def test_qr_factor_is_a_rotation_and_the_determinant_is_the_product_of_s():
    g, rp, ls, sg = _qr_params(40, 1)
    Q, RD, s = ao.qr_factors(g, rp, ls, sg)
    assert np.allclose(Q.T @ Q, np.eye(40), atol=1e-12) and np.isclose(np.linalg.det(Q), 1.0)
    assert np.array_equal(np.tril(RD, -1), np.zeros((40, 40))) and np.allclose(np.diag(RD), s)
    sign, logdet = np.linalg.slogdet(ao.qr_compose(g, rp, ls, sg))
    assert np.isclose(logdet, ls.sum(), atol=1e-10) and sign == np.prod(sg)
    sym = g + g.T                                             # a symmetric G gives Q = I: A is upper triangular
    assert np.allclose(ao.qr_compose(sym, rp, ls, sg), RD, atol=1e-13)


def test_qr_gradients_against_finite_differences():
    d = 5
    g, rp, ls, sg = _qr_params(d, 2)
    g *= 3.0                                                  # a rotation well away from the identity
    c = np.random.default_rng(0).standard_normal((d, d))
    loss = lambda g_, rp_, ls_: float(np.sum(c * np.tanh(ao.qr_compose(g_, rp_, ls_, sg))))
    a = ao.qr_compose(g, rp, ls, sg)
    dg, dr, dls = ao.qr_gradients(c * (1.0 - np.tanh(a) ** 2), g, rp, ls, sg)
    h = 1e-6
    for i in range(d):
        for j in range(d):
            e = np.zeros((d, d)); e[i, j] = h
            assert abs((loss(g + e, rp, ls) - loss(g - e, rp, ls)) / (2 * h) - dg[i, j]) < 1e-7
            assert abs((loss(g, rp + e, ls) - loss(g, rp - e, ls)) / (2 * h) - dr[i, j]) < 1e-7
        e = np.zeros(d); e[i] = h
        assert abs((loss(g, rp, ls + e) - loss(g, rp, ls - e)) / (2 * h) - dls[i]) < 1e-7
    assert np.allclose(dg, -dg.T) and np.array_equal(np.tril(dr), np.zeros((d, d)))     # only the skew part of G acts


def test_qr_initialisation_is_block_diagonal_orthogonal():
    d, b = 96, 32
    g, rp, ls, sg = _qr_params(d, 3, kind="bd_orthogonal")
    a = ao.qr_compose(g, rp, ls, sg)
    off = np.kron(np.eye(d // b), np.ones((b, b))) == 0
    assert np.allclose(a @ a.T, np.eye(d), atol=1e-5) and np.abs(a[off]).max() < 1e-6
    assert np.abs(a[~off]).max() > 0.2 and ao.vol_penalty(ls)[0] == 0.0
    g2, rp2, _, _ = _qr_params(d, 3, kind="bd_orthogonal", noise=1e-3)
    a2 = ao.qr_compose(g2, rp2, ls, sg)
    assert 0 < np.abs(a2 - a).max() < 0.05
