"""Pins of oracle/fold_oracle.py: the folded layers compute exactly what the unfolded network with explicit
transformations computes (the paper's appendix on folding), on a small attention block written out in float64 —
including the cancellation of the value shift through the softmax (rows sum to one)."""
import numpy as np

from oracle import fold_oracle as fo


def _affine(rng, d):
    a = rng.standard_normal((d, d)) + 3.0 * np.eye(d)
    return a, np.linalg.inv(a), rng.standard_normal(d)


def test_input_side_fold_undoes_the_transformation():
    rng = np.random.default_rng(0)
    d, out = 12, 7
    a, ainv, v = _affine(rng, d)
    W, b = rng.standard_normal((out, d)), rng.standard_normal(out)
    Wt, bt = fo.fold_linear(W, b, a_right_inv=ainv, v_right=v)
    x = rng.standard_normal((5, d))
    xt = x @ a.T + v                                        # transformed activations
    assert np.allclose(xt @ Wt.T + bt, x @ W.T + b, rtol=1e-11, atol=1e-11)
    assert np.allclose(Wt, W @ ainv) and np.allclose(bt, b - W @ ainv @ v)       # the paper's W~, b~ of the K, Q, V layers


def test_output_side_fold_applies_the_matrix_only():
    rng = np.random.default_rng(1)
    d, inn = 10, 6
    a, _, _ = _affine(rng, d)
    W, b = rng.standard_normal((d, inn)), rng.standard_normal(d)
    Wt, bt = fo.fold_linear(W, b, a_left=a)
    x = rng.standard_normal((4, inn))
    assert np.allclose(x @ Wt.T + bt, (x @ W.T + b) @ a.T, rtol=1e-12)
    # on the residual path the shift is carried by the stream: T1(r) + A1 f(x) = T1(r + f(x))
    v = rng.standard_normal(d)
    r = rng.standard_normal((4, d))
    assert np.allclose((r @ a.T + v) + (x @ Wt.T + bt), (r + x @ W.T + b) @ a.T + v, rtol=1e-12)


def test_embedding_fold():
    rng = np.random.default_rng(2)
    a, _, v = _affine(rng, 8)
    E = rng.standard_normal((20, 8))
    Et = fo.fold_embedding(E, a, v)
    for j in (0, 7, 19):
        assert np.allclose(Et[j], a @ E[j] + v, rtol=1e-13)


def test_attention_block_with_both_transformations_is_unchanged():
    """Residual stream transformed by T1, value vectors of every head by one shared T2 (d_head x d_head): the folded
    block maps T1(x) to A1 * (attention output), so that the transformed residual stream stays T1 of the original."""
    rng = np.random.default_rng(3)
    d, heads, dh, nt = 16, 4, 4, 6
    a1, a1inv, v1 = _affine(rng, d)
    a2, a2inv, v2 = _affine(rng, dh)
    Wq, Wk, Wv, Wo = (rng.standard_normal((d, d)) / 4 for _ in range(4))
    bq, bk, bv, bo = (rng.standard_normal(d) for _ in range(4))
    x = rng.standard_normal((nt, d))

    def attention(q, k, v_):
        outs = []
        for h in range(heads):
            s = slice(h * dh, (h + 1) * dh)
            logits = q[:, s] @ k[:, s].T / np.sqrt(dh)
            p = np.exp(logits - logits.max(axis=1, keepdims=True))
            p /= p.sum(axis=1, keepdims=True)
            outs.append(p @ v_[:, s])
        return np.concatenate(outs, axis=1)

    y_ref = attention(x @ Wq.T + bq, x @ Wk.T + bk, x @ Wv.T + bv) @ Wo.T + bo
    # folded layers
    fq = fo.fold_linear(Wq, bq, a_right_inv=a1inv, v_right=v1)
    fk = fo.fold_linear(Wk, bk, a_right_inv=a1inv, v_right=v1)
    fv = fo.fold_linear(Wv, bv, a_left=a2, v_left=v2, a_right_inv=a1inv, v_right=v1)      # T2 after, T1^-1 before
    fo_ = fo.fold_linear(Wo, bo, a_left=a1, a_right_inv=a2inv, v_right=v2)                # A1 after, T2^-1 before
    xt = x @ a1.T + v1
    vt = xt @ fv[0].T + fv[1]
    # the folded values ARE the transformed values, head by head
    vals = x @ Wv.T + bv
    for h in range(heads):
        s = slice(h * dh, (h + 1) * dh)
        assert np.allclose(vt[:, s], vals[:, s] @ a2.T + v2, rtol=1e-10, atol=1e-10)
    yt = attention(xt @ fq[0].T + fq[1], xt @ fk[0].T + fk[1], vt) @ fo_[0].T + fo_[1]
    assert np.allclose(yt, y_ref @ a1.T, rtol=1e-9, atol=1e-9)        # the shift v2 cancelled: softmax rows sum to one
    # the paper's closed forms of the doubly folded layers
    big2, big2inv = np.kron(np.eye(heads), a2), np.kron(np.eye(heads), a2inv)
    assert np.allclose(fv[0], big2 @ Wv @ a1inv)
    assert np.allclose(fv[1], big2 @ bv - big2 @ Wv @ a1inv @ v1 + np.tile(v2, heads))
    assert np.allclose(fo_[0], a1 @ Wo @ big2inv)
    assert np.allclose(fo_[1], a1 @ bo - a1 @ Wo @ big2inv @ np.tile(v2, heads))


def test_identity_transformations_fold_to_the_layer_itself():
    rng = np.random.default_rng(4)
    W, b = rng.standard_normal((6, 8)), rng.standard_normal(6)
    Wt, bt = fo.fold_linear(W, b, a_left=np.eye(6), v_left=np.zeros(6), a_right_inv=np.eye(8), v_right=np.zeros(8))
    assert np.array_equal(Wt, W) and np.array_equal(bt, b)
    Wt, bt = fo.fold_linear(W, None)
    assert np.array_equal(Wt, W) and np.array_equal(bt, np.zeros(6))
