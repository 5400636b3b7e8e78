"""Oracle of the folding of affine transformations into linear layers (the paper's appendix "Folding &
Transformation Structure" and "Affine Transformation inside MHA").

TEST INFRASTRUCTURE ONLY: plain numpy float64, written from the algebra; only tests/, __graft_entry__.smoke() and
bench.py's cpu_baseline leg import it; the product path (the HIP library) shares no code with it.

A transformation acts on column vectors, T(x) = A x + v.  A linear layer is f(x) = W x + b with W [out][in].
  * folding T_r^-1 into the input side:  f(T_r^-1(x)) = (W A_r^-1) x + (b - W A_r^-1 v_r);
  * folding T_l into the output side:    T_l(f(x))    = (A_l W) x + (A_l b + v_l)   (v_l absent where the paper applies
    the matrix only, as on the residual path);
  * both at once (values projection: T_2 after, T_1^-1 before; output projection: A_1 after, T_2^-1 before).
A matrix smaller than the side it acts on is applied block-wise (the same p x p matrix on each group of p features:
one transformation shared by the heads), its shift replicated.
"""
import numpy as np


def _blockdiag(m, n):
    m = np.asarray(m, dtype=np.float64)
    return np.kron(np.eye(n // m.shape[0]), m)


def fold_linear(W, b, a_left=None, v_left=None, a_right_inv=None, v_right=None):
    """(W~, b~) of  x -> T_l(f(T_r^-1(x)))."""
    W = np.asarray(W, dtype=np.float64)
    out, inn = W.shape
    b = np.zeros(out) if b is None else np.asarray(b, dtype=np.float64)
    Wt = W.copy()
    bt = b.copy()
    if a_right_inv is not None:
        Wt = Wt @ _blockdiag(a_right_inv, inn)
    if a_left is not None:
        L = _blockdiag(a_left, out)
        Wt = L @ Wt
        bt = L @ bt
    if v_right is not None:
        bt = bt - Wt @ np.tile(np.asarray(v_right, dtype=np.float64), inn // len(v_right))
    if v_left is not None:
        bt = bt + np.tile(np.asarray(v_left, dtype=np.float64), out // len(v_left))
    return Wt, bt


def fold_embedding(E, A, v):
    """Every embedding vector w_j (a row of E) becomes T(w_j) = A w_j + v."""
    return np.asarray(E, dtype=np.float64) @ np.asarray(A, dtype=np.float64).T + np.asarray(v, dtype=np.float64)
