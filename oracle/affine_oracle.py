"""Oracle of the LU parametrisation of a learnable invertible matrix (the paper's Section on learning affine
transformations: Eq. 4, the volume regulariser of Eq. 6 and its practical log form).

TEST INFRASTRUCTURE ONLY: plain numpy float64, no blocking or fusion, written from the definitions so that it can be
checked against the paper by eye.  Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg import it;
the product path (the HIP library) shares no code with it.

Conventions (the paper fixes the factorisation, not the storage):
  * Lp, Up: full d x d arrays of free parameters; only the strictly lower part of Lp and the strictly upper part of
    Up are used (L = I + tril(Lp, -1) is unit lower triangular, U = triu(Up, 1) has a zero diagonal);
  * the diagonal vector is s = sign * exp(log_s): the paper learns log|s| and keeps the signs fixed;
  * the fixed permutation matrix P is given as an index vector: (P M)[i, :] = M[perm[i], :].
"""
import numpy as np


def lu_factors(Lp, Up, log_s, sign):
    """L (unit lower), U + diag(s) (upper) and s of Eq. 4."""
    Lp = np.asarray(Lp, dtype=np.float64)
    Up = np.asarray(Up, dtype=np.float64)
    s = np.asarray(sign, dtype=np.float64) * np.exp(np.asarray(log_s, dtype=np.float64))
    d = s.shape[0]
    L = np.tril(Lp, -1) + np.eye(d)
    UD = np.triu(Up, 1) + np.diag(s)
    return L, UD, s


def lu_compose(Lp, Up, log_s, sign, perm):
    """A = P L (U + diag(s)), Eq. 4."""
    L, UD, _ = lu_factors(Lp, Up, log_s, sign)
    return (L @ UD)[np.asarray(perm)]


def lu_gradients(G, Lp, Up, log_s, sign, perm):
    """Gradients of a scalar loss with respect to the free parameters, given G = d loss / d A.
    With B = P^T G (the gradient with respect to L (U + diag s)):  d/dL = B (U + diag s)^T restricted to the strictly
    lower part, d/d(U + diag s) = L^T B, of which the strictly upper part belongs to U and the diagonal to s;
    s = sign * exp(log_s) gives d/dlog_s = (d/ds) * s."""
    L, UD, s = lu_factors(Lp, Up, log_s, sign)
    perm = np.asarray(perm)
    B = np.empty_like(np.asarray(G, dtype=np.float64))
    B[perm] = np.asarray(G, dtype=np.float64)          # row perm[i] of B is row i of G
    dL = np.tril(B @ UD.T, -1)
    dUD = L.T @ B
    dU = np.triu(dUD, 1)
    dlog_s = np.diag(dUD) * s
    return dL, dU, dlog_s


def vol_loss(s):
    """Eq. 6: (prod |s_i| - 1)^2."""
    return (np.prod(np.abs(np.asarray(s, dtype=np.float64))) - 1.0) ** 2


def vol_penalty(log_s):
    """The form used in practice: (sum_i log|s_i|)^2 and its gradient with respect to log|s|."""
    t = float(np.sum(np.asarray(log_s, dtype=np.float64)))
    return t * t, np.full(np.shape(log_s), 2.0 * t)


# ---- QR parametrisation (Eq. 5):  Q = exp((G - G^T) / 2),  A = Q (R + diag(s)) ------------------------------------
# G: full d x d array of free parameters; Rp: full d x d array of which the strictly upper part is used; s as above.
# The matrix exponential and its Frechet derivative are library routines (scipy.linalg), used as single steps.

def qr_factors(G, Rp, log_s, sign):
    """Q (orthogonal, determinant +1), R + diag(s) (upper triangular) and s of Eq. 5."""
    import scipy.linalg
    G = np.asarray(G, dtype=np.float64)
    s = np.asarray(sign, dtype=np.float64) * np.exp(np.asarray(log_s, dtype=np.float64))
    S = 0.5 * (G - G.T)
    Q = scipy.linalg.expm(S)
    RD = np.triu(np.asarray(Rp, dtype=np.float64), 1) + np.diag(s)
    return Q, RD, s


def qr_compose(G, Rp, log_s, sign):
    """A = Q (R + diag(s)), Eq. 5."""
    Q, RD, _ = qr_factors(G, Rp, log_s, sign)
    return Q @ RD


def qr_gradients(dA, G, Rp, log_s, sign):
    """Gradients of a scalar loss with respect to G, the strictly upper part of R and log|s|, given dA = d loss / d A.
    d/d(R + diag s) = Q^T dA; d/dQ = dA (R + diag s)^T; the exponential's adjoint maps d/dQ to d/dS =
    L_exp(S^T, d/dQ) (the Frechet derivative of exp at S^T in the direction d/dQ); S = (G - G^T)/2 gives
    d/dG = (d/dS - (d/dS)^T) / 2."""
    import scipy.linalg
    dA = np.asarray(dA, dtype=np.float64)
    Q, RD, s = qr_factors(G, Rp, log_s, sign)
    dRD = Q.T @ dA
    dR = np.triu(dRD, 1)
    dlog_s = np.diag(dRD) * s
    dQ = dA @ RD.T
    S = 0.5 * (np.asarray(G, dtype=np.float64) - np.asarray(G, dtype=np.float64).T)
    dS = scipy.linalg.expm_frechet(S.T, dQ, compute_expm=False)
    dG = 0.5 * (dS - dS.T)
    return dG, dR, dlog_s
