"""Closed-form ADMM for the dual SVM QP (oracle; test infrastructure).

Problem (eq. 1):  min 1/2 x^T Y K Y x - e^T x,  y^T x = 0,  0 <= x <= C.
Splitting x = z (eq. 3), augmented Lagrangian (eq. 4) with multiplier mu and
penalty beta.  One iteration (Algorithm 2), with q^k = e + mu^k + beta z^k and
K_beta = K + beta I:

   x^{k+1}  = Y K_beta^{-1} Y q^k - (e^T K_beta^{-1} Y q^k / e^T K_beta^{-1} e) Y K_beta^{-1} e
   z^{k+1}  = clip(x^{k+1} - mu^k / beta, 0, C)                          (eq. 6)
   mu^{k+1} = mu^k - beta (x^{k+1} - z^{k+1})

Algorithm 3 precomputes w = Y K_beta^{-1} e and w1 = e^T K_beta^{-1} e once per
(h, beta).  Readings where the printed text is garbled or silent:
  * Algorithm 3's inner loop prints x^k where q^k is meant (with x^k the
    iterates z, mu would never feed back); Algorithm 2 and the derivation in
    Sec. 2.1 fix it: q^k.
  * Start: x = z = mu = 0 for every (C, beta) (the paper re-initialises inside
    the loop over C and gives no values).
  * The model is z^{MaxIt} (Algorithm 3 uses it for the bias and the labels).
  * Bias: eq. (2)/(7) and Algorithm 3 print b = sum_i y_i x_i K_ij - y_j, which
    together with the classifier sign(sum_i y_i x_i K(f_i, f) + b) contradicts
    the margin condition y_j (sum_i y_i x_i K_ij + b) = 1 for 0 < x_j < C.  The
    sign that satisfies it is b = y_j - sum_i y_i x_i K_ij, averaged over the
    margin set M as in eq. (7).  tests/test_oracle_admm.py checks the margin
    identity on an exact QP solution, which decides the sign.
"""
import numpy as np
import scipy.linalg as sla

from .kernel import gaussian_kernel


def admm(solve, y, C, beta, maxit, history=False):
    """Run `maxit` iterations.  `solve(v)` applies K_beta^{-1} to a vector.

    Returns dict(x, z, mu) (and per-iteration y^T x if history).
    """
    y = np.asarray(y, dtype=np.float64)
    n = y.size
    e = np.ones(n)
    wbar = solve(e)
    w1 = float(e @ wbar)
    w = y * wbar
    x = np.zeros(n)
    z = np.zeros(n)
    mu = np.zeros(n)
    ytx = []
    for _ in range(maxit):
        q = e + mu + beta * z
        w2 = float(w @ q)
        x = y * solve(y * q) - (w2 / w1) * w
        z = np.minimum(np.maximum(x - mu / beta, 0.0), C)
        mu = mu - beta * (x - z)
        if history:
            ytx.append(float(y @ x))
    out = {"x": x, "z": z, "mu": mu}
    if history:
        out["ytx"] = np.array(ytx)
    return out


def admm_dense(K, y, C, beta, maxit, history=False):
    """ADMM with K_beta^{-1} applied through a dense Cholesky factor."""
    n = K.shape[0]
    cf = sla.cho_factor(K + beta * np.eye(n), lower=True)
    return admm(lambda v: sla.cho_solve(cf, v), y, C, beta, maxit, history)


def margin_set(z, C):
    """M = {j : 0 < z_j < C}, strict, on the projected iterate."""
    return (z > 0.0) & (z < C)


def bias(z, y, C, kmatvec, M=None):
    """Averaged bias over the margin set with one kernel mat-vec (eq. 7 with the
    sign fixed by the margin identity).  kmatvec(v) = K v (or K~ v).
    M: the margin set as a boolean mask; default {j : 0 < z_j < C}.  (A caller
    comparing two nearly equal iterates passes one of the two sets to both, so
    that an entry within rounding of a bound does not change the average.)
    Returns (b, |M|); b = 0 when M is empty."""
    if M is None:
        M = margin_set(z, C)
    cnt = int(M.sum())
    if cnt == 0:
        return 0.0, 0
    ebar = M.astype(np.float64)
    zy = y * z
    b = (float(y[M].sum()) - float(zy @ kmatvec(ebar))) / cnt
    return b, cnt


def decision(F, y, z, b, G, h, block=2048):
    """dec_j = sum_i y_i z_i K(f_i, g_j) + b with the exact kernel (label
    assignment loop of Algorithm 3)."""
    zy = y * z
    out = np.empty(G.shape[0])
    for j0 in range(0, G.shape[0], block):
        j1 = min(G.shape[0], j0 + block)
        out[j0:j1] = gaussian_kernel(G[j0:j1], F, h) @ zy + b
    return out


def labels(dec):
    return np.where(dec >= 0.0, 1.0, -1.0)


def accuracy(dec, y_true):
    return float((labels(dec) == y_true).mean()) * 100.0
