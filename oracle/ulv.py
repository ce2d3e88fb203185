"""ULV factorization and solve of A = K~ + beta*I for a symmetric HSS matrix K~
(oracle; test infrastructure).

The paper uses this as a library call (Algorithm 3: "ULVfactorization" and the
repeated application of (ULV)^{-1}); Sec. 3.1 describes it as a factorization
into orthogonal U, V and a lower-triangular L, computed once per (h, beta) and
reused for every solve.  Written out sequentially from that idea:

  node t with diagonal block D (size m) and basis U (m x k):
     Q = full Householder QR factor of U, so Q^T U = [R; 0]
     Dh = Q^T D Q = [[Drr, Dre], [Der, Dee]]       (r: first k rows, e: last m-k)
     the e-rows no longer couple outside the node -> eliminate them with an LU
     of Dee;  Schur complement Dt = Drr - Dre Dee^{-1} Der and Ut = R go up.
  parent t of (a, b): D = [[Dt_a, Ut_a B Ut_b^T], [sym, Dt_b]],
                      U = blkdiag(Ut_a, Ut_b) U_t
  root: dense LU of D.

Pinned by tests/test_oracle_ulv.py against a dense solve of densify(K~)+beta*I,
the one-leaf case and a Sherman-Morrison closed form.
"""
import numpy as np
import scipy.linalg as sla


class ULV:
    def __init__(self, H, beta):
        self.H = H
        self.beta = float(beta)
        nn = H.nnodes
        self.Q = [None] * nn
        self.k = [0] * nn
        self.m = [0] * nn
        self.Dre = [None] * nn
        self.Der = [None] * nn
        self.lu_ee = [None] * nn
        self.root_lu = None


def ulv_factor(H, beta):
    F = ULV(H, beta)
    nn = H.nnodes
    fl = H.first_leaf()
    Dt = [None] * nn      # reduced diagonal block passed to the parent
    Ut = [None] * nn      # reduced basis passed to the parent
    for t in range(nn - 1, -1, -1):
        if H.is_leaf(t):
            D = H.D[t - fl] + beta * np.eye(H.D[t - fl].shape[0])
            U = H.U[t]
        else:
            a, b = 2 * t + 1, 2 * t + 2
            off = Ut[a] @ H.B[t] @ Ut[b].T
            D = np.block([[Dt[a], off], [off.T, Dt[b]]])
            if t != 0:
                ka = Ut[a].shape[0]
                U = np.vstack([Ut[a] @ H.U[t][:ka], Ut[b] @ H.U[t][ka:]])
            Dt[a] = Dt[b] = Ut[a] = Ut[b] = None
        m = D.shape[0]
        F.m[t] = m
        if t == 0:
            F.root_lu = sla.lu_factor(D) if m else None
            break
        k = U.shape[1]
        F.k[t] = k
        if k == m:                       # nothing to eliminate
            Dt[t], Ut[t] = D, U
            continue
        if k == 0:
            Q = np.eye(m)
            R = np.zeros((0, 0))
        else:
            Q, Rfull = sla.qr(U, mode="full")
            R = Rfull[:k]
        Dh = Q.T @ D @ Q
        Dee = Dh[k:, k:]
        lu = sla.lu_factor(Dee)
        F.Q[t] = Q
        F.lu_ee[t] = lu
        F.Dre[t] = Dh[:k, k:]
        F.Der[t] = Dh[k:, :k]
        Dt[t] = Dh[:k, :k] - Dh[:k, k:] @ sla.lu_solve(lu, Dh[k:, :k])
        Ut[t] = R
    return F


def ulv_solve(F, b):
    """x = (K~ + beta I)^{-1} b for b in cluster-tree order (1-D or (n, nrhs))."""
    H = F.H
    b = np.asarray(b, dtype=np.float64)
    one = b.ndim == 1
    Bm = b.reshape(H.n, -1)
    nn = H.nnodes
    fl = H.first_leaf()
    lo = H.loff              # rows of leaf i: lo[i] .. lo[i+1]-1
    red = [None] * nn        # reduced right-hand side passed up
    ce = [None] * nn         # Dee^{-1} b_e kept for the way down
    for t in range(nn - 1, -1, -1):
        if H.is_leaf(t):
            bt = Bm[lo[t - fl]:lo[t - fl + 1]]
        else:
            bt = np.vstack([red[2 * t + 1], red[2 * t + 2]])
        if t == 0:
            xroot = sla.lu_solve(F.root_lu, bt) if F.m[0] else bt
            break
        k = F.k[t]
        if k == F.m[t]:
            red[t] = bt
            continue
        bh = F.Q[t].T @ bt
        c = sla.lu_solve(F.lu_ee[t], bh[k:])
        ce[t] = c
        red[t] = bh[:k] - F.Dre[t] @ c
    X = np.empty_like(Bm)
    xin = [None] * nn
    xin[0] = xroot
    for t in range(nn):
        if t == 0:
            xt = xin[0]
        else:
            k = F.k[t]
            if k == F.m[t]:
                xt = xin[t]
            else:
                xe = ce[t] - sla.lu_solve(F.lu_ee[t], F.Der[t] @ xin[t])
                xt = F.Q[t] @ np.vstack([xin[t], xe])
        if H.is_leaf(t):
            X[lo[t - fl]:lo[t - fl + 1]] = xt
        else:
            ka = F.k[2 * t + 1]
            xin[2 * t + 1] = xt[:ka]
            xin[2 * t + 2] = xt[ka:]
    return X[:, 0] if one else X
