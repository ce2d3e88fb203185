"""Randomized symmetric HSS compression of a Gaussian kernel matrix (oracle; test
infrastructure).

The paper treats HSS compression as a library call (Algorithm 3, first line)
and cites the literature for it: the HSS form (hierarchical 2x2 partition with
low-rank off-diagonal blocks, Sec. 3.1), randomized sampling of block rows with
oversampling, and per-block truncation to a tolerance eps giving a global
O(eps) error (end of Sec. 3.2).  This file writes that construction out
sequentially, node by node, from those definitions:

  leaf t (rows I_t):   D_t = K(I_t, I_t)
                       S_t = S(I_t,:) - D_t Omega(I_t,:)          (= K(I_t, rest) Omega(rest,:))
                       row interpolative decomposition  S_t ~= U_t S_t(J_t,:)
  inner t = (a, b):    B_ab = K(skel_a, skel_b)                   (entries of K itself)
                       S_t = [S~_a - B_ab Om~_b ; S~_b - B_ab^T Om~_a]
                       row ID again, unless t is the root
  with  S~_t = S_t(J_t,:),  Om~_t = U_t^T [Om~_a; Om~_b]  (Omega(I_t,:) at leaves).

Represented matrix: diagonal leaf blocks D_t exactly; K~(I_a, I_b) = Uh_a B_ab Uh_b^T
with Uh_leaf = U_leaf and Uh_t = blkdiag(Uh_a, Uh_b) U_t.

Nodes are numbered in heap order: root 0, children of t are 2t+1 and 2t+2; the
leaves are the last 2^L nodes, left to right.  Any n: the tree has the shape
`oracle.tree` defines (all leaves on level L, sizes ceil/floor of n / 2^L, leaf i
holds the rows loff[i] .. loff[i+1]-1 of the cluster-tree order).

Which rows an ID picks (and so the ranks) is not unique: "parity unpinned".
What is pinned (tests/test_oracle_hss_ulv.py): reconstruction error <= tolerance
against the dense kernel, exactness when the sample is wide and the tolerance
tiny, the rank-one limit, densify/mat-vec agreement; for the adaptive width:
identity with the fixed-width construction when nothing is cut, the tolerance
met against the dense kernel where the first width alone fails it, and the
width trajectory on a case with known block ranks.
"""
import numpy as np
import scipy.linalg as sla

from .kernel import gaussian_kernel
from .tree import tree_depth, leaf_offsets


def sample(Fp, Omega, h, block=512):
    """S = K(Fp, Fp) @ Omega with K never held whole (row-blocked)."""
    n = Fp.shape[0]
    S = np.empty((n, Omega.shape[1]), dtype=np.float64)
    for i0 in range(0, n, block):
        i1 = min(n, i0 + block)
        S[i0:i1] = gaussian_kernel(Fp[i0:i1], Fp, h) @ Omega
    return S


def row_id(A, rel_tol, abs_tol, kmax):
    """Row interpolative decomposition  A ~= U A[J, :].

    Householder QR with column pivoting of A^T.  Rank k = number of leading
    pivots with |R_jj| > max(rel_tol*|R_00|, abs_tol), capped at kmax.
    Returns (J, U): J (k,) local row indices, U (rows, k) with U[J] = I_k and
    the remaining rows T = (R11^{-1} R12)^T.
    """
    rows = A.shape[0]
    if rows == 0 or A.shape[1] == 0:
        return np.zeros(0, dtype=np.int64), np.zeros((rows, 0))
    R, piv = sla.qr(A.T, mode="r", pivoting=True)
    d = np.abs(np.diag(R))
    thr = max(rel_tol * d[0], abs_tol) if d.size else 0.0
    k = 0
    while k < d.size and k < kmax and d[k] > thr:
        k += 1
    J = np.asarray(piv[:k], dtype=np.int64)
    U = np.zeros((rows, k), dtype=np.float64)
    if k:
        U[J, np.arange(k)] = 1.0
        if k < rows:
            T = sla.solve_triangular(R[:k, :k], R[:k, k:], lower=False)   # k x (rows-k)
            U[piv[k:], :] = T.T
    return J, U


class HSS:
    """Container for the generators of a symmetric HSS matrix."""

    def __init__(self, n, leaf):
        self.n = int(n)
        self.leaf = int(leaf)                   # largest leaf size
        self.L = tree_depth(self.n, self.leaf)
        nl = 1 << self.L
        self.loff = leaf_offsets(self.n, self.L)   # rows of leaf i: loff[i] .. loff[i+1]-1
        self.nnodes = 2 * nl - 1
        self.D = [None] * nl                    # leaf diagonal blocks, left to right
        self.U = [None] * self.nnodes           # (size_t, k_t); None at the root
        self.J = [None] * self.nnodes           # local skeleton rows
        self.B = [None] * self.nnodes           # (k_a, k_b) at inner nodes
        self.skel = [None] * self.nnodes        # global (permuted-order) skeleton indices

    def first_leaf(self):
        return (1 << self.L) - 1

    def is_leaf(self, t):
        return t >= self.first_leaf()

    def level_nodes(self, l):
        return range((1 << l) - 1, (1 << (l + 1)) - 1)

    def rank(self, t):
        return 0 if self.U[t] is None else self.U[t].shape[1]

    def leaf_rows(self, i):
        """Rows (cluster-tree order) of leaf i, counted from the left."""
        return np.arange(self.loff[i], self.loff[i + 1])

    def span(self, t):
        """First row and one past the last row of the points under node t."""
        l = (t + 1).bit_length() - 1
        i = t - ((1 << l) - 1)
        w = 1 << (self.L - l)                   # leaves under a node of level l
        return int(self.loff[i * w]), int(self.loff[(i + 1) * w])

    def size(self, t):
        if self.is_leaf(t):
            i = t - self.first_leaf()
            return int(self.loff[i + 1] - self.loff[i])
        return self.rank(2 * t + 1) + self.rank(2 * t + 2)

    def ranks(self):
        return np.array([self.rank(t) for t in range(self.nnodes)], dtype=np.int64)


def compress(Fp, h, leaf, Omega, rel_tol, abs_tol=0.0, kmax=None, S=None):
    """Build the HSS generators of K(Fp, Fp) from the random sample S = K Omega.

    Fp: points already in cluster-tree order.  Omega: (n, s).  kmax: rank cap
    (default s).  S may be passed if already computed.
    """
    Fp = np.asarray(Fp, dtype=np.float64)
    n = Fp.shape[0]
    s = Omega.shape[1]
    if kmax is None:
        kmax = s
    H = HSS(n, leaf)
    if S is None:
        S = sample(Fp, Omega, h)
    Sred = [None] * H.nnodes     # S~_t
    Ored = [None] * H.nnodes     # Om~_t
    fl = H.first_leaf()
    for l in range(H.L, -1, -1):
        for t in H.level_nodes(l):
            if H.is_leaf(t):
                i = t - fl
                rows = H.leaf_rows(i)
                Dt = gaussian_kernel(Fp[rows], Fp[rows], h)
                H.D[i] = Dt
                St = S[rows] - Dt @ Omega[rows]
                Ot = Omega[rows]
                idx = rows
            else:
                a, b = 2 * t + 1, 2 * t + 2
                Bab = gaussian_kernel(Fp[H.skel[a]], Fp[H.skel[b]], h)
                H.B[t] = Bab
                St = np.vstack([Sred[a] - Bab @ Ored[b], Sred[b] - Bab.T @ Ored[a]])
                Ot = np.vstack([Ored[a], Ored[b]])
                idx = np.concatenate([H.skel[a], H.skel[b]])
                Sred[a] = Sred[b] = Ored[a] = Ored[b] = None
            if t == 0:
                break
            J, U = row_id(St, rel_tol, abs_tol, kmax)
            H.J[t], H.U[t] = J, U
            H.skel[t] = idx[J]
            Sred[t] = St[J]
            Ored[t] = U.T @ Ot
    return H


def compress_adaptive(Fp, h, leaf, Omega, rel_tol, abs_tol=0.0, s0=None, step=128, oversample=None, kmax=None,
                      S=None):
    """The same construction with an adaptive sample width (oversampling and per-block
    truncation to the tolerance, end of Sec. 3.2): the decompositions of a level first
    see only the leading `width` columns of the sample; while some node of the level is
    cut by the sample's rank cap (and not by the tolerance) and columns are left, the
    width grows by `step` and the cut nodes -- only those -- are decomposed again from
    the wider sample.  The width never shrinks on the way up the tree.

    Omega (n, s) holds ALL columns that may ever be used; s0 is the first width
    (default s: no adaptivity, identical to `compress`).  Rank cap at width c:
    c - p with p = `oversample` (default c // 2), never above `kmax` (default: the
    cap at the full width s).

    A column of S~_t = S_t(J_t, :) or Om~_t = U_t^T Om_t depends on the same column
    of S and Omega only, so using "the first c columns" of quantities computed at
    full width equals computing the new columns when the width grows.

    Returns (H, info): info["width"] = final width, info["level_width"][l] = width
    in use when level l was finished, info["redone"] = number of node
    decompositions repeated, info["nodes_at_cap"] = nodes still cut by a cap.
    """
    Fp = np.asarray(Fp, dtype=np.float64)
    n = Fp.shape[0]
    s = Omega.shape[1]
    width = s if s0 is None else min(int(s0), s)
    cap_at = lambda c: c - (c // 2 if oversample is None else int(oversample))
    kfinal = cap_at(s) if kmax is None else int(kmax)
    H = HSS(n, leaf)
    if S is None:
        S = sample(Fp, Omega, h)
    Sred = [None] * H.nnodes
    Ored = [None] * H.nnodes
    fl = H.first_leaf()
    info = {"level_width": {}, "redone": 0, "nodes_at_cap": 0}
    for l in range(H.L, -1, -1):
        St, Ot, idx = {}, {}, {}
        for t in H.level_nodes(l):
            if H.is_leaf(t):
                i = t - fl
                rows = H.leaf_rows(i)
                H.D[i] = gaussian_kernel(Fp[rows], Fp[rows], h)
                St[t] = S[rows] - H.D[i] @ Omega[rows]
                Ot[t] = Omega[rows]
                idx[t] = rows
            else:
                a, b = 2 * t + 1, 2 * t + 2
                H.B[t] = gaussian_kernel(Fp[H.skel[a]], Fp[H.skel[b]], h)
                St[t] = np.vstack([Sred[a] - H.B[t] @ Ored[b], Sred[b] - H.B[t].T @ Ored[a]])
                Ot[t] = np.vstack([Ored[a], Ored[b]])
                idx[t] = np.concatenate([H.skel[a], H.skel[b]])
                Sred[a] = Sred[b] = Ored[a] = Ored[b] = None
        if l == 0:
            break
        todo = list(H.level_nodes(l))
        while True:
            cap = min(cap_at(width), kfinal)
            if cap < 1:
                raise ValueError("rank cap below 1")
            cut = []
            for t in todo:
                J, U = row_id(St[t][:, :width], rel_tol, abs_tol, cap)
                H.J[t], H.U[t] = J, U
                if J.size == cap and J.size < St[t].shape[0]:
                    cut.append(t)
            if not cut or width >= s or cap >= kfinal:
                info["nodes_at_cap"] += len(cut)
                break
            width = min(s, width + int(step))
            todo = cut
            info["redone"] += len(cut)
        info["level_width"][l] = width
        for t in H.level_nodes(l):
            H.skel[t] = idx[t][H.J[t]]
            Sred[t] = St[t][H.J[t]]
            Ored[t] = H.U[t].T @ Ot[t]
    info["width"] = width
    return H, info


def nested_basis(H, t):
    """Uh_t: (number of points under t, k_t)."""
    if H.is_leaf(t):
        return H.U[t]
    a, b = 2 * t + 1, 2 * t + 2
    Ua, Ub = nested_basis(H, a), nested_basis(H, b)
    blk = np.zeros((Ua.shape[0] + Ub.shape[0], Ua.shape[1] + Ub.shape[1]))
    blk[:Ua.shape[0], :Ua.shape[1]] = Ua
    blk[Ua.shape[0]:, Ua.shape[1]:] = Ub
    return blk @ H.U[t]


def densify(H):
    """The n x n matrix the generators represent (small n only)."""
    n = H.n
    A = np.zeros((n, n))
    fl = H.first_leaf()
    for i in range(len(H.D)):
        a0, a1 = H.loff[i], H.loff[i + 1]
        A[a0:a1, a0:a1] = H.D[i]
    span = H.span
    for t in range(fl):
        a, b = 2 * t + 1, 2 * t + 2
        Ua, Ub = nested_basis(H, a), nested_basis(H, b)
        blk = Ua @ H.B[t] @ Ub.T
        a0, a1 = span(a)
        b0, b1 = span(b)
        A[a0:a1, b0:b1] = blk
        A[b0:b1, a0:a1] = blk.T
    return A


def matvec(H, x):
    """y = K~ x for x in cluster-tree order: up-sweep x~ = U^T(.), down-sweep
    through B, leaves add D x (the standard two-pass HSS product)."""
    x = np.asarray(x, dtype=np.float64)
    lo = H.loff
    fl = H.first_leaf()
    xt = [None] * H.nnodes
    for t in range(H.nnodes - 1, 0, -1):
        if H.is_leaf(t):
            i = t - fl
            xt[t] = H.U[t].T @ x[lo[i]:lo[i + 1]]
        else:
            xt[t] = H.U[t].T @ np.concatenate([xt[2 * t + 1], xt[2 * t + 2]])
    g = [None] * H.nnodes
    y = np.empty_like(x)
    for t in range(H.nnodes):
        if H.is_leaf(t):
            i = t - fl
            y[lo[i]:lo[i + 1]] = H.D[i] @ x[lo[i]:lo[i + 1]]
            if t != 0:
                y[lo[i]:lo[i + 1]] += H.U[t] @ g[t]
            continue
        a, b = 2 * t + 1, 2 * t + 2
        ka = H.rank(a)
        if t == 0:
            ha = np.zeros(ka)
            hb = np.zeros(H.rank(b))
        else:
            hv = H.U[t] @ g[t]
            ha, hb = hv[:ka], hv[ka:]
        g[a] = ha + H.B[t] @ xt[b]
        g[b] = hb + H.B[t].T @ xt[a]
    return y


def psd_shift(H, safety=1.1, tol=1e-3):
    """delta >= 0 such that K~ + delta*I is (numerically) positive semidefinite.

    The paper's trainer presupposes a convex approximate problem (eq. 8): ADMM is
    called convergent and the ULV factors are those of a definite matrix.  When
    the ranks saturate, the compressed matrix can lose definiteness; the guard
    adds delta = safety * max(0, -lambda_min(K~)) to the diagonal (only the leaf
    blocks change, exactly as for the beta shift).  delta = 0 whenever K~ is
    already positive semidefinite.  lambda_min comes from a Lanczos run on the
    HSS mat-vec (library routine)."""
    import scipy.sparse.linalg as spla
    if H.n <= 512:
        lam = float(np.linalg.eigvalsh(densify(H))[0])
    else:
        op = spla.LinearOperator((H.n, H.n), matvec=lambda v: matvec(H, v), dtype=np.float64)
        lam = float(spla.eigsh(op, k=1, which="SA", tol=tol, return_eigenvectors=False)[0])
    return safety * max(0.0, -lam)


def add_diagonal(H, delta):
    """K~ <- K~ + delta*I (in place, leaf diagonal blocks only)."""
    if delta != 0.0:
        for i in range(len(H.D)):
            H.D[i] = H.D[i] + delta * np.eye(H.D[i].shape[0])
    return H
