"""Approximate nearest neighbours and the neighbour-based HSS construction (oracle; test
infrastructure).

The paper's own compressor (Sec. 3.1, first bullet) does not sample K with a random
matrix: it uses the kernel as a similarity measure, takes the columns that belong to the
dominating approximate nearest neighbours of a node's points as the sample of that
node's off-diagonal block row, and decomposes that.  The paper gives no algorithm for it
(it cites the literature); the reading implemented here, step by step:

  neighbours   every point i gets a list of `k` (index, squared distance) pairs, ascending
               by (distance, index), never containing i.  `knn_exact` is the definition;
               `ann_projection_trees` is the approximate search: `trees` random projection
               trees (a cell is split at the median of the projections on a random
               direction until it holds `cell` points), exact search inside every cell,
               the lists of the trees merged (distinct indices, the k closest).  Tree 0
               uses the cells of the cluster-tree order itself (contiguous runs).
  node t       rows R_t: its points (leaf) or the skeleton points of its two children;
               candidate columns: every neighbour-list entry of every row of R_t whose
               index lies OUTSIDE the node's own index range, scored by its squared distance
               (an index listed by several rows keeps its smallest distance); the sample
               columns N_t are the `s` candidates with the smallest (score, index);
               S_t = K(R_t, N_t)  (entries of K itself);  row interpolative decomposition
               S_t ~= U_t S_t(J_t, :) as in the randomized construction; B_ab = K(skel_a, skel_b).
The result has the same generators (D, U, J, B) as oracle.hss.compress produces, so that
densify, mat-vec and the ULV solve apply unchanged.

Which neighbours an approximate search finds, and which rows a decomposition picks, is
not unique: "parity unpinned".  Pinned (tests/test_oracle_ann.py): knn_exact against a
full sort, the approximate search against it (valid entries, exact distances, recall, exact
within a cell), exactness of the construction when every outside column is a candidate,
reconstruction error on separated clusters, and the generator invariants.
"""
import numpy as np

from .hss import HSS, row_id
from .kernel import gaussian_kernel


def _dist2_block(A, B):
    """Squared distances by direct differences, one feature after the other."""
    d2 = np.zeros((A.shape[0], B.shape[0]))
    for f in range(A.shape[1]):
        diff = A[:, f][:, None] - B[:, f][None, :]
        d2 += diff * diff
    return d2


def _k_smallest(d2, ids, k):
    """Per row: the k smallest (distance, index) pairs, ascending; rows may hold fewer
    than k finite candidates (padded with index -1, distance inf)."""
    m = d2.shape[0]
    order = np.lexsort((np.broadcast_to(ids, d2.shape), d2), axis=1)[:, :k]
    out_d = np.take_along_axis(d2, order, axis=1)
    out_i = np.take_along_axis(np.broadcast_to(ids, d2.shape), order, axis=1).astype(np.int64)
    out_i = np.where(np.isfinite(out_d), out_i, -1)
    if out_d.shape[1] < k:
        pad = k - out_d.shape[1]
        out_d = np.hstack([out_d, np.full((m, pad), np.inf)])
        out_i = np.hstack([out_i, np.full((m, pad), -1, dtype=np.int64)])
    return out_i, out_d


def knn_exact(F, k, block=512):
    """The k nearest neighbours of every point among all others (the definition)."""
    n = F.shape[0]
    idx = np.empty((n, k), dtype=np.int64)
    dist = np.empty((n, k))
    ids = np.arange(n)
    for i0 in range(0, n, block):
        i1 = min(n, i0 + block)
        d2 = _dist2_block(F[i0:i1], F)
        d2[np.arange(i1 - i0), np.arange(i0, i1)] = np.inf      # never the point itself
        idx[i0:i1], dist[i0:i1] = _k_smallest(d2, ids, k)
    return idx, dist


def _merge_lists(idx_a, dist_a, idx_b, dist_b, k):
    """Row-wise union of two neighbour lists: distinct indices, the k closest."""
    n = idx_a.shape[0]
    out_i = np.full((n, k), -1, dtype=np.int64)
    out_d = np.full((n, k), np.inf)
    for i in range(n):
        ii = np.concatenate([idx_a[i], idx_b[i]])
        dd = np.concatenate([dist_a[i], dist_b[i]])
        keep = ii >= 0
        ii, dd = ii[keep], dd[keep]
        order = np.lexsort((dd, ii))                 # by index, then distance: first of each index = closest
        ii, dd = ii[order], dd[order]
        first = np.ones(ii.size, dtype=bool)
        first[1:] = ii[1:] != ii[:-1]
        ii, dd = ii[first], dd[first]
        order = np.lexsort((ii, dd))[:k]
        out_i[i, :order.size] = ii[order]
        out_d[i, :order.size] = dd[order]
    return out_i, out_d


def cells_of_projection_tree(F, cell, direction):
    """Leaves (index arrays, left to right) of one random projection tree: a set is split at
    the median of the projections of its points on a random direction until it holds at
    most `cell` points.  direction(level, node) -> (r,) vector of the node-th set (left to
    right) of a level.  A projection is accumulated feature by feature in index order,
    every product and sum rounded on its own; ties go to the lowest index."""
    r = F.shape[1]
    level = [np.arange(F.shape[0], dtype=np.int64)]
    l = 0
    while level[0].size > cell:
        nxt = []
        for node, idx in enumerate(level):
            d = direction(l, node)
            p = np.zeros(idx.size)
            for f in range(r):
                p = p + F[idx, f] * d[f]
            order = np.lexsort((idx, p))
            half = (idx.size + 1) // 2           # same shape as the cluster tree: ceil(p/2) points go left
            nxt.append(idx[order[:half]])
            nxt.append(idx[order[half:]])
        level = nxt
        l += 1
    return level


def knn_in_cells(F, cells, k):
    """Exact k nearest neighbours of every point among the other points of its own cell."""
    n = F.shape[0]
    idx = np.full((n, k), -1, dtype=np.int64)
    dist = np.full((n, k), np.inf)
    for c in cells:
        d2 = _dist2_block(F[c], F[c])
        d2[np.arange(c.size), np.arange(c.size)] = np.inf
        idx[c], dist[c] = _k_smallest(d2, c, k)
    return idx, dist


def ann_projection_trees(F, k, cell, trees, seed=0, directions=None, first_cells=None):
    """Approximate k nearest neighbours: tree 0 = contiguous runs of `cell` points in the
    given order (for points in cluster-tree order: the cells of that tree; `first_cells`
    = offsets of the runs when they are not all `cell` long, then `cell` is the longest),
    trees 1 .. trees-1 = random projection trees; exact search inside every cell; lists
    merged.  directions(tree, level, node) -> (r,) supplies the random directions
    (default: normal numbers from a generator seeded with `seed`)."""
    n = F.shape[0]
    if directions is None:
        rng = np.random.default_rng(seed)
        directions = lambda t, l, node: rng.standard_normal(F.shape[1])
    if first_cells is None:
        first_cells = list(range(0, n, cell)) + [n]
    cells = [np.arange(a, b, dtype=np.int64) for a, b in zip(first_cells[:-1], first_cells[1:])]
    idx, dist = knn_in_cells(F, cells, k)
    for t in range(1, trees):
        tree_cells = cells_of_projection_tree(F, cell, lambda l, node: directions(t, l, node))
        i2, d2 = knn_in_cells(F, tree_cells, k)
        idx, dist = _merge_lists(idx, dist, i2, d2, k)
    return idx, dist


def select_columns(rows, nbr_idx, nbr_dist, lo, hi, s):
    """The sample columns of a node with index range [lo, hi) and row points `rows`:
    neighbour-list entries of the rows that fall outside the range, distinct (smallest
    distance kept), the s smallest by (distance, index)."""
    ii = nbr_idx[rows].reshape(-1)
    dd = nbr_dist[rows].reshape(-1)
    keep = (ii >= 0) & ((ii < lo) | (ii >= hi))
    ii, dd = ii[keep], dd[keep]
    order = np.lexsort((dd, ii))
    ii, dd = ii[order], dd[order]
    first = np.ones(ii.size, dtype=bool)
    first[1:] = ii[1:] != ii[:-1]
    ii, dd = ii[first], dd[first]
    order = np.lexsort((ii, dd))[:s]
    return ii[order]


def compress_ann(Fp, h, leaf, nbr_idx, nbr_dist, s, rel_tol, abs_tol=0.0, kmax=None):
    """Neighbour-based HSS construction (see the module header).  Fp: points in
    cluster-tree order; nbr_idx/nbr_dist: (n, k) neighbour lists in that order; s:
    number of sample columns per node; kmax: rank cap (default s).
    Returns (H, info) with info["columns"][t] = number of sample columns of node t."""
    Fp = np.asarray(Fp, dtype=np.float64)
    n = Fp.shape[0]
    if kmax is None:
        kmax = s
    H = HSS(n, leaf)
    fl = H.first_leaf()
    info = {"columns": {}}
    for l in range(H.L, -1, -1):
        for t in H.level_nodes(l):
            lo, hi = H.span(t)
            if H.is_leaf(t):
                rows = np.arange(lo, hi)
                H.D[t - fl] = gaussian_kernel(Fp[rows], Fp[rows], h)
            else:
                a, b = 2 * t + 1, 2 * t + 2
                H.B[t] = gaussian_kernel(Fp[H.skel[a]], Fp[H.skel[b]], h)
                rows = np.concatenate([H.skel[a], H.skel[b]])
            if t == 0:
                break
            cols = select_columns(rows, nbr_idx, nbr_dist, lo, hi, s)
            info["columns"][t] = int(cols.size)
            St = gaussian_kernel(Fp[rows], Fp[cols], h) if cols.size else np.zeros((rows.size, 0))
            J, U = row_id(St, rel_tol, abs_tol, kmax)
            if J.size == 0:                     # no column at all (or a zero block): keep one row, as the device does
                J = np.zeros(1, dtype=np.int64)
                U = np.zeros((rows.size, 1))
                U[0, 0] = 1.0
            H.J[t], H.U[t] = J, U
            H.skel[t] = rows[J]
    return H, info
