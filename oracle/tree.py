"""Cluster trees by balanced bisection (oracle; test infrastructure): along a coordinate
(`cluster_tree`) or along the line between the two centres of a 2-means pass over the
node (`cluster_tree_2means`, data-driven).

Shape of the tree for any number of points n and largest leaf size `leaf`
(`tree_depth`, `leaf_offsets`): the depth L is the smallest one with
ceil(n / 2^L) <= leaf; a node of p points gives its lower ceil(p/2) points (in the
node's sort order) to the left child and the other floor(p/2) to the right one, on
every level down to L.  All leaves are on level L and their sizes differ by at most
one; with n = leaf * 2^L every leaf holds exactly `leaf` points.

The paper only says that the points are clustered/reordered before compression
so that off-diagonal blocks become low-rank (Sec. 1.2, first bullet; Fig. 1).
The reading used here: a perfect binary tree; a node's points are split at the
median of the coordinate with the largest variance over the node.  Variances
within a relative 1e-9 of the largest count as equal (the lowest coordinate
wins), so that the choice does not hinge on the rounding of a sum -- columns
standardised to unit variance differ only by that.
"""
import numpy as np

TIE = 1e-9   # relative width of a tie between variances


def tree_depth(n, leaf):
    """Smallest L with ceil(n / 2^L) <= leaf."""
    n, leaf = int(n), int(leaf)
    if n < 1 or leaf < 1:
        raise ValueError("n and leaf must be positive")
    L = 0
    while -(-n // (1 << L)) > leaf:
        L += 1
    return L


def leaf_offsets(n, L):
    """Offsets (length 2^L + 1) of the leaves in leaf order: ceil(p/2) of a node's p
    points go left, floor(p/2) right, L times."""
    off = [0, int(n)]
    for _ in range(L):
        nxt = [0]
        for a, b in zip(off[:-1], off[1:]):
            mid = a + (b - a + 1) // 2
            nxt += [mid, b]
        off = nxt
    return np.asarray(off, dtype=np.int64)


def cluster_tree(F, leaf):
    """Return perm (int64, length n): the points in leaf order, left to right.

    Node rule: c = lowest coordinate whose population variance over the node
    is at least (1 - 1e-9) times the largest one; sort the node's points by
    (value of coordinate c, original index); lower ceil(p/2) points -> left child,
    the rest -> right child; stop on level `tree_depth(n, leaf)`.
    """
    F = np.asarray(F, dtype=np.float64)
    n = F.shape[0]
    L = tree_depth(n, leaf)
    out = []

    def split(idx, depth):
        if depth == L:
            out.append(idx)
            return
        sub = F[idx]
        var = ((sub - sub.mean(axis=0)) ** 2).mean(axis=0)
        c = int(np.flatnonzero(var >= var.max() * (1.0 - TIE))[0])
        order = np.lexsort((idx, sub[:, c]))     # primary key value, secondary original index
        idx = idx[order]
        half = (idx.size + 1) // 2
        split(idx[:half], depth + 1)
        split(idx[half:], depth + 1)

    split(np.arange(n, dtype=np.int64), 0)
    return np.concatenate(out)


QBITS = 38   # fixed-point bits of a feature value in the exact centre sums


def _dist2(sub, c):
    """Squared distances of the rows of `sub` to the point c, one feature after the
    other in index order, every product and sum rounded on its own."""
    d2 = np.zeros(sub.shape[0])
    for f in range(sub.shape[1]):
        diff = sub[:, f] - c[f]
        d2 = d2 + diff * diff
    return d2


def cluster_tree_2means(F, leaf, iters=2):
    """Data-driven cluster tree (the paper's clustering preprocess, Sec. 1.1 last
    paragraph / Sec. 1.2 first bullet: the points are grouped so that off-diagonal
    blocks of the kernel matrix get low rank).  Tree shape as in
    `cluster_tree`, but a node is split along the line between the two centres of a
    2-means pass over its points instead of along a coordinate axis.

    The rule is free of summation order, so that any implementation can reproduce
    the permutation exactly:
      * centres are means taken from EXACT integer sums of the features in fixed
        point (value * 2^k rounded to the nearest integer, 2^k chosen from the largest
        |feature| of the whole set so that |integer| <= 2^38), then
        ((float)sum / (float)count) / 2^k;
      * everything else is per point: squared distances and projections accumulated
        feature by feature in index order with every operation rounded on its own,
        compared or sorted across points, ties to the lowest original index.
    Node rule:  c = mean of the node;  a = the point farthest from c;  b = the point
    farthest from a;  centres (ca, cb) = (a, b);  `iters` times: points with
    dist2(., ca) <= dist2(., cb) form A, the others B; stop if one is empty;
    (ca, cb) = (mean A, mean B);  then sort the node by
    (sum_f (x_f - ca_f) (cb_f - ca_f), original index), lower ceil(p/2) -> left child.
    """
    F = np.asarray(F, dtype=np.float64)
    n, r = F.shape
    L = tree_depth(n, leaf)
    amax = float(np.abs(F).max()) if n else 0.0
    if not np.isfinite(amax):
        raise ValueError("non-finite feature")
    e = np.frexp(amax)[1] if amax > 0 else 0           # amax < 2^e
    scale = np.ldexp(1.0, QBITS - int(e))
    Q = np.rint(F * scale).astype(np.int64)

    def mean(rows):
        return (Q[rows].sum(axis=0).astype(np.float64) / float(rows.size)) / scale

    def farthest(idx, sub, c):
        d2 = _dist2(sub, c)
        cand = idx[d2 == d2.max()]
        return int(cand.min())                          # ties -> lowest original index

    out = []

    def split(idx, depth):
        if depth == L:
            out.append(idx)
            return
        sub = F[idx]
        a = farthest(idx, sub, mean(idx))
        b = farthest(idx, sub, F[a])
        ca, cb = F[a].copy(), F[b].copy()
        for _ in range(iters):
            inA = _dist2(sub, ca) <= _dist2(sub, cb)
            if inA.all() or not inA.any():
                break
            ca, cb = mean(idx[inA]), mean(idx[~inA])
        d = cb - ca
        p = np.zeros(idx.size)
        for f in range(r):
            p = p + (sub[:, f] - ca[f]) * d[f]
        idx = idx[np.lexsort((idx, p))]
        half = (idx.size + 1) // 2
        split(idx[:half], depth + 1)
        split(idx[half:], depth + 1)

    split(np.arange(n, dtype=np.int64), 0)
    return np.concatenate(out)
