"""Cluster tree by balanced coordinate bisection (oracle; test infrastructure).

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


def cluster_tree(F, leaf):
    """Return perm (int64, length n): the points in leaf order, left to right.

    Node rule: c = lowest coordinate whose population variance over the node
    is at least (1 - 1e-9) times the largest one; sort the node's points by
    (value of coordinate c, original index); lower half -> left child, upper
    half -> right child; stop when the node holds `leaf` points.
    n must equal leaf * 2^L.
    """
    F = np.asarray(F, dtype=np.float64)
    n = F.shape[0]
    nl = n // leaf
    if nl * leaf != n or nl & (nl - 1):
        raise ValueError("n must be leaf * 2^L")
    out = []

    def split(idx):
        if idx.size == leaf:
            out.append(idx)
            return
        sub = F[idx]
        var = ((sub - sub.mean(axis=0)) ** 2).mean(axis=0)
        c = int(np.flatnonzero(var >= var.max() * (1.0 - TIE))[0])
        order = np.lexsort((idx, sub[:, c]))     # primary key value, secondary original index
        idx = idx[order]
        half = idx.size // 2
        split(idx[:half])
        split(idx[half:])

    split(np.arange(n, dtype=np.int64))
    return np.concatenate(out)
