"""Pins for the oracle on point counts that are not leaf * 2^L (CPU only): the shape of the tree against its closed
form, the trees on inputs whose answer is known, and compression / mat-vec / ULV / ADMM / neighbour-based
construction against dense linear algebra, as for the regular sizes."""
import numpy as np
import pytest

from oracle import admm, ann, hss, ulv
from oracle.kernel import gaussian_kernel
from oracle.tree import cluster_tree, cluster_tree_2means, leaf_offsets, tree_depth


def _bitrev(t, bits):
    return int(format(t, "0%db" % bits)[::-1], 2) if bits else 0


@pytest.mark.parametrize("n,leaf", [(1, 16), (15, 16), (16, 16), (17, 16), (33, 16), (1000, 64), (1023, 64), (1025, 64),
                                    (2048, 64), (32561, 128), (49990, 256), (100, 32), (96, 32)])
def test_tree_shape_closed_form(n, leaf):
    """Depth: the smallest L with ceil(n / 2^L) <= leaf.  Sizes: floor or ceil of n / 2^L, and (ceil goes left on every
    level) leaf t is a large one exactly when the bit reversal of t is below n mod 2^L."""
    L = tree_depth(n, leaf)
    assert -(-n // 2 ** L) <= leaf and (L == 0 or -(-n // 2 ** (L - 1)) > leaf)
    off = leaf_offsets(n, L)
    assert off[0] == 0 and off[-1] == n and off.size == 2 ** L + 1
    sizes = np.diff(off)
    q, rem = divmod(n, 2 ** L)
    expect = np.array([q + (1 if _bitrev(t, L) < rem else 0) for t in range(2 ** L)])
    assert np.array_equal(sizes, expect)
    if n == leaf * 2 ** L:
        assert np.all(sizes == leaf)
    # the offsets of a coarser level are every other offset of the next one
    for l in range(L):
        assert np.array_equal(leaf_offsets(n, l), leaf_offsets(n, l + 1)[::2])


@pytest.mark.parametrize("tree", [cluster_tree, cluster_tree_2means])
@pytest.mark.parametrize("n,leaf", [(1000, 64), (777, 32), (33, 16), (15, 16)])
def test_one_dimensional_points_come_out_sorted(tree, n, leaf):
    """With one feature every split is along it (for the 2-means rule: along the line between two centres on it,
    in either direction), so the leaf order is the sorted order or its mirror image inside every node -- and every
    leaf holds a contiguous run of the sorted values."""
    rng = np.random.default_rng(n)
    F = rng.standard_normal((n, 1))
    perm = tree(F, leaf)
    assert np.array_equal(np.sort(perm), np.arange(n))
    off = leaf_offsets(n, tree_depth(n, leaf))
    rank = np.empty(n, dtype=np.int64)
    rank[np.argsort(F[:, 0], kind="stable")] = np.arange(n)
    for a, b in zip(off[:-1], off[1:]):
        rk = np.sort(rank[perm[a:b]])
        assert np.array_equal(rk, np.arange(rk[0], rk[0] + b - a))
    if tree is cluster_tree and off.size > 2:                 # the last split sorted every pair of sibling leaves
        assert np.array_equal(perm, np.argsort(F[:, 0], kind="stable"))


def test_ragged_split_is_ceil_left_along_the_widest_coordinate():
    rng = np.random.default_rng(3)
    n, leaf = 301, 64
    F = rng.standard_normal((n, 3)) * np.array([1.0, 5.0, 2.0])
    perm = cluster_tree(F, leaf)
    L = tree_depth(n, leaf)
    assert L == 3
    left, right = perm[:151], perm[151:]                      # ceil(301 / 2) go left
    assert F[left, 1].max() <= F[right, 1].min()
    sizes = np.diff(leaf_offsets(n, L))
    assert sizes.max() - sizes.min() == 1 and sizes.sum() == n


def _compress(n, r, h, leaf, s, rel, seed=0, kmax=None):
    rng = np.random.default_rng(seed)
    F = rng.standard_normal((n, r))
    Fp = F[cluster_tree(F, leaf)]
    Om = rng.standard_normal((n, s))
    return Fp, Om, hss.compress(Fp, h, leaf, Om, rel, 0.0, kmax), rng


@pytest.mark.parametrize("n,r,h,leaf,s,tol", [(1000, 2, 1.5, 32, 128, 1e-4), (523, 3, 2.0, 64, 128, 1e-6),
                                              (250, 2, 0.8, 16, 64, 1e-3)])
def test_ragged_reconstruction_error_within_tolerance(n, r, h, leaf, s, tol):
    Fp, Om, H, _ = _compress(n, r, h, leaf, s, tol / 10.0, kmax=s - 10)
    assert len({d.shape[0] for d in H.D}) == 2                # really ragged
    K = gaussian_kernel(Fp, Fp, h)
    Kt = hss.densify(H)
    assert np.array_equal(Kt, Kt.T)
    err = np.linalg.norm(K - Kt) / np.linalg.norm(K)
    assert err <= tol, (err, H.ranks().max())
    assert H.ranks().max() < s - 10
    for a, b in zip(H.loff[:-1], H.loff[1:]):                 # diagonal blocks are entries of K itself
        assert np.array_equal(Kt[a:b, a:b], K[a:b, a:b])


def test_ragged_exact_when_sample_is_wide_and_tolerance_tiny():
    n, leaf, h = 250, 32, 1.0
    Fp, Om, H, _ = _compress(n, 3, h, leaf, n, 1e-15)
    K = gaussian_kernel(Fp, Fp, h)
    assert np.linalg.norm(K - hss.densify(H)) <= 1e-10 * np.linalg.norm(K)


def test_ragged_matvec_equals_dense_product():
    for (n, leaf, tol) in [(500, 32, 1e-3), (250, 64, 1e-1), (63, 64, 1e-3), (65, 64, 1e-3)]:
        Fp, Om, H, rng = _compress(n, 3, 1.2, leaf, min(n, 96), tol)
        x = rng.standard_normal(n)
        ref = hss.densify(H) @ x
        assert np.linalg.norm(hss.matvec(H, x) - ref) <= 1e-12 * np.linalg.norm(ref)


@pytest.mark.parametrize("n,r,h,leaf,s,tol,beta", [
    (1000, 3, 1.5, 32, 96, 1e-5, 1.0),
    (500, 4, 1.0, 64, 64, 1e-1, 0.5),
    (250, 2, 2.0, 16, 64, 1e-8, 2.0),
    (500, 6, 0.7, 32, 128, 1e-12, 1.0),   # leaves are full rank: nothing eliminated there
    (37, 2, 1.0, 16, 32, 1e-6, 1.0),
])
def test_ragged_ulv_solve_equals_dense_solve(n, r, h, leaf, s, tol, beta):
    Fp, Om, H, rng = _compress(n, r, h, leaf, s, tol, kmax=s - 8)
    A = hss.densify(H) + beta * np.eye(n)
    Fz = ulv.ulv_factor(H, beta)
    b = rng.standard_normal(n)
    ref = np.linalg.solve(A, b)
    assert np.linalg.norm(ulv.ulv_solve(Fz, b) - ref) <= 1e-10 * np.linalg.norm(ref)
    B = rng.standard_normal((n, 3))
    X = ulv.ulv_solve(Fz, B)
    assert np.linalg.norm(X - np.linalg.solve(A, B)) <= 1e-10 * np.linalg.norm(X)


def test_ragged_admm_through_ulv_equals_admm_through_dense_solve():
    n, leaf = 333, 32
    Fp, Om, H, rng = _compress(n, 3, 1.0, leaf, 96, 1e-4, kmax=80)
    y = np.where(rng.standard_normal(n) > 0, 1.0, -1.0)
    beta, C = 1.0, 1.0
    Fz = ulv.ulv_factor(H, beta)
    A = hss.densify(H) + beta * np.eye(n)
    r1 = admm.admm(lambda t: ulv.ulv_solve(Fz, t), y, C, beta, 40)
    r2 = admm.admm(lambda t: np.linalg.solve(A, t), y, C, beta, 40)
    for key in ("x", "z", "mu"):
        assert np.linalg.norm(r1[key] - r2[key]) <= 1e-9 * max(1.0, np.linalg.norm(r2[key]))


def test_ragged_adaptive_equals_fixed_width_when_it_starts_at_the_full_width():
    n, leaf, s = 500, 32, 128
    rng = np.random.default_rng(5)
    F = rng.standard_normal((n, 3))
    Fp = F[cluster_tree(F, leaf)]
    Om = rng.standard_normal((n, s))
    H1 = hss.compress(Fp, 1.5, leaf, Om, 1e-5, 0.0, s // 2)
    H2, info = hss.compress_adaptive(Fp, 1.5, leaf, Om, 1e-5, 0.0)
    assert info["width"] == s
    assert np.array_equal(hss.densify(H1), hss.densify(H2))


def test_ragged_neighbour_based_construction():
    """Every outside column a candidate (k = n - 1 neighbours, width n): the sample block is the whole off-diagonal
    block row, so a tiny tolerance reproduces K; and on a local kernel a modest list meets the tolerance."""
    n, leaf, h = 250, 32, 1.0
    rng = np.random.default_rng(2)
    F = rng.standard_normal((n, 3))
    Fp = F[cluster_tree(F, leaf)]
    idx, dist = ann.knn_exact(Fp, n - 1)
    H, info = ann.compress_ann(Fp, h, leaf, idx, dist, n, 1e-14, 0.0, n)
    K = gaussian_kernel(Fp, Fp, h)
    assert np.linalg.norm(K - hss.densify(H)) <= 1e-9 * np.linalg.norm(K)
    n, leaf, h, k, s, tol = 1500, 64, 0.25, 96, 128, 1e-3
    F = rng.uniform(-2.0, 2.0, size=(n, 2))
    Fp = F[cluster_tree(F, leaf)]
    L = tree_depth(n, leaf)
    cells = leaf_offsets(n, L - 2)                       # cells of four leaves each: 187 or 188 points
    idx, dist = ann.ann_projection_trees(Fp, k, cell=int(np.diff(cells).max()), trees=4, seed=1, first_cells=list(cells))
    assert (idx >= 0).all()
    H, info = ann.compress_ann(Fp, h, leaf, idx, dist, s, tol / 10.0, 1e-10, s - 10)
    K = gaussian_kernel(Fp, Fp, h)
    assert np.linalg.norm(K - hss.densify(H)) <= 2.0 * tol * np.linalg.norm(K)


def test_ragged_projection_tree_cells_have_the_shape_of_the_cluster_tree():
    n = 1500
    rng = np.random.default_rng(0)
    F = rng.standard_normal((n, 4))
    dirs = {}
    def direction(l, node):
        return dirs.setdefault((l, node), rng.standard_normal(4))
    lc = 3
    cell = -(-n // 2 ** lc)
    cells = ann.cells_of_projection_tree(F, cell, direction)
    assert [c.size for c in cells] == list(np.diff(leaf_offsets(n, lc)))
    assert np.array_equal(np.sort(np.concatenate(cells)), np.arange(n))
    # the root split: lower ceil(n/2) projections on the first direction go left
    p = F @ dirs[(0, 0)]
    left = np.concatenate(cells[:4])
    right = np.concatenate(cells[4:])
    assert left.size == 750 and p[left].max() <= p[right].min()
