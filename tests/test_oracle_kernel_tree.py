"""Pins for oracle.kernel and oracle.tree (CPU only)."""
import math

import numpy as np
import pytest
from scipy.spatial.distance import cdist

from oracle.kernel import gaussian_kernel
from oracle.tree import cluster_tree


def test_kernel_two_points_by_hand():
    # ||(1,2)-(4,6)||^2 = 25, h = 2.5 -> exp(-25/12.5) = exp(-2)
    K = gaussian_kernel(np.array([[1.0, 2.0]]), np.array([[4.0, 6.0]]), 2.5)
    assert K.shape == (1, 1)
    assert K[0, 0] == pytest.approx(math.exp(-2.0), rel=1e-15)


def test_kernel_diag_symmetry_and_library_distance():
    rng = np.random.default_rng(1)
    F = rng.standard_normal((70, 5))
    G = rng.standard_normal((33, 5))
    h = 0.7
    K = gaussian_kernel(F, F, h, block=16)
    assert np.all(np.diag(K) == 1.0)
    assert np.array_equal(K, K.T)
    Kfg = gaussian_kernel(F, G, h, block=7)
    ref = np.exp(-cdist(F, G, "sqeuclidean") / (2 * h * h))
    assert np.max(np.abs(Kfg - ref)) < 1e-15
    # transposed operands must transpose the result
    assert np.allclose(gaussian_kernel(G, F, h), Kfg.T, rtol=0, atol=1e-16)


def test_kernel_h_limits():
    rng = np.random.default_rng(2)
    F = rng.standard_normal((20, 3))
    assert np.allclose(gaussian_kernel(F, F, 1e9), 1.0, atol=1e-15)
    assert np.array_equal(gaussian_kernel(F, F, 1e-6), np.eye(20))


def test_tree_is_permutation_and_balanced():
    rng = np.random.default_rng(3)
    F = rng.standard_normal((512, 4))
    perm = cluster_tree(F, 32)
    assert perm.dtype == np.int64
    assert np.array_equal(np.sort(perm), np.arange(512))


def test_tree_one_dimensional_is_a_sort():
    rng = np.random.default_rng(4)
    F = rng.standard_normal((256, 1))
    perm = cluster_tree(F, 16)
    # on a line every bisection is on the same coordinate: the leaf order is the sorted order
    assert np.array_equal(perm, np.argsort(F[:, 0], kind="stable"))


def test_tree_top_split_uses_widest_coordinate_and_median():
    rng = np.random.default_rng(5)
    F = rng.standard_normal((128, 3))
    F[:, 1] *= 5.0                       # coordinate 1 has by far the largest variance
    perm = cluster_tree(F, 16)
    left, right = perm[:64], perm[64:]
    assert F[left, 1].max() <= F[right, 1].min()


def test_tree_ties_are_broken_by_index():
    # two identical binary columns and duplicates: ties -> lowest coordinate, then original index
    F = np.zeros((64, 2))
    F[32:, 0] = 1.0
    F[32:, 1] = 1.0
    perm = cluster_tree(F, 32)
    assert np.array_equal(perm, np.arange(64))


def test_tree_variances_equal_up_to_rounding_count_as_tied():
    # column 1 is a shuffled copy of column 0 scaled by 1 + 1e-12: its variance is larger, but only at the
    # level of a sum's rounding -> the lowest coordinate is taken; a relative excess of 1e-6 is a real difference
    rng = np.random.default_rng(6)
    x = rng.standard_normal(256)
    for scale, coord in ((1.0 + 1e-12, 0), (1.0 + 1e-6, 1)):
        F = np.stack([x, rng.permutation(x) * scale], axis=1)
        perm = cluster_tree(F, 128)
        left, right = perm[:128], perm[128:]
        assert F[left, coord].max() <= F[right, coord].min()
        other = 1 - coord
        assert F[left, other].max() > F[right, other].min()


def test_tree_rejects_bad_sizes():
    with pytest.raises(ValueError):
        cluster_tree(np.zeros((0, 2)), 32)
    with pytest.raises(ValueError):
        cluster_tree(np.zeros((96, 2)), 0)


# ---- data-driven cluster tree (2-means bisection) ----

def _clustered(n, r, k, seed, spread=3.0, std=0.3):
    """A mixture of k well-separated Gaussian clusters (the setting of the paper's Fig. 1: once the points are
    grouped, the off-diagonal blocks of the kernel matrix have fast-decaying singular values)."""
    g = np.random.default_rng(seed)
    centres = g.standard_normal((k, r)) * spread
    lab = g.integers(0, k, n)
    return centres[lab] + std * g.standard_normal((n, r)), lab


def _leaves(perm, leaf):
    return {frozenset(perm[i:i + leaf].tolist()) for i in range(0, perm.size, leaf)}


def test_2means_tree_is_a_permutation_and_sorts_in_one_dimension():
    from oracle.tree import cluster_tree_2means
    rng = np.random.default_rng(0)
    F = rng.standard_normal((256, 1))
    perm = cluster_tree_2means(F, 16)
    assert sorted(perm.tolist()) == list(range(256))
    # in one dimension every split is a median split of the values: leaves are runs of the sorted order
    order = np.argsort(F[:, 0], kind="stable")
    assert _leaves(perm, 16) == {frozenset(order[i:i + 16].tolist()) for i in range(0, 256, 16)}


def test_2means_tree_separates_two_clusters_at_the_root():
    from oracle.tree import cluster_tree_2means
    rng = np.random.default_rng(1)
    A = rng.standard_normal((128, 5)) * 0.2 + 4.0
    B = rng.standard_normal((128, 5)) * 0.2 - 4.0
    F = np.vstack([A, B])
    mix = rng.permutation(256)
    perm = cluster_tree_2means(F[mix], 32)
    halves = [set(mix[perm[:128]].tolist()), set(mix[perm[128:]].tolist())]
    assert set(range(128)) in halves and set(range(128, 256)) in halves


def test_2means_tree_does_not_depend_on_the_order_of_the_points():
    """The partition into leaves is a function of the point SET: exact fixed-point centre sums and per-point
    arithmetic leave no room for a summation order (ties aside, which continuous data does not have)."""
    from oracle.tree import cluster_tree_2means
    F, _ = _clustered(1024, 6, 8, 2)
    perm = cluster_tree_2means(F, 32)
    shuffle = np.random.default_rng(3).permutation(1024)
    perm_s = cluster_tree_2means(F[shuffle], 32)
    assert _leaves(perm, 32) == _leaves(shuffle[perm_s], 32)
    # leaves in the same left-to-right order, too
    same = [frozenset(shuffle[perm_s][i:i + 32].tolist()) for i in range(0, 1024, 32)]
    assert [frozenset(perm[i:i + 32].tolist()) for i in range(0, 1024, 32)] == same


def test_2means_tree_handles_identical_points_and_exact_ties():
    from oracle.tree import cluster_tree_2means
    F = np.zeros((64, 3))
    assert np.array_equal(cluster_tree_2means(F, 16), np.arange(64))      # all ties: original order
    F = np.repeat(np.array([[0.0, 0.0], [1.0, 0.0]]), 32, axis=0)          # two stacks of 32 identical points
    perm = cluster_tree_2means(F, 16)
    assert set(perm[:32].tolist()) in ({*range(32)}, {*range(32, 64)})


def test_2means_tree_lowers_the_compression_error_on_clustered_points():
    """What the clustering preprocess is for (Sec. 1.1 / Fig. 1): grouping the points lowers the ranks of the
    off-diagonal blocks.  With equal-size children a split cannot always follow a cluster boundary, so the effect on
    a single input is erratic (either tree can be the better one by orders of magnitude); over a family of
    clustered inputs the data-driven tree lowers the achieved error at equal ranks (geometric mean), and it wins
    clearly more often than it loses by a wide margin."""
    from oracle import hss
    from oracle.tree import cluster_tree_2means
    ratios = []
    for seed in range(8):
        g = np.random.default_rng(100 + seed)
        r = int(g.choice([4, 8, 12, 20, 32]))
        k = int(g.choice([8, 16, 32, 64]))
        h = float(np.sqrt(r) * 0.45)
        F, _ = _clustered(2048, r, k, seed)
        Om = np.random.default_rng(9).standard_normal((2048, 128))
        errs = []
        for perm in (cluster_tree(F, 64), cluster_tree_2means(F, 64, iters=2)):
            Fp = F[perm]
            H = hss.compress(Fp, h, 64, Om[perm], 1e-4, 1e-8, 64)
            K = gaussian_kernel(Fp, Fp, h)
            errs.append(np.linalg.norm(K - hss.densify(H)) / np.linalg.norm(K))
        ratios.append(errs[1] / errs[0])
    ratios = np.array(ratios)
    assert np.exp(np.log(ratios).mean()) < 0.9, ratios
    assert (ratios < 0.8).sum() > (ratios > 1.25).sum(), ratios
