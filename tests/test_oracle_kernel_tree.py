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
        cluster_tree(np.zeros((100, 2)), 32)
    with pytest.raises(ValueError):
        cluster_tree(np.zeros((96, 2)), 32)
