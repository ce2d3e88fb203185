"""Pins for oracle.ann (CPU only): nearest-neighbour search against its definition, and the neighbour-based
HSS construction against the dense kernel."""
import numpy as np
import pytest

from oracle import ann, hss
from oracle.kernel import gaussian_kernel
from oracle.tree import cluster_tree


def _points(n, r, seed):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((n, r)), rng


def test_knn_exact_is_the_sorted_distance_list():
    F, _ = _points(200, 3, 0)
    idx, dist = ann.knn_exact(F, 7, block=64)
    for i in range(200):
        d = [(float(((F[i] - F[j]) ** 2).sum()), j) for j in range(200) if j != i]
        d.sort()
        assert [j for _, j in d[:7]] == idx[i].tolist()
        assert np.allclose([v for v, _ in d[:7]], dist[i], rtol=1e-13, atol=0)
    # more neighbours asked for than there are other points: the tail is padded
    idx, dist = ann.knn_exact(F[:5], 8)
    assert (idx[:, 4:] == -1).all() and np.isinf(dist[:, 4:]).all() and (idx[:, :4] >= 0).all()


def _check_lists(F, idx, dist):
    n, k = idx.shape
    for i in range(n):
        ii = idx[i][idx[i] >= 0]
        assert i not in ii and len(set(ii.tolist())) == ii.size              # never itself, no duplicates
        d = ((F[ii] - F[i]) ** 2).sum(axis=1)
        assert np.allclose(d, dist[i][:ii.size], rtol=1e-12, atol=1e-300)     # the distances are the true ones
        key = list(zip(dist[i][:ii.size].tolist(), ii.tolist()))
        assert key == sorted(key)                                              # ascending by (distance, index)


def test_projection_tree_search_is_valid_exact_in_cells_and_has_recall():
    F, _ = _points(2048, 3, 1)
    k = 16
    ex_i, ex_d = ann.knn_exact(F, k)
    # one tree whose single cell holds everything: the definition
    i1, d1 = ann.ann_projection_trees(F, k, cell=2048, trees=1)
    assert np.array_equal(i1, ex_i) and np.array_equal(d1, ex_d)
    prev = 0.0
    for trees in (1, 3, 6):
        idx, dist = ann.ann_projection_trees(F, k, cell=256, trees=trees, seed=5)
        _check_lists(F, idx, dist)
        # at least as good as the exact search inside the point's own contiguous cell (tree 0)
        for c0 in range(0, 2048, 256):
            cell = np.arange(c0, c0 + 256)
            ci, cd = ann.knn_in_cells(F, [cell], k)
            assert (dist[cell] <= cd[cell] + 0.0).all()
        recall = np.mean([len(set(idx[i]) & set(ex_i[i])) / k for i in range(2048)])
        assert recall >= prev - 1e-12                                          # more trees never lose neighbours
        prev = recall
    assert prev > 0.85


def test_merge_keeps_the_closest_distinct_entries():
    ia = np.array([[3, 5, -1]])
    da = np.array([[0.1, 0.4, np.inf]])
    ib = np.array([[5, 7, 9]])
    db = np.array([[0.4, 0.2, 0.3]])
    oi, od = ann._merge_lists(ia, da, ib, db, 3)
    assert oi.tolist() == [[3, 7, 9]] and od.tolist() == [[0.1, 0.2, 0.3]]


def test_select_columns_takes_the_closest_outside_candidates():
    nbr_idx = np.array([[1, 9, 4], [0, 8, 9], [7, 3, -1]])
    nbr_dist = np.array([[0.1, 0.9, 0.5], [0.1, 0.3, 0.2], [0.05, 0.6, np.inf]])
    # node = indices [0, 3): candidates 9 (0.9 and 0.2 -> 0.2), 4 (0.5), 8 (0.3), 7 (0.05), 3 (0.6)
    cols = ann.select_columns(np.array([0, 1, 2]), nbr_idx, nbr_dist, 0, 3, 4)
    assert cols.tolist() == [7, 9, 8, 4]
    assert ann.select_columns(np.array([0]), nbr_idx, nbr_dist, 0, 10, 4).size == 0      # everything inside


def test_neighbour_based_construction_is_exact_when_every_outside_column_is_a_candidate():
    n, leaf, h = 256, 32, 1.0
    F, _ = _points(n, 3, 2)
    Fp = F[cluster_tree(F, leaf)]
    idx, dist = ann.knn_exact(Fp, n - 1)
    H, info = ann.compress_ann(Fp, h, leaf, idx, dist, n, 1e-14)
    K = gaussian_kernel(Fp, Fp, h)
    Kt = hss.densify(H)
    assert np.array_equal(Kt, Kt.T)
    assert np.linalg.norm(K - Kt) <= 1e-10 * np.linalg.norm(K)
    assert info["columns"][H.first_leaf()] == n - leaf         # a leaf's sample block is its whole off-diagonal block row
    for t in range(1, H.nnodes):
        assert np.array_equal(H.U[t][H.J[t]], np.eye(H.rank(t)))


@pytest.mark.parametrize("n,r,h,leaf,k,s,tol", [(2048, 2, 0.25, 64, 96, 128, 1e-3), (1024, 3, 0.5, 32, 64, 128, 1e-2)])
def test_neighbour_based_construction_meets_the_tolerance_on_a_local_kernel(n, r, h, leaf, k, s, tol):
    """A kernel that is narrow against the extent of the data: the entries that matter in an off-diagonal
    block row are those of the nearest outside points, so a few dozen neighbours per point carry the block.
    (A neighbour sample has no probabilistic error bound as a random one has; the achieved error is asserted within
    twice the requested tolerance.)"""
    rng = np.random.default_rng(4)
    F = rng.uniform(-2.0, 2.0, size=(n, r))
    Fp = F[cluster_tree(F, leaf)]
    idx, dist = ann.ann_projection_trees(Fp, k, cell=256, trees=4, seed=1)
    H, info = ann.compress_ann(Fp, h, leaf, idx, dist, s, tol / 10.0, 1e-10, s - 10)
    K = gaussian_kernel(Fp, Fp, h)
    err = np.linalg.norm(K - hss.densify(H)) / np.linalg.norm(K)
    assert err <= 2.0 * tol, err
    assert H.ranks().max() < s - 10
    for i in range(n // leaf):
        blk = slice(i * leaf, (i + 1) * leaf)
        assert np.array_equal(hss.densify(H)[blk, blk], K[blk, blk])


def test_neighbour_based_construction_is_as_good_as_random_sampling_on_a_saturated_workload():
    """On the workloads of this build (ranks at the cap) the neighbour-based sample gives an approximation that is
    no worse than the random sample of the same width and rank cap -- without the O(n^2) product K Omega."""
    from paper_2108_04167_amd import synth
    w = synth.make_workload(3, n=2048, leaf=64, s=128)
    Fp = w.F[cluster_tree(w.F, w.leaf)]
    K = gaussian_kernel(Fp, Fp, w.h)
    Hr = hss.compress(Fp, w.h, w.leaf, np.random.default_rng(0).standard_normal((2048, 128)), 1e-4, 1e-8, 64)
    idx, dist = ann.ann_projection_trees(Fp, 64, cell=256, trees=3, seed=0)
    Ha, _ = ann.compress_ann(Fp, w.h, w.leaf, idx, dist, 128, 1e-4, 1e-8, 64)
    er = np.linalg.norm(K - hss.densify(Hr)) / np.linalg.norm(K)
    ea = np.linalg.norm(K - hss.densify(Ha)) / np.linalg.norm(K)
    assert ea <= 1.1 * er, (ea, er)
