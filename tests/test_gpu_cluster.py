"""The data-driven cluster tree (2-means bisection, option "clustering" = 1) on the GPU against the oracle's
cluster_tree_2means: the permutation must be IDENTICAL (the rule is free of summation order: exact fixed-point
centre sums, per-point arithmetic with every operation rounded on its own), on clustered inputs, on the
workloads' generators (binary columns: exact ties), on identical points, and at a full workload size."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import hss as ohss            # noqa: E402
from oracle.kernel import gaussian_kernel  # noqa: E402
from oracle.tree import cluster_tree, cluster_tree_2means      # noqa: E402
from paper_2108_04167_amd import binding, synth   # noqa: E402


def _dev(a):
    import torch
    return torch.tensor(np.ascontiguousarray(a), device="cuda:0")


def _clustered(n, r, k, seed, spread=3.0, std=0.3):
    g = np.random.default_rng(seed)
    centres = g.standard_normal((k, r)) * spread
    return centres[g.integers(0, k, n)] + std * g.standard_normal((n, r))


def _gpu_perm(F, leaf, h=1.0, iters=None, s=128):
    n = F.shape[0]
    y = np.where(np.arange(n) % 2 == 0, 1.0, -1.0)
    ctx = binding.Context()
    ctx.hss_set_i64("clustering", 1)
    if iters is not None:
        ctx.hss_set_i64("clustering_iterations", iters)
    ctx.hss_set_i64("sample_width", s)
    ctx.hss_compress(_dev(F), _dev(y), h, leaf, 1e-2)
    exp = ctx.hss_export()
    ctx.close()
    return exp["perm"]


CASES = {
    "clustered_r8": lambda: (_clustered(4096, 8, 16, 0), 64),
    "clustered_r20": lambda: (_clustered(8192, 20, 32, 1), 128),
    "clustered_r3": lambda: (_clustered(2048, 3, 8, 2, std=0.05), 32),
    "one_feature": lambda: (np.random.default_rng(3).standard_normal((1024, 1)), 16),
    "cfg1": lambda: (synth.make_workload(1).F, 64),
    "cfg2_cut": lambda: (synth.make_workload(2, n=16384).F, 128),
    "cfg3_cut_binary_columns": lambda: (synth.make_workload(3, n=16384).F, 256),
    "cfg4_cut": lambda: (synth.make_workload(4, n=8192).F, 256),
    "cfg5_cut_r90": lambda: (synth.make_workload(5, n=4096).F, 256),
    "identical_points": lambda: (np.repeat(np.array([[0.0, 1.0, 2.0], [5.0, 1.0, 2.0]]), 128, axis=0), 32),
    "all_zero": lambda: (np.zeros((256, 4)), 64),
    "binary_only": lambda: ((np.random.default_rng(4).random((2048, 12)) < 0.3).astype(np.float64), 64),
    "large_values": lambda: (np.random.default_rng(5).standard_normal((1024, 5)) * 1e6 + 3e7, 64),
}


@pytest.mark.parametrize("name", list(CASES))
def test_2means_tree_is_the_oracles(name):
    F, leaf = CASES[name]()
    perm = _gpu_perm(F, leaf)
    ref = cluster_tree_2means(F, leaf)
    assert np.array_equal(perm, ref), int((perm != ref).sum())


@pytest.mark.parametrize("iters", [0, 1, 5])
def test_2means_tree_iteration_counts(iters):
    F = _clustered(4096, 6, 12, 7)
    assert np.array_equal(_gpu_perm(F, 64, iters=iters), cluster_tree_2means(F, 64, iters=iters))


def test_2means_tree_full_size_workload_2():
    w = synth.make_workload(2)
    perm = _gpu_perm(w.F, w.leaf, h=w.h, s=w.s)
    assert np.array_equal(perm, cluster_tree_2means(w.F, w.leaf))


def test_2means_tree_on_clustered_points_through_the_whole_path():
    """Compression, solve and training run on the data-driven tree like on the default one; the achieved error on
    a clustered input is what the oracle gets with the same tree and sample, and here below the coordinate tree's."""
    from gpu_helpers import oracle_hss_from_export
    n, r, h, leaf = 4096, 12, 1.5, 64
    F = _clustered(n, r, 32, 5)
    y = np.where(F[:, 0] + F[:, 1] >= 0, 1.0, -1.0)
    Om = np.random.default_rng(9).standard_normal((n, 128))
    errs = {}
    for rule in (0, 1):
        ctx = binding.Context()
        ctx.hss_set_i64("clustering", rule)
        ctx.hss_compress(_dev(F), _dev(y), h, leaf, 1e-3, _dev(Om))
        exp = ctx.hss_export()
        perm = exp["perm"]
        assert np.array_equal(perm, cluster_tree_2means(F, leaf) if rule else cluster_tree(F, leaf))
        Fp = F[perm]
        K = gaussian_kernel(Fp, Fp, h)
        err = np.linalg.norm(K - ohss.densify(oracle_hss_from_export(exp, with_shift=False))) / np.linalg.norm(K)
        Ho = ohss.compress(Fp, h, leaf, Om[perm], 1e-4, 1e-8, 64)
        err_or = np.linalg.norm(K - ohss.densify(Ho)) / np.linalg.norm(K)
        assert err <= max(1e-3, 1.5 * err_or)
        errs[rule] = err
        out = ctx.admm_svm_train(1.0, 1.0, 50)
        z = out["z"].cpu().numpy()
        assert z.min() >= 0.0 and z.max() <= 1.0 and np.isfinite(out["bias"])
        ctx.close()
    assert errs[1] < errs[0], errs


def test_clustering_option_errors():
    ctx = binding.Context()
    with pytest.raises(binding.HssError):
        ctx.hss_set_i64("clustering", 2)
    with pytest.raises(binding.HssError):
        ctx.hss_set_i64("clustering_iterations", -1)
    ctx.hss_set_i64("clustering", 1)
    F = np.random.default_rng(0).standard_normal((256, 3))
    F[17, 1] = np.inf
    with pytest.raises(binding.HssError) as e:
        ctx.hss_compress(_dev(F), _dev(np.ones(256)), 1.0, 64, 1e-2)
    assert e.value.code == binding.HSS_EINVAL
    ctx.close()
