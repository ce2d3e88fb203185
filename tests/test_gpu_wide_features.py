"""More features than the fused kernels hold in LDS (r above 112 after padding, up to 384; GPU only).  The kernel
products then go through row stripes of the kernel matrix in HBM (batched GEMM, elementwise exp, batched GEMM); the
trees, the neighbour search and the leaf / coupling blocks take any feature count.  Checked against the oracle as for
the narrow data: S = K Omega, both trees and the neighbour lists bit for bit, compression quality, the path on the
exported matrix, decision values, the error estimate against the dense definition."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import admm as oadmm          # noqa: E402
from oracle import ann as oann            # noqa: E402
from oracle import hss as ohss            # noqa: E402
from oracle import ulv as oulv            # noqa: E402
from oracle.kernel import gaussian_kernel  # noqa: E402
from oracle.tree import cluster_tree, cluster_tree_2means, leaf_offsets, tree_depth      # noqa: E402
from paper_2108_04167_amd import binding   # noqa: E402


def _dev(a):
    import torch
    return torch.tensor(np.ascontiguousarray(a), device="cuda:0")


def _rel(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)


def _data(n, r, seed, binary=False):
    """Points with a few informative directions and many weak ones (the kernel stays compressible), optionally sparse
    binary columns as in the paper's wide data sets (exact ties in the trees)."""
    g = np.random.default_rng(seed)
    F = 0.15 * g.standard_normal((n, r))
    F[:, :4] += g.standard_normal((n, 4))
    if binary:
        F[:, 8:] = (g.random((n, r - 8)) < 0.05).astype(np.float64)
    y = np.where(F[:, 0] * F[:, 1] + 0.3 * g.standard_normal(n) > 0, 1.0, -1.0)
    return F, y, g


@pytest.mark.parametrize("n,r", [(1000, 113), (777, 123), (2048, 300), (1500, 384)])
def test_wide_sample_product(n, r):
    F, y, g = _data(n, r, n + r)
    Om = g.standard_normal((n, 130))
    h = 0.8 * np.sqrt(r) * 0.3
    ctx = binding.Context()
    S = ctx.hss_kernel_sample(_dev(F), h, _dev(Om)).cpu().numpy()
    ref = gaussian_kernel(F, F, h) @ Om
    assert np.abs(S - ref).max() <= 1e-12 * np.abs(ref).max()
    ctx.close()


@pytest.mark.parametrize("n,r,leaf,s,binary,clustering", [(3001, 123, 128, 256, True, 0), (2048, 300, 64, 128, False, 1),
                                                          (1234, 254, 64, 128, True, 1)])
def test_wide_features_through_the_whole_path(n, r, leaf, s, binary, clustering):
    from gpu_helpers import oracle_hss_from_export
    F, y, g = _data(n, r, 7 * n + r, binary)
    G = F[g.integers(0, n, 300)] + 0.1 * g.standard_normal((300, r))
    Om = g.standard_normal((n, s))
    h, tol, beta, C = 2.0, 1e-3, 1.0, 1.0
    ctx = binding.Context()
    ctx.hss_set_i64("clustering", clustering)
    rc = ctx.hss_compress(_dev(F), _dev(y), h, leaf, tol, _dev(Om))
    exp = ctx.hss_export()
    perm = exp["perm"]
    assert np.array_equal(perm, cluster_tree_2means(F, leaf, 2) if clustering else cluster_tree(F, leaf))
    st = ctx.hss_stats()
    K = gaussian_kernel(F[perm], F[perm], h)
    H0 = oracle_hss_from_export(exp, with_shift=False)
    Kt = ohss.densify(H0)
    for a, b in zip(H0.loff[:-1], H0.loff[1:]):
        assert np.abs(Kt[a:b, a:b] - K[a:b, a:b]).max() <= 1e-13
    err = np.linalg.norm(K - Kt) / np.linalg.norm(K)
    Ho = ohss.compress(F[perm], h, leaf, Om[perm], tol / 10.0, 1e-8, st["rank_cap"])
    err_o = np.linalg.norm(K - ohss.densify(Ho)) / np.linalg.norm(K)
    print(f"[wide n={n} r={r}] err {err:.2e} oracle {err_o:.2e} rank max {exp['ranks'].max()} rc {rc}")
    assert err <= max(1.5 * err_o, tol), (err, err_o)
    nprobe, seed = 5, 3
    est = ctx.hss_error_estimate(nprobe, seed)
    assert 0.2 * err <= est <= 5.0 * err + 1e-12
    H = oracle_hss_from_export(exp)
    v = g.standard_normal(n)
    mv = ctx.hss_matvec(_dev(v)).cpu().numpy()
    mref = np.empty(n)
    mref[perm] = ohss.matvec(H, v[perm])
    assert _rel(mv, mref) <= 1e-12
    ctx.hss_ulv_factor(beta)
    x = _dev(v)
    ctx.hss_ulv_solve(x)
    Fz = oulv.ulv_factor(H, beta)
    xref = np.empty(n)
    xref[perm] = oulv.ulv_solve(Fz, v[perm])
    assert _rel(x.cpu().numpy(), xref) <= 1e-10
    out = ctx.admm_svm_train(C, beta, 20)
    oref = oadmm.admm(lambda t: oulv.ulv_solve(Fz, t), y[perm], C, beta, 20)
    for key in ("x", "z", "mu"):
        assert _rel(out[key].cpu().numpy()[perm], oref[key]) <= 1e-6, key
    z = out["z"].cpu().numpy()
    dec = ctx.svm_decision(_dev(G), out["z"], out["bias"]).cpu().numpy()
    dref = oadmm.decision(F, y, z, out["bias"], G, h)
    assert np.abs(dec - dref).max() <= 1e-10 * max(1.0, np.abs(dref).max())
    ctx.close()


@pytest.mark.parametrize("n,r,leaf,k,trees", [(2048, 123, 64, 32, 3), (1500, 300, 64, 64, 2)])
def test_wide_features_neighbour_based(n, r, leaf, k, trees):
    from gpu_helpers import oracle_hss_from_export
    from test_gpu_ann import _library_directions
    F, y, g = _data(n, r, 3 * n + r, binary=(r == 123))
    h, tol, s, seed = 2.0, 1e-2, 128, 4
    ctx = binding.Context()
    ctx.hss_set_i64("sampling", 1)
    ctx.hss_set_i64("sample_width", s)
    for key, v in dict(ann_neighbours=k, ann_cell=256, ann_trees=trees, seed=seed).items():
        ctx.hss_set_i64(key, v)
    ctx.hss_compress(_dev(F), _dev(y), h, leaf, tol)
    idx, dist = ctx.hss_export_neighbours()
    exp = ctx.hss_export()
    perm = exp["perm"]
    L = tree_depth(n, leaf)
    lc = L
    while lc > 0 and (n >> lc) < 256:
        lc -= 1
    cells = leaf_offsets(n, lc)
    ri, rd = oann.ann_projection_trees(F[perm], k, int(np.diff(cells).max()), trees, directions=_library_directions(seed, r),
                                       first_cells=list(cells))
    assert np.array_equal(idx, ri) and np.array_equal(dist, rd)
    K = gaussian_kernel(F[perm], F[perm], h)
    err = np.linalg.norm(K - ohss.densify(oracle_hss_from_export(exp, with_shift=False))) / np.linalg.norm(K)
    Ho, _ = oann.compress_ann(F[perm], h, leaf, idx.astype(np.int64), dist, s, tol / 10.0, 1e-8, ctx.hss_stats()["rank_cap"])
    err_o = np.linalg.norm(K - ohss.densify(Ho)) / np.linalg.norm(K)
    print(f"[wide ann n={n} r={r}] err {err:.2e} oracle {err_o:.2e}")
    assert err <= max(2.0 * err_o, tol), (err, err_o)
    ctx.close()


def test_wide_features_adaptive_width():
    """Adaptive sample width over the stripe path: the column windows of Omega (offset, leading dimension of the
    whole matrix) give the same widths, redone nodes, ranks and error as the oracle's adaptive compression."""
    from gpu_helpers import oracle_hss_from_export
    n, r, leaf, s, h, tol = 1500, 200, 64, 384, 2.0, 1e-3
    F, y, g = _data(n, r, 11)
    Om = g.standard_normal((n, s))
    ctx = binding.Context()
    ctx.hss_set_i64("adaptive_start", 128)
    ctx.hss_compress(_dev(F), _dev(y), h, leaf, tol, _dev(Om))
    st = ctx.hss_stats()
    exp = ctx.hss_export()
    perm = exp["perm"]
    assert np.array_equal(perm, cluster_tree(F, leaf))
    K = gaussian_kernel(F[perm], F[perm], h)
    err = np.linalg.norm(K - ohss.densify(oracle_hss_from_export(exp, with_shift=False))) / np.linalg.norm(K)
    Ho, info = ohss.compress_adaptive(F[perm], h, leaf, Om[perm], tol / 10.0, 1e-8, s0=128, step=128)
    err_o = np.linalg.norm(K - ohss.densify(Ho)) / np.linalg.norm(K)
    assert st["sample_width_used"] == info["width"] and st["nodes_redone"] == info["redone"]
    assert np.array_equal(exp["ranks"], Ho.ranks())
    assert abs(err - err_o) <= 1e-9 * err_o
    ctx.close()


def test_feature_limit():
    ctx = binding.Context()
    F = np.zeros((256, 385))
    with pytest.raises(binding.HssError) as e:
        ctx.hss_compress(_dev(F), _dev(np.ones(256)), 1.0, 64, 1e-2)
    assert e.value.code == binding.HSS_EUNSUPPORTED
    ctx.close()
