"""The limits of the library's shapes (GPU only): feature counts 1, 28/29 (a padding boundary) and 96 (more features
in test_gpu_wide_features.py), leaf sizes 16 and 1024 (the maximum; smaller leaves in test_gpu_ragged.py), sample width 512
with the rank cap at its maximum 512 (node sizes up to 1024, the solve kernel's widest block), and odd ranks
(scalar-load kernels).  Each case checks
S = K Omega, the mat-vec, the ULV solve and a short ADMM run against the oracle on the exported matrix."""
import copy

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import admm as oadmm          # noqa: E402
from oracle import hss as ohss            # noqa: E402
from oracle import ulv as oulv            # noqa: E402
from oracle.kernel import gaussian_kernel  # noqa: E402
from oracle.tree import cluster_tree      # noqa: E402
from paper_2108_04167_amd import binding, synth   # noqa: E402


def _dev(a):
    import torch
    return torch.tensor(np.ascontiguousarray(a), device="cuda:0")


def _rel(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)


def _with_features(w, r):
    """The workload with r feature columns: a prefix of its own, or its columns followed by fresh normal ones."""
    w = copy.copy(w)
    have = w.F.shape[1]
    if r <= have:
        w.F, w.F_test = np.ascontiguousarray(w.F[:, :r]), np.ascontiguousarray(w.F_test[:, :r])
    else:
        g = np.random.default_rng(1234)
        w.F = np.ascontiguousarray(np.hstack([w.F, g.standard_normal((w.F.shape[0], r - have))]))
        w.F_test = np.ascontiguousarray(np.hstack([w.F_test, g.standard_normal((w.F_test.shape[0], r - have))]))
    return w


# name -> (cfg, n, leaf, s, r or None, h or None, options)
EDGES = {
    "one_feature": (1, 1024, 64, 128, 1, 0.5, {}),
    "r28": (3, 1024, 64, 128, 28, None, {}),
    "r29": (3, 1024, 64, 128, 29, None, {}),
    "r96_max": (5, 1024, 128, 256, 96, None, {}),
    "leaf16_min": (1, 512, 16, 128, None, None, {}),
    "leaf1024_max": (4, 4096, 1024, 512, None, None, {}),
    "rank_cap_512_max": (3, 4096, 512, 512, None, None, {"oversample": 0}),       # nodes of 1024 rows
    "odd_ranks": (1, 1024, 64, 128, None, 6.0, {"max_rank": 37}),
}


@pytest.mark.parametrize("name", list(EDGES))
def test_edge_shape(name):
    from gpu_helpers import oracle_hss_from_export
    cfg, n, leaf, s, r, h, opts = EDGES[name]
    w = synth.make_workload(cfg, n=n, leaf=leaf, s=s)
    if r is not None:
        w = _with_features(w, r)
    if h is not None:
        w.h = h
    ctx = binding.Context()
    for k, v in opts.items():
        ctx.hss_set_i64(k, v)
    F, y, Om = _dev(w.F), _dev(w.y), w.omega()
    # S = K Omega against the oracle
    S = ctx.hss_kernel_sample(F, w.h, _dev(Om)).cpu().numpy()
    ref = gaussian_kernel(w.F, w.F, w.h) @ Om
    assert np.abs(S - ref).max() <= 1e-12 * np.abs(ref).max()
    ctx.hss_compress(F, y, w.h, w.leaf, w.tol, _dev(Om))
    exp = ctx.hss_export()
    perm = exp["perm"]
    assert np.array_equal(perm, cluster_tree(w.F, w.leaf))
    st = ctx.hss_stats()
    if name == "rank_cap_512_max":
        assert st["rank_cap"] == 512 and exp["sizes"].max() == 1024
    if name == "odd_ranks":
        assert (exp["ranks"][1:] % 2 == 1).any()
    H = oracle_hss_from_export(exp)
    rng = np.random.default_rng(0)
    v = rng.standard_normal(w.n)
    mv = ctx.hss_matvec(_dev(v)).cpu().numpy()
    mref = np.empty(w.n)
    mref[perm] = ohss.matvec(H, v[perm])
    assert _rel(mv, mref) <= 1e-12
    ctx.hss_ulv_factor(w.beta)
    x = _dev(v)
    ctx.hss_ulv_solve(x)
    Fz = oulv.ulv_factor(H, w.beta)
    xref = np.empty(w.n)
    xref[perm] = oulv.ulv_solve(Fz, v[perm])
    assert _rel(x.cpu().numpy(), xref) <= 1e-10
    out = ctx.admm_svm_train(w.C, w.beta, 15)
    oref = oadmm.admm(lambda t: oulv.ulv_solve(Fz, t), w.y[perm], w.C, w.beta, 15)
    for key in ("x", "z", "mu"):
        assert _rel(out[key].cpu().numpy()[perm], oref[key]) <= 1e-6, key
    G = w.F_test[:64]
    dec = ctx.svm_decision(_dev(G), out["z"], out["bias"]).cpu().numpy()
    dref = oadmm.decision(w.F[perm], w.y[perm], oref["z"], out["bias"], G, w.h)
    assert np.abs(dec - dref).max() <= 1e-6 * max(1.0, np.abs(dref).max())
    ctx.close()


def test_limits_are_rejected_not_run():
    w = synth.make_workload(1, n=2048, leaf=64, s=128)
    ctx = binding.Context()
    y = _dev(w.y)
    wide = _dev(np.zeros((2048, 385)))
    with pytest.raises(binding.HssError) as e:
        ctx.hss_compress(wide, y, 1.0, 64, 1e-3)
    assert e.value.code == binding.HSS_EUNSUPPORTED
    with pytest.raises(binding.HssError) as e:            # leaf above 1024
        ctx.hss_compress(_dev(w.F), y, 1.0, 2048, 1e-3)
    assert e.value.code == binding.HSS_EUNSUPPORTED
    ctx.hss_set_i64("sample_width", 2049)                 # sample wider than 2048 columns
    with pytest.raises(binding.HssError) as e:
        ctx.hss_compress(_dev(w.F), y, 1.0, 64, 1e-3)
    assert e.value.code == binding.HSS_EUNSUPPORTED
    ctx.hss_set_i64("sample_width", 1152)                 # rank cap 576 > 512
    with pytest.raises(binding.HssError) as e:
        ctx.hss_compress(_dev(w.F), y, 1.0, 64, 1e-3)
    assert e.value.code == binding.HSS_EUNSUPPORTED
    ctx.hss_set_i64("max_rank", 512)                      # Gram-Schmidt form (tol < 3e-5): at most 1024 columns
    with pytest.raises(binding.HssError) as e:
        ctx.hss_compress(_dev(w.F), y, 1.0, 64, 1e-6)
    assert e.value.code == binding.HSS_EUNSUPPORTED
    ctx.close()


def test_wide_sample_1024_columns_rank_cap_512():
    """The widest default configuration: 1024 sample columns, rank cap 512 (nodes of 1024 rows)."""
    from gpu_helpers import oracle_hss_from_export
    w = synth.make_workload(3, n=4096, leaf=256, s=1024)
    ctx = binding.Context()
    rc = ctx.hss_compress(_dev(w.F), _dev(w.y), w.h, w.leaf, w.tol, _dev(w.omega()))
    st = ctx.hss_stats()
    assert rc >= 0 and st["rank_cap"] == 512 and st["sample_width"] == 1024
    exp = ctx.hss_export()
    perm = exp["perm"]
    H = oracle_hss_from_export(exp)
    v = np.random.default_rng(0).standard_normal(w.n)
    ctx.hss_ulv_factor(1.0)
    x = _dev(v)
    ctx.hss_ulv_solve(x)
    Fz = oulv.ulv_factor(H, 1.0)
    ref = np.empty(w.n)
    ref[perm] = oulv.ulv_solve(Fz, v[perm])
    assert np.linalg.norm(x.cpu().numpy() - ref) <= 1e-10 * np.linalg.norm(ref)
    # as good as the oracle's compression of the same sample
    Fp = w.F[perm]
    K = gaussian_kernel(Fp, Fp, w.h)
    err = np.linalg.norm(K - ohss.densify(oracle_hss_from_export(exp, with_shift=False))) / np.linalg.norm(K)
    Ho = ohss.compress(Fp, w.h, w.leaf, w.omega()[perm], w.tol / 10.0, 1e-8, 512)
    err_or = np.linalg.norm(K - ohss.densify(Ho)) / np.linalg.norm(K)
    assert err <= max(w.tol, 1.5 * err_or), (err, err_or)
    ctx.close()


@pytest.mark.parametrize("r,n,n_test", [(3, 1000, 1), (30, 3001, 100), (60, 2048, 5000), (96, 777, 300), (8, 20000, 64)])
def test_label_assignment_shapes(r, n, n_test):
    """Decision values (Algorithm 3, last line) against the oracle's direct sum over the exact kernel, for every
    feature padding of the 16-column product (28, 56, 84, 112) and for row counts from one test point (the column
    blocks split over the grid) to thousands; the error estimate on the same context, narrow (<= 16 probes) against
    wide (the 128-column sampling block) on the same probe vectors."""
    rng = np.random.default_rng(r * 1000 + n_test)
    F = rng.standard_normal((n, r))
    G = rng.standard_normal((n_test, r))
    y = np.where(rng.random(n) < 0.5, 1.0, -1.0)
    h = 0.7 * np.sqrt(r)
    ctx = binding.Context()
    ctx.hss_compress(_dev(F), _dev(y), h, 64, 1e-2)
    z = rng.random(n)
    z[rng.random(n) < 0.3] = 0.0
    dec = ctx.svm_decision(_dev(G), _dev(z), 0.25).cpu().numpy()
    ref = oadmm.decision(F, y, z, 0.25, G, h)
    assert np.abs(dec - ref).max() <= 1e-10 * max(1.0, np.abs(ref).max())
    e16 = ctx.hss_error_estimate(16, 5)
    e17 = ctx.hss_error_estimate(17, 5)          # one more probe through the other kernel: nearly the same estimate
    assert abs(e16 - e17) <= 0.25 * e17
    ctx.close()


@pytest.mark.parametrize("offset", [1e3, 1e6, -3e7])
def test_features_with_a_large_common_offset(offset):
    """The Gaussian kernel sees differences of points only.  The kernel products expand ||f_i - f_j||^2 into norms and
    an inner product, which would lose log10(offset^2) digits on points far from the origin; the library subtracts
    the feature means first, so the results must match the oracle (direct differences) as on centred data: S = K Omega
    to 1e-12, the whole path on the exported matrix, and decision values for test points with the same offset."""
    from gpu_helpers import oracle_hss_from_export
    rng = np.random.default_rng(11)
    n, r, h, leaf, s = 1500, 8, 1.5, 64, 128
    F = rng.standard_normal((n, r)) + offset
    G = rng.standard_normal((200, r)) + offset
    y = np.where(rng.random(n) < 0.5, 1.0, -1.0)
    Om = rng.standard_normal((n, s))
    ctx = binding.Context()
    S = ctx.hss_kernel_sample(_dev(F), h, _dev(Om)).cpu().numpy()
    K = gaussian_kernel(F, F, h)
    ref = K @ Om
    assert np.abs(S - ref).max() <= 1e-12 * np.abs(ref).max()
    import torch
    Sn = torch.empty((n, s), dtype=torch.float64, device="cuda:0")
    ctx.hss_kernel_sample_noalloc(_dev(F), h, _dev(Om), Sn)
    torch.cuda.synchronize()
    assert np.array_equal(S, Sn.cpu().numpy())
    ctx.hss_compress(_dev(F), _dev(y), h, leaf, 1e-3, _dev(Om))
    exp = ctx.hss_export()
    perm = exp["perm"]
    assert np.array_equal(perm, cluster_tree(F, leaf))
    H = oracle_hss_from_export(exp, with_shift=False)
    Kp = K[np.ix_(perm, perm)]
    Kt = ohss.densify(H)
    for a, b in zip(H.loff[:-1], H.loff[1:]):
        assert np.abs(Kt[a:b, a:b] - Kp[a:b, a:b]).max() <= 1e-13
    Ho = ohss.compress(F[perm], h, leaf, Om[perm], 1e-4, 1e-8, ctx.hss_stats()["rank_cap"])
    err = np.linalg.norm(Kp - Kt) / np.linalg.norm(Kp)
    err_o = np.linalg.norm(Kp - ohss.densify(Ho)) / np.linalg.norm(Kp)
    assert err <= max(1.5 * err_o, 1e-3), (err, err_o)
    est = ctx.hss_error_estimate(16, 1)
    assert 0.3 * err <= est <= 3.0 * err + 1e-12
    z = rng.random(n)
    dec = ctx.svm_decision(_dev(G), _dev(z), -0.5).cpu().numpy()
    dref = oadmm.decision(F, y, z, -0.5, G, h)
    assert np.abs(dec - dref).max() <= 1e-10 * max(1.0, np.abs(dref).max())
    # neighbour-based sampling searches on the values as given: lists identical to the oracle's
    ctx2 = binding.Context()
    ctx2.hss_set_i64("sampling", 1)
    ctx2.hss_set_i64("ann_neighbours", 16)
    ctx2.hss_set_i64("ann_trees", 1)
    ctx2.hss_compress(_dev(F), _dev(y), h, leaf, 1e-2)
    idx, dist = ctx2.hss_export_neighbours()
    from oracle import ann as oann
    from oracle.tree import leaf_offsets, tree_depth
    L = tree_depth(n, leaf)
    lc = L
    while lc > 0 and (n >> lc) < 512:
        lc -= 1
    cells = leaf_offsets(n, lc)
    ri, rd = oann.ann_projection_trees(F[perm], 16, int(np.diff(cells).max()), 1, first_cells=list(cells))
    assert np.array_equal(idx, ri) and np.array_equal(dist, rd)
    ctx2.close()
    ctx.close()


@pytest.mark.parametrize("cfg,n", [(2, 8192), (4, 5000)])
def test_loosest_truncation_of_the_papers_first_table(cfg, n):
    """The parameter set under the paper's first results table: relative truncation threshold 1, absolute 0.1, rank cap
    200, 64 approximate neighbours per point.  A relative threshold of 1 keeps one pivot per block (the first pivot is
    always kept), so every rank is 1 and the compressed matrix is the leaf diagonal blocks plus rank-one couplings;
    the path on that matrix against the oracle as usual."""
    from gpu_helpers import oracle_hss_from_export
    w = synth.make_workload(cfg, n=n)
    ctx = binding.Context()
    ctx.hss_set_i64("sampling", 1)
    ctx.hss_set_i64("ann_neighbours", 64)
    ctx.hss_set_i64("sample_width", 256)
    ctx.hss_set_i64("max_rank", 200)
    ctx.hss_set_f64("abs_tol", 0.1)
    ctx.hss_compress(_dev(w.F), _dev(w.y), w.h, 128, 10.0)
    exp = ctx.hss_export()
    assert (exp["ranks"][1:] == 1).all()
    perm = exp["perm"]
    H = oracle_hss_from_export(exp)
    rng = np.random.default_rng(0)
    v = rng.standard_normal(n)
    mv = ctx.hss_matvec(_dev(v)).cpu().numpy()
    mref = np.empty(n)
    mref[perm] = ohss.matvec(H, v[perm])
    assert _rel(mv, mref) <= 1e-12
    ctx.hss_ulv_factor(w.beta)
    x = _dev(v)
    ctx.hss_ulv_solve(x)
    Fz = oulv.ulv_factor(H, w.beta)
    xref = np.empty(n)
    xref[perm] = oulv.ulv_solve(Fz, v[perm])
    assert _rel(x.cpu().numpy(), xref) <= 1e-10
    out = ctx.admm_svm_train(w.C, w.beta, 30)
    oref = oadmm.admm(lambda t: oulv.ulv_solve(Fz, t), w.y[perm], w.C, w.beta, 30)
    for key in ("x", "z", "mu"):
        assert _rel(out[key].cpu().numpy()[perm], oref[key]) <= 1e-6, key
    dec = ctx.svm_decision(_dev(w.F_test[:500]), out["z"], out["bias"]).cpu().numpy()
    acc = float(np.mean(np.where(dec >= 0, 1.0, -1.0) == w.y_test[:500])) * 100
    print(f"[table-1 parameters, cfg{cfg} n={n}] all ranks 1, delta {exp['delta']:.3f}, accuracy after 30 iterations {acc:.1f} %")
    ctx.close()
