"""Point counts that are not leaf * 2^L (GPU only): the tree has leaves of two sizes (ceil and floor of n / 2^L, the
larger ones where the bit reversal of the leaf number is below n mod 2^L).  Checked against the oracle exactly as
the regular sizes are: both cluster trees bit for bit, S = K Omega, the reconstruction error where the ranks do
not saturate, and mat-vec / ULV solve / ADMM / bias / decision values on the exported matrix; the neighbour lists
and the neighbour-based construction; the import of ragged generators; several box bounds at once."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import admm as oadmm          # noqa: E402
from oracle import ann as oann            # noqa: E402
from oracle import hss as ohss            # noqa: E402
from oracle import ulv as oulv            # noqa: E402
from oracle.kernel import gaussian_kernel  # noqa: E402
from oracle.tree import cluster_tree, cluster_tree_2means, leaf_offsets, tree_depth      # noqa: E402
from paper_2108_04167_amd import binding, synth   # noqa: E402


def _dev(a):
    import torch
    return torch.tensor(np.ascontiguousarray(a), device="cuda:0")


def _rel(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)


def _downstream_parity(ctx, w, perm, H, iters=15, decision=True):
    """mat-vec, ULV solve, ADMM, bias and decision values of the library against the oracle on the matrix H."""
    rng = np.random.default_rng(0)
    n = w.n
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
    out = ctx.admm_svm_train(w.C, w.beta, iters)
    oref = oadmm.admm(lambda t: oulv.ulv_solve(Fz, t), w.y[perm], w.C, w.beta, iters)
    for key in ("x", "z", "mu"):
        assert _rel(out[key].cpu().numpy()[perm], oref[key]) <= 1e-6, key
    z = out["z"].cpu().numpy()
    M = oadmm.margin_set(z[perm], w.C)
    bref, cnt = oadmm.bias(z[perm], w.y[perm], w.C, lambda t: ohss.matvec(H, t), M=M)
    assert out["n_margin"] == cnt
    if cnt:
        assert abs(out["bias"] - bref) <= 1e-6 * max(1.0, abs(bref))
    if decision:
        G = w.F_test[:64]
        dec = ctx.svm_decision(_dev(G), out["z"], out["bias"]).cpu().numpy()
        dref = oadmm.decision(w.F[perm], w.y[perm], z[perm], out["bias"], G, w.h)
        assert np.abs(dec - dref).max() <= 1e-6 * max(1.0, np.abs(dref).max())
    return out


# name -> (cfg, n, leaf, s, options)
SHAPES = {
    "n1000_leaf64": (1, 1000, 64, 128, {}),
    "n2049_leaf64": (1, 2049, 64, 128, {}),              # one point over a power of two: leaves of 33 and 32
    "n2047_leaf64": (1, 2047, 64, 128, {}),              # one under: leaves of 64 and 63
    "n777_leaf32": (2, 777, 32, 128, {}),
    "n37_leaf16": (1, 37, 16, 128, {}),                  # leaves of 10, 9, 9, 9
    "n15_one_leaf": (1, 15, 16, 128, {}),                # a single leaf below the leaf size
    "n17_two_leaves": (1, 17, 16, 128, {}),
    "n1_single_point": (1, 1, 16, 128, {}),
    "n2_two_points": (1, 2, 16, 128, {}),
    "n3_leaf2": (1, 3, 2, 128, {}),                      # leaves of 2 and 1 points
    "n3001_r54": (3, 3001, 256, 512, {}),
    "n1000_leaf10": (1, 1000, 10, 128, {}),              # leaf sizes that are no multiple of anything: 7 and 8
    "n1234_leaf100": (2, 1234, 100, 128, {}),
    "n500_leaf3": (1, 500, 3, 128, {"max_rank": 2}),     # leaves of 1 and 2 points
    "n5000_r90": (5, 5000, 256, 512, {}),
    "n4099_leaf1024": (4, 4099, 1024, 512, {}),
    "n1500_odd_ranks": (1, 1500, 64, 128, {"max_rank": 37}),
    "n3000_adaptive": (1, 3000, 64, 512, {"adaptive_start": 128}),
    # smooth kernels: the tolerance, not the rank cap, ends the decompositions (both forms of the decomposition)
    "n2000_lowrank_gram": (1, 2000, 32, 128, {"h": 20.0, "tol": 1e-3, "max_rank": 118}),
    "n1999_lowrank_gram": (1, 1999, 64, 128, {"h": 12.0, "tol": 1e-4, "max_rank": 100}),
    "n2001_lowrank_gs": (1, 2001, 32, 128, {"h": 20.0, "tol": 1e-6, "max_rank": 118}),
}


@pytest.mark.parametrize("name", list(SHAPES))
def test_ragged_shape(name):
    from gpu_helpers import oracle_hss_from_export
    cfg, n, leaf, s, opts = SHAPES[name]
    w = synth.make_workload(cfg, n=n, leaf=leaf, s=s)
    opts = dict(opts)
    w.h = opts.pop("h", w.h)
    w.tol = opts.pop("tol", w.tol)
    ctx = binding.Context()
    for k, v in opts.items():
        ctx.hss_set_i64(k, v)
    F, y, Om = _dev(w.F), _dev(w.y), w.omega()
    S = ctx.hss_kernel_sample(F, w.h, _dev(Om)).cpu().numpy()
    K = gaussian_kernel(w.F, w.F, w.h)
    ref = K @ Om
    assert np.abs(S - ref).max() <= 1e-12 * np.abs(ref).max()
    rc = ctx.hss_compress(F, y, w.h, w.leaf, w.tol, _dev(Om))
    exp = ctx.hss_export()
    perm = exp["perm"]
    assert np.array_equal(perm, cluster_tree(w.F, w.leaf))
    L = tree_depth(n, leaf)
    st = ctx.hss_stats()
    assert st["levels"] == L and st["n"] == n
    nl = 2 ** L
    assert np.array_equal(exp["sizes"][nl - 1:], np.diff(leaf_offsets(n, L)))
    H = oracle_hss_from_export(exp, with_shift=False)
    Kp = K[np.ix_(perm, perm)]
    Kt = ohss.densify(H)
    for a, b in zip(H.loff[:-1], H.loff[1:]):             # leaf blocks are entries of K
        assert np.abs(Kt[a:b, a:b] - Kp[a:b, a:b]).max() <= 1e-14
    err = np.linalg.norm(Kp - Kt) / np.linalg.norm(Kp)
    if "lowrank" in name:
        assert not (rc & binding.HSS_WRANK) and st["nodes_at_cap"] == 0        # these cases exist for this branch
    if not (rc & binding.HSS_WRANK):
        assert err <= w.tol, err
    # the oracle's own compression of the same points from the same sample: same quality
    Ho = ohss.compress(w.F[perm], w.h, leaf, Om[perm], w.tol / 10.0, 1e-8, st["rank_cap"])
    err_o = np.linalg.norm(Kp - ohss.densify(Ho)) / np.linalg.norm(Kp)
    assert err <= max(2.0 * err_o, w.tol), (err, err_o)
    print(f"[{name}] L={L} leaves {exp['sizes'][nl - 1:].min()}..{exp['sizes'][nl - 1:].max()} "
          f"rank max {exp['ranks'].max()} err {err:.2e} (oracle {err_o:.2e})")
    _downstream_parity(ctx, w, perm, oracle_hss_from_export(exp))
    ctx.close()


@pytest.mark.parametrize("n,r,leaf", [(1000, 8, 64), (2049, 3, 32), (777, 20, 16), (33, 2, 16), (5001, 12, 128)])
def test_ragged_2means_tree_is_the_oracles(n, r, leaf):
    g = np.random.default_rng(n)
    centres = g.standard_normal((16, r)) * 3.0
    F = centres[g.integers(0, 16, n)] + 0.3 * g.standard_normal((n, r))
    y = np.where(np.arange(n) % 2 == 0, 1.0, -1.0)
    ctx = binding.Context()
    ctx.hss_set_i64("clustering", 1)
    ctx.hss_compress(_dev(F), _dev(y), 1.0, leaf, 1e-2)
    perm = ctx.hss_export()["perm"]
    ctx.close()
    assert np.array_equal(perm, cluster_tree_2means(F, leaf, 2))


@pytest.mark.parametrize("n,r,leaf,k,cell,trees,seed", [
    (1000, 3, 64, 16, 256, 4, 5), (2049, 8, 64, 64, 512, 3, 1), (777, 5, 16, 8, 64, 3, 2), (300, 4, 64, 64, 4096, 3, 0),
    (3001, 54, 256, 33, 512, 2, 7)])
def test_ragged_neighbour_lists_are_the_oracles(n, r, leaf, k, cell, trees, seed):
    from test_gpu_ann import _library_directions
    rng = np.random.default_rng(100 + n + r)
    F = rng.standard_normal((n, r))
    if r == 54:
        F[:, 10:] = (rng.random((n, 44)) < 0.1).astype(np.float64)
    y = np.where(rng.random(n) < 0.5, 1.0, -1.0)
    ctx = binding.Context()
    ctx.hss_set_i64("sampling", 1)
    for key, v in dict(ann_neighbours=k, ann_cell=cell, ann_trees=trees, seed=seed).items():
        ctx.hss_set_i64(key, v)
    ctx.hss_compress(_dev(F), _dev(y), 1.0, leaf, 1e-2)
    idx, dist = ctx.hss_export_neighbours()
    perm = ctx.hss_export()["perm"]
    ctx.close()
    L = tree_depth(n, leaf)
    lc = L
    while lc > 0 and (n >> lc) < cell:                       # deepest level whose nodes all hold >= cell points
        lc -= 1
    cells = leaf_offsets(n, lc)
    ref_i, ref_d = oann.ann_projection_trees(F[perm], k, int(np.diff(cells).max()), trees,
                                             directions=_library_directions(seed, r), first_cells=list(cells))
    assert np.array_equal(idx, ref_i)
    assert np.array_equal(dist, ref_d)


@pytest.mark.parametrize("cfg,n,leaf,s", [(2, 3000, 128, 256), (4, 5003, 256, 512)])
def test_ragged_neighbour_based_compression(cfg, n, leaf, s):
    from gpu_helpers import oracle_hss_from_export
    w = synth.make_workload(cfg, n=n, leaf=leaf, s=s)
    ctx = binding.Context()
    ctx.hss_set_i64("sampling", 1)
    ctx.hss_set_i64("sample_width", s)
    ctx.hss_compress(_dev(w.F), _dev(w.y), w.h, leaf, w.tol)
    exp = ctx.hss_export()
    perm = exp["perm"]
    idx, dist = ctx.hss_export_neighbours()
    st = ctx.hss_stats()
    K = gaussian_kernel(w.F[perm], w.F[perm], w.h)
    err = np.linalg.norm(K - ohss.densify(oracle_hss_from_export(exp, with_shift=False))) / np.linalg.norm(K)
    Ho, _ = oann.compress_ann(w.F[perm], w.h, leaf, idx.astype(np.int64), dist, s, w.tol / 10.0, 1e-8, st["rank_cap"])
    err_o = np.linalg.norm(K - ohss.densify(Ho)) / np.linalg.norm(K)
    print(f"[ragged ann cfg{cfg} n={n}] err {err:.2e} oracle {err_o:.2e} rank max {exp['ranks'].max()}")
    assert err <= max(2.0 * err_o, w.tol), (err, err_o)
    _downstream_parity(ctx, w, perm, oracle_hss_from_export(exp))
    ctx.close()


def test_ragged_import_round_trip_and_oracle_generators():
    """Generators the oracle built on a ragged tree, imported: the library's solve and ADMM on them against the
    oracle's; and export -> import -> export gives the same arrays back."""
    from gpu_helpers import export_from_oracle_hss, oracle_hss_from_export
    w = synth.make_workload(1, n=1234, leaf=64, s=128)
    perm = cluster_tree(w.F, w.leaf)
    Om = w.omega()
    H = ohss.compress(w.F[perm], w.h, w.leaf, Om[perm], w.tol / 10.0, 1e-8, 64)
    gen = export_from_oracle_hss(H, perm)
    ctx = binding.Context()
    ctx.hss_import(_dev(w.F), _dev(w.y), w.h, w.leaf, gen)
    exp = ctx.hss_export()
    for key in ("perm", "sizes", "ranks", "U", "J", "B"):
        assert np.array_equal(exp[key], gen[key]), key
    assert all(np.array_equal(a, b) for a, b in zip(exp["D"], gen["D"]))
    _downstream_parity(ctx, w, perm, H)
    # a leaf size that does not belong to the tree of this n is refused
    bad = dict(gen)
    bad["sizes"] = gen["sizes"].copy()
    bad["sizes"][-1] += 1
    ctx2 = binding.Context()
    with pytest.raises(binding.HssError) as e:
        ctx2.hss_import(_dev(w.F), _dev(w.y), w.h, w.leaf, bad)
    assert e.value.code == binding.HSS_EINVAL
    ctx2.close()
    ctx.close()


def test_ragged_several_box_bounds_and_right_hand_sides():
    from gpu_helpers import oracle_hss_from_export
    w = synth.make_workload(2, n=3333, leaf=128, s=256)
    ctx = binding.Context()
    ctx.hss_compress(_dev(w.F), _dev(w.y), w.h, w.leaf, w.tol, _dev(w.omega()))
    exp = ctx.hss_export()
    perm = exp["perm"]
    H = oracle_hss_from_export(exp)
    beta = 2.0
    Cs = [0.1, 1.0, 10.0, 100.0]
    out = ctx.admm_svm_train_multi(Cs, beta, 20)
    Fz = oulv.ulv_factor(H, beta)
    for j, C in enumerate(Cs):
        oref = oadmm.admm(lambda t: oulv.ulv_solve(Fz, t), w.y[perm], C, beta, 20)
        for key in ("x", "z", "mu"):
            assert _rel(out[key][j].cpu().numpy()[perm], oref[key]) <= 1e-6, (key, C)
    ctx.close()


def test_ragged_mid_size_like_a_public_data_set():
    """n = 32561 (the size of a data set of the paper's Table 1) with workload 2's generator, leaf 128: ULV solve and
    a short ADMM run against the oracle on the exported matrix, residual of the solve through the oracle's mat-vec."""
    from gpu_helpers import oracle_hss_from_export
    w = synth.make_workload(2, n=32561)
    ctx = binding.Context()
    ctx.hss_set_i64("sample_width", w.s)
    ctx.hss_compress(_dev(w.F), _dev(w.y), w.h, w.leaf, w.tol)
    exp = ctx.hss_export()
    st = ctx.hss_stats()
    L = tree_depth(w.n, w.leaf)
    assert st["levels"] == L == 8
    assert sorted(set(exp["sizes"][2 ** L - 1:].tolist())) == [127, 128]
    perm = exp["perm"]
    assert np.array_equal(perm, cluster_tree(w.F, w.leaf))
    _downstream_parity(ctx, w, perm, oracle_hss_from_export(exp), iters=10, decision=True)
    ctx.close()


def _draw_ragged(seed):
    g = np.random.default_rng(5000 + seed)
    leaf = int(g.choice([16, 32, 48, 64, 80, 128, 176, 256]))
    n = int(g.integers(1, 40 * leaf)) if g.random() < 0.8 else int(g.integers(1, 3 * leaf))
    n = min(n, 5000)
    r = int(g.choice([1, 2, 3, 5, 8, 13, 28, 29, 57, 84, 96, 97, 112, 113, 123, 200, 300, 384]))
    s = int(g.choice([32, 100, 128, 256]))
    F = g.standard_normal((n, r)) * g.uniform(0.3, 2.0, size=r)
    if g.random() < 0.3:                      # some binary columns: exact ties in the trees
        k = max(1, r // 3)
        F[:, :k] = (g.random((n, k)) < 0.3).astype(np.float64)
    if g.random() < 0.2:                      # a common offset
        F += g.choice([1e2, -1e4, 1e5])
    y = np.where(g.random(n) < 0.5, -1.0, 1.0)
    h = float(np.sqrt(r) * g.choice([0.5, 1.0, 3.0, 10.0]))
    tol = float(g.choice([1e-2, 1e-3, 1e-4, 3e-5, 1e-5, 1e-6]))
    opts = {"clustering": int(g.random() < 0.3), "sampling": int(g.random() < 0.3)}
    if g.random() < 0.4:
        opts["max_rank"] = int(g.integers(3, max(4, min(s, 2 * leaf))))
    if g.random() < 0.2:
        opts["psd_guard"] = 0
    if opts["sampling"]:
        opts["ann_neighbours"] = int(g.choice([8, 33, 64]))
        opts["ann_trees"] = int(g.choice([1, 2, 3]))
        opts["ann_cell"] = int(g.choice([64, 512]))
    return dict(n=n, leaf=leaf, r=r, s=s, F=F, y=y, h=h, tol=tol, opts=opts, C=float(g.choice([0.1, 1.0, 10.0])),
                beta=float(g.choice([0.5, 1.0, 4.0])), Om=g.standard_normal((n, s)))


@pytest.mark.parametrize("seed", range(24))
def test_random_ragged_problem(seed):
    """Seeded random problems with any point count (1 .. 5000), 1 .. 384 features, offsets, both trees and both
    samplings, through the whole path against the oracle."""
    from gpu_helpers import oracle_hss_from_export
    p = _draw_ragged(seed)
    n = p["n"]
    ctx = binding.Context()
    ctx.hss_set_i64("sample_width", p["s"])
    for k, v in p["opts"].items():
        ctx.hss_set_i64(k, v)
    F, y = _dev(p["F"]), _dev(p["y"])
    K = gaussian_kernel(p["F"], p["F"], p["h"])
    S = ctx.hss_kernel_sample(F, p["h"], _dev(p["Om"])).cpu().numpy()
    ref = K @ p["Om"]
    assert np.abs(S - ref).max() <= 1e-12 * max(np.abs(ref).max(), 1e-300), "sample"
    if p["opts"]["sampling"]:
        ctx.hss_compress(F, y, p["h"], p["leaf"], p["tol"])
    else:
        ctx.hss_compress(F, y, p["h"], p["leaf"], p["tol"], _dev(p["Om"]))
    exp = ctx.hss_export()
    perm = exp["perm"]
    tree = cluster_tree_2means(p["F"], p["leaf"], 2) if p["opts"]["clustering"] else cluster_tree(p["F"], p["leaf"])
    assert np.array_equal(perm, tree), "tree"
    H = oracle_hss_from_export(exp)
    st = ctx.hss_stats()
    g = np.random.default_rng(seed)
    v = g.standard_normal(n)
    mv = ctx.hss_matvec(_dev(v)).cpu().numpy()
    mref = np.empty(n)
    mref[perm] = ohss.matvec(H, v[perm])
    assert _rel(mv, mref) <= 1e-12, "matvec"
    # compression quality: as good as the oracle's on the same sample (or the same neighbour lists)
    Kp = K[np.ix_(perm, perm)]
    Kt = ohss.densify(oracle_hss_from_export(exp, with_shift=False))
    err = np.linalg.norm(Kp - Kt) / np.linalg.norm(Kp)
    if p["opts"]["sampling"] and tree_depth(n, p["leaf"]) >= 1:
        idx, dist = ctx.hss_export_neighbours()
        Ho, _ = oann.compress_ann(p["F"][perm], p["h"], p["leaf"], idx.astype(np.int64), dist, p["s"], p["tol"] / 10,
                                  1e-8, st["rank_cap"])
    else:
        Ho = ohss.compress(p["F"][perm], p["h"], p["leaf"], p["Om"][perm], p["tol"] / 10, 1e-8, st["rank_cap"])
    err_o = np.linalg.norm(Kp - ohss.densify(Ho)) / np.linalg.norm(Kp)
    assert err <= max(2.0 * err_o, p["tol"], 1e-12), ("quality", err, err_o)
    ctx.hss_ulv_factor(p["beta"])
    x = _dev(v)
    ctx.hss_ulv_solve(x)
    Fz = oulv.ulv_factor(H, p["beta"])
    xref = np.empty(n)
    xref[perm] = oulv.ulv_solve(Fz, v[perm])
    cond = np.linalg.cond(ohss.densify(H) + p["beta"] * np.eye(n)) if n <= 1500 else 1.0   # guard off: can be large
    assert _rel(x.cpu().numpy(), xref) <= 1e-10 * max(1.0, cond / 1e4), ("solve", cond)
    out = ctx.admm_svm_train(p["C"], p["beta"], 12)
    oref = oadmm.admm(lambda t: oulv.ulv_solve(Fz, t), p["y"][perm], p["C"], p["beta"], 12)
    for key in ("x", "z", "mu"):
        assert _rel(out[key].cpu().numpy()[perm], oref[key]) <= 1e-6 * max(1.0, cond / 1e6), (key, cond)
    G = p["F"][:min(n, 50)] + 0.1
    dec = ctx.svm_decision(_dev(G), out["z"], out["bias"]).cpu().numpy()
    dref = oadmm.decision(p["F"], p["y"], out["z"].cpu().numpy(), out["bias"], G, p["h"])
    assert np.abs(dec - dref).max() <= 1e-9 * max(1.0, np.abs(dref).max()), "decision"
    ctx.close()


def _draw_solve_options(seed):
    g = np.random.default_rng(9000 + seed)
    leaf = int(g.choice([8, 16, 32, 48, 64, 100, 128, 256]))
    n = int(g.integers(1, 30 * leaf)) if g.random() < 0.85 else int(g.integers(1, 3 * leaf))
    n = min(n, 4000)
    r = int(g.choice([1, 2, 5, 8, 18, 54, 90, 123]))
    s = int(g.choice([32, 100, 128, 256]))
    F = g.standard_normal((n, r)) * g.uniform(0.3, 2.0, size=r)
    y = np.where(g.random(n) < 0.5, -1.0, 1.0)
    h = float(np.sqrt(r) * g.choice([1.0, 3.0, 10.0]))
    tol = float(g.choice([1e-2, 1e-3, 1e-4, 1e-6]))
    opts = {"merge_top": int(g.random() < 0.5), "graph": int(g.random() < 0.5), "cache_basis": int(g.random() < 0.5)}
    if g.random() < 0.4:
        opts["max_rank"] = int(g.integers(3, max(4, min(s, 2 * leaf))))
    if g.random() < 0.3:
        opts["adaptive_start"] = 128
        opts["adaptive_step"] = int(g.choice([128, 256]))
        s = int(g.choice([256, 384, 512]))
    if g.random() < 0.3:
        opts["clustering"] = 1
    betas = [float(b) for b in g.choice([0.25, 0.5, 1.0, 2.0, 8.0], size=3)]
    return dict(n=n, leaf=leaf, r=r, s=s, F=F, y=y, h=h, tol=tol, opts=opts, betas=betas,
                Cs=[0.1, 1.0, 10.0][:int(g.integers(1, 4))], nrhs=int(g.integers(1, 6)), Om=g.standard_normal((n, s)))


@pytest.mark.parametrize("seed", range(10))
def test_random_ragged_solve_options(seed):
    """Seeded random problems on uneven trees with the options of the solve drawn at random (merged top, graph replay,
    cached bases across beta, adaptive width, either tree): three factorizations in a row on one compression, several
    right-hand sides solved twice each (the second call replays), several box bounds in lockstep and one alone, all
    against the oracle's ULV and ADMM on the exported matrix."""
    from gpu_helpers import oracle_hss_from_export
    p = _draw_solve_options(seed)
    n = p["n"]
    ctx = binding.Context()
    for k, v in p["opts"].items():
        ctx.hss_set_i64(k, v)
    ctx.hss_compress(_dev(p["F"]), _dev(p["y"]), p["h"], p["leaf"], p["tol"], _dev(p["Om"]))
    exp = ctx.hss_export()
    perm = exp["perm"]
    H = oracle_hss_from_export(exp)
    g = np.random.default_rng(seed)
    cond = np.linalg.cond(ohss.densify(H) + min(p["betas"]) * np.eye(n)) if n <= 1500 else 1.0
    for beta in p["betas"]:
        ctx.hss_ulv_factor(beta)
        Fz = oulv.ulv_factor(H, beta)
        V = g.standard_normal((p["nrhs"], n))
        for rep in range(2):
            X = _dev(V if p["nrhs"] > 1 else V[0])
            ctx.hss_ulv_solve(X)
            X = X.cpu().numpy().reshape(p["nrhs"], n)
            for j in range(p["nrhs"]):
                xref = np.empty(n)
                xref[perm] = oulv.ulv_solve(Fz, V[j][perm])
                assert _rel(X[j], xref) <= 1e-10 * max(1.0, cond / 1e4), ("solve", beta, rep, j, cond)
        out = ctx.admm_svm_train_multi(p["Cs"], beta, 10)
        for ci, Cb in enumerate(p["Cs"]):
            oref = oadmm.admm(lambda t: oulv.ulv_solve(Fz, t), p["y"][perm], Cb, beta, 10)
            for key in ("x", "z", "mu"):
                assert _rel(out[key].cpu().numpy()[ci][perm], oref[key]) <= 1e-6 * max(1.0, cond / 1e6), (key, beta, Cb)
        one = ctx.admm_svm_train(p["Cs"][-1], beta, 10)
        for key in ("x", "z", "mu"):
            assert _rel(one[key].cpu().numpy()[perm], oref[key]) <= 1e-6 * max(1.0, cond / 1e6), (key, beta)
    ctx.close()
