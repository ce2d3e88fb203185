"""Parity at the full workload sizes, in the launch configuration the benchmark times (GPU only).

cfg2 (n = 65 536), cfg3 (n = 262 144, the benchmark's workload), cfg5 (n = 262 144, r = 90) and cfg4
(n = 1 048 576): sampled rows of S = K Omega against the oracle, then the exported compressed matrix goes through
the oracle's ULV factorization, solve and a few ADMM iterations (same staging as tests/test_gpu_path.py; an oracle
solve takes 0.25 ... 4 s at these sizes, which bounds the iteration count here).  The workloads' FULL iteration
counts (500 / 500 / 300 / 300) run against the oracle on cuts of n = 16 384 points with the workload's own leaf
size, sample width and parameters (workload 1 runs whole, 200 iterations, in tests/test_gpu_path.py).  cfg4 and
cfg5 additionally: the residual of (K~ + delta I + beta I) x = b with the ORACLE's HSS mat-vec for every beta of
the sweep, and the invariants of the ADMM iterates.  cfg2: the guard's shift against the oracle's.
"""
import ctypes as C
import time

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


_T0 = time.time()


def _say(msg):
    """Progress line (visible with pytest -s): the oracle legs are silent for a while otherwise."""
    print(f"[fullsize +{time.time() - _T0:6.0f}s] {msg}", flush=True)


def _rel(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)


def _library_omega(n, s, seed=0):
    """The Omega hss_compress draws for this seed (through the library's generator hook)."""
    import torch
    from gpu_helpers import lib, ptr
    L = lib()
    Om = torch.empty((n, s), dtype=torch.float64, device="cuda:0")
    L.hsx_omega.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_uint64]
    assert L.hsx_omega(None, ptr(Om), n, s, seed) == 0
    return Om


def _check_sampled_rows(ctx, w, Om_dev, nrows, seed):
    """S = K Omega on the GPU (all rows) against the oracle on a few rows computed one block at a time."""
    F = _dev(w.F)
    S = ctx.hss_kernel_sample(F, w.h, Om_dev)
    rows = np.random.default_rng(seed).choice(w.n, nrows, replace=False)
    Om = Om_dev.cpu().numpy()
    ref = gaussian_kernel(w.F[rows], w.F, w.h) @ Om
    got = S[_dev(rows)].cpu().numpy()
    scale = np.abs(ref).max()
    assert np.abs(got - ref).max() <= 1e-12 * scale
    del S


def _bias_and_labels(ctx, w, out, oref, H, perm, name, n_test=512):
    """eq. (7) and the label loop of Algorithm 3: the oracle's formula on the library's iterate, and on the
    oracle's iterate over the library's margin set; the flips between the two margin sets are reported."""
    yp = w.y[perm]
    kmv = lambda v: ohss.matvec(H, v)
    z = out["z"].cpu().numpy()[perm]
    M_lib = oadmm.margin_set(z, w.C)
    flips = int((M_lib != oadmm.margin_set(oref["z"], w.C)).sum())
    _say(f"{name}: margin set {int(M_lib.sum())} of {w.n}, flips vs oracle {flips}")
    assert flips <= 1e-3 * w.n
    b_own, cnt_own = oadmm.bias(z, yp, w.C, kmv)
    assert out["n_margin"] == cnt_own
    assert abs(out["bias"] - b_own) <= 1e-6 * max(1.0, abs(b_own))
    b_cross, _ = oadmm.bias(oref["z"], yp, w.C, kmv, M=M_lib)
    assert abs(out["bias"] - b_cross) <= 1e-6 * max(1.0, abs(b_cross))
    if flips == 0:
        b_ref, _ = oadmm.bias(oref["z"], yp, w.C, kmv)
        assert abs(out["bias"] - b_ref) <= 1e-6 * max(1.0, abs(b_ref))
    G = w.F_test[:n_test]
    dec = ctx.svm_decision(_dev(G), out["z"], out["bias"]).cpu().numpy()
    dec_ref = oadmm.decision(w.F[perm], yp, oref["z"], b_cross, G, w.h)
    assert np.abs(dec - dec_ref).max() <= 1e-6 * max(1.0, np.abs(dec_ref).max())
    assert abs(oadmm.accuracy(dec, w.y_test[:n_test]) - oadmm.accuracy(dec_ref, w.y_test[:n_test])) <= 0.1


def _stage_compress(w, check_guard=False, sample_rows=16, options=None):
    """Sampled rows of S, compression with the in-library Omega (the benchmark's path), export, tree and one
    leaf block against the oracle.  Returns the state the later stages work on."""
    from gpu_helpers import oracle_hss_from_export
    ctx = binding.Context()
    ctx.hss_set_i64("sample_width", w.s)
    for key, val in (options or {}).items():
        ctx.hss_set_i64(key, val)
    F, y = _dev(w.F), _dev(w.y)
    if sample_rows:
        Om = _library_omega(w.n, w.s)
        _say(f"{w.name}: sampled rows of S")
        _check_sampled_rows(ctx, w, Om, sample_rows, 1)
        del Om
    _say(f"{w.name}: compress")
    rc = ctx.hss_compress(F, y, w.h, w.leaf, w.tol)
    assert rc >= 0
    _say("export")
    exp = ctx.hss_export()
    perm = exp["perm"]
    _say("oracle tree")
    assert np.array_equal(perm, cluster_tree(w.F, w.leaf))
    if check_guard:
        _say("oracle guard")
        d_or = ohss.psd_shift(oracle_hss_from_export(exp, with_shift=False))
        _say(f"delta: library {exp['delta']:.6g}, oracle {d_or:.6g}")
        assert d_or / 1.1 <= exp["delta"] <= 1.1 * d_or
    H = oracle_hss_from_export(exp)
    i = w.n // w.leaf // 3
    blk = slice(i * w.leaf, (i + 1) * w.leaf)
    Fp = w.F[perm]
    assert np.abs(exp["D"][i] - gaussian_kernel(Fp[blk], Fp[blk], w.h)).max() <= 1e-14
    return {"w": w, "ctx": ctx, "H": H, "perm": perm, "stats": ctx.hss_stats()}


def _stage_solve(st):
    """P2: ULV solve and mat-vec on the same compressed matrix."""
    w, ctx, H, perm = st["w"], st["ctx"], st["H"], st["perm"]
    ctx.hss_ulv_factor(w.beta)
    rng = np.random.default_rng(3)
    b = rng.standard_normal(w.n)
    x = _dev(b)
    ctx.hss_ulv_solve(x)
    x = x.cpu().numpy()
    _say("oracle ULV factor")
    st["Fz"] = Fz = oulv.ulv_factor(H, w.beta)
    _say("oracle ULV solve")
    ref = np.empty(w.n)
    ref[perm] = oulv.ulv_solve(Fz, b[perm])
    assert _rel(x, ref) <= 1e-10, _rel(x, ref)
    yv = ctx.hss_matvec(_dev(b)).cpu().numpy()
    mref = np.empty(w.n)
    mref[perm] = ohss.matvec(H, b[perm])
    assert _rel(yv, mref) <= 1e-12


def _stage_admm(st, admm_iters):
    """P3: ADMM, bias and labels on the same compressed matrix."""
    w, ctx, H, perm, Fz = st["w"], st["ctx"], st["H"], st["perm"], st["Fz"]
    _say(f"ADMM, {admm_iters} iterations")
    out = ctx.admm_svm_train(w.C, w.beta, admm_iters)
    oref = oadmm.admm(lambda v: oulv.ulv_solve(Fz, v), w.y[perm], w.C, w.beta, admm_iters)
    for key in ("x", "z", "mu"):
        got = out[key].cpu().numpy()[perm]
        assert _rel(got, oref[key]) <= 1e-6, (key, _rel(got, oref[key]))
    _say("bias / decision")
    _bias_and_labels(ctx, w, out, oref, H, perm, w.name)


def _full_oracle_parity(w, admm_iters, check_guard=False):
    st = _stage_compress(w, check_guard)
    _stage_solve(st)
    _stage_admm(st, admm_iters)
    st["ctx"].close()


def test_cfg3_full_size_neighbour_based_against_oracle():
    """Workload 3 at full size compressed from the neighbour-based sample (Sec. 3.1, first bullet): the exported
    matrix through the oracle's ULV factorization, solve, mat-vec, ADMM, bias and labels like the random sample's."""
    st = _stage_compress(synth.make_workload(3), sample_rows=0, options={"sampling": 1})
    assert st["stats"]["sample_flops"] == 0.0                # no product with a random matrix was formed
    _stage_solve(st)
    _stage_admm(st, 6)
    st["ctx"].close()


def test_cfg2_full_size_neighbour_lists_against_oracle():
    """The neighbour lists of workload 2 at full size (65 536 points, 64 neighbours each, three trees) against the
    oracle's search with the library's random directions: identical indices, bit-identical distances."""
    from oracle import ann as oann
    from test_gpu_ann import _library_directions
    w = synth.make_workload(2)
    ctx = binding.Context()
    ctx.hss_set_i64("sample_width", w.s)
    ctx.hss_set_i64("sampling", 1)
    ctx.hss_compress(_dev(w.F), _dev(w.y), w.h, w.leaf, w.tol)
    idx, dist = ctx.hss_export_neighbours()
    perm = ctx.hss_export()["perm"]
    ctx.close()
    _say("cfg2: oracle neighbour search")
    ref_i, ref_d = oann.ann_projection_trees(w.F[perm], 64, 512, 3, directions=_library_directions(0, w.r))
    assert np.array_equal(idx, ref_i)
    assert np.array_equal(dist, ref_d)


def test_cfg2_full_size_against_oracle():
    _full_oracle_parity(synth.make_workload(2), admm_iters=25, check_guard=True)


def test_cfg3_full_size_against_oracle():
    _full_oracle_parity(synth.make_workload(3), admm_iters=6)


def test_cfg5_full_size_against_oracle():
    _full_oracle_parity(synth.make_workload(5), admm_iters=6)


# Workload 4 (n = 1 048 576) in stages of its own, so that no single test is silent for minutes: generating
# and compressing, the oracle's factorization (80 s), the iterations, the properties.
@pytest.fixture(scope="module")
def cfg4_state():
    st = {}
    yield st
    if "ctx" in st:
        st["ctx"].close()
    st.clear()


def test_cfg4_full_size_compression_against_oracle(cfg4_state):
    cfg4_state.update(_stage_compress(synth.make_workload(4), sample_rows=4))


def test_cfg4_full_size_ulv_solve_against_oracle(cfg4_state):
    _stage_solve(cfg4_state)


def test_cfg4_full_size_admm_against_oracle(cfg4_state):
    _stage_admm(cfg4_state, admm_iters=2)


def test_cfg4_full_size_properties(cfg4_state):
    _property_parity(cfg4_state["w"], admm_iters=20, state=cfg4_state)


@pytest.mark.parametrize("cfg", [2, 3, 4, 5])
def test_full_iteration_count_on_a_cut(cfg):
    """Algorithm 3 end to end with the workload's own iteration count: x, z, mu, bias and labels after
    500 / 500 / 300 / 300 iterations against the oracle on the same compressed matrix (n = 16 384 points of
    the workload's generator, its leaf size, sample width, tolerance, h, C, beta)."""
    from gpu_helpers import oracle_hss_from_export
    w = synth.make_workload(cfg, n=16384)
    ctx = binding.Context()
    ctx.hss_set_i64("sample_width", w.s)
    rc = ctx.hss_compress(_dev(w.F), _dev(w.y), w.h, w.leaf, w.tol)
    assert rc >= 0
    exp = ctx.hss_export()
    perm = exp["perm"]
    H = oracle_hss_from_export(exp)
    _say(f"{w.name} cut: {w.maxit} iterations, delta {exp['delta']:.4g}")
    out = ctx.admm_svm_train(w.C, w.beta, w.maxit)
    Fz = oulv.ulv_factor(H, w.beta)
    oref = oadmm.admm(lambda v: oulv.ulv_solve(Fz, v), w.y[perm], w.C, w.beta, w.maxit)
    for key in ("x", "z", "mu"):
        got = out[key].cpu().numpy()[perm]
        assert _rel(got, oref[key]) <= 1e-6, (key, _rel(got, oref[key]))
    _bias_and_labels(ctx, w, out, oref, H, perm, w.name + " cut", n_test=2048)
    ctx.close()


def _property_parity(w, admm_iters, sweep=False, state=None):
    from gpu_helpers import oracle_hss_from_export
    if state is None:
        ctx = binding.Context()
        ctx.hss_set_i64("sample_width", w.s)
        F, y = _dev(w.F), _dev(w.y)
        _say(f"{w.name}: compress")
        rc = ctx.hss_compress(F, y, w.h, w.leaf, w.tol)
        assert rc >= 0
        st = ctx.hss_stats()
        _say("export")
        exp = ctx.hss_export()
        perm = exp["perm"]
        H = oracle_hss_from_export(exp)
        del exp
    else:
        ctx, H, perm, st = state["ctx"], state["H"], state["perm"], state["stats"]
    rng = np.random.default_rng(5)
    b = rng.standard_normal(w.n)
    betas = w.beta_grid if sweep else (w.beta,)
    for beta in betas:
        _say(f"factor/solve beta={beta}")
        ctx.hss_ulv_factor(beta)
        x = _dev(b)
        ctx.hss_ulv_solve(x)
        x = x.cpu().numpy()
        # residual with the oracle's mat-vec: (K~ + delta I) x + beta x = b
        r = ohss.matvec(H, x[perm]) + beta * x[perm] - b[perm]
        # the matrix is symmetric positive definite with lambda_min >= ~beta, so the error is bounded by the
        # residual over beta
        assert np.linalg.norm(r) <= 1e-10 * beta * np.linalg.norm(x), (beta, np.linalg.norm(r) / np.linalg.norm(x))
    _say("ADMM")
    out = ctx.admm_svm_train(w.C, betas[-1], admm_iters)
    xg, zg = out["x"].cpu().numpy(), out["z"].cpu().numpy()
    assert zg.min() >= 0.0 and zg.max() <= w.C
    assert abs(float(w.y @ xg)) <= 1e-9 * max(1.0, np.linalg.norm(xg))          # y^T x^k = 0 (Sec. 2.1)
    mu = out["mu"].cpu().numpy()
    # z^{k+1} = clip(x^{k+1} - mu^k / beta) and mu^{k+1} = mu^k - beta (x - z): eliminate mu^k
    beta = betas[-1]
    muk = mu + beta * (xg - zg)
    assert np.abs(zg - np.clip(xg - muk / beta, 0.0, w.C)).max() <= 1e-12 * max(1.0, np.abs(xg).max())
    assert st["rank_max"] <= st["rank_cap"]
    if state is None:
        ctx.close()


def test_cfg5_full_size_properties_and_beta_sweep():
    _property_parity(synth.make_workload(5), admm_iters=30, sweep=True)
