"""Adaptive sample width on the GPU (oversampling and truncation of every block to the tolerance, end of Sec. 3.2)
against the oracle's compress_adaptive on the same Omega, and against the dense kernel (GPU only).

The entries of a compression are not unique (which rows a decomposition picks), so what is compared is: the
tolerance is met against the dense kernel with no node cut by a cap, the width the two sides end up with, the
total rank, and -- on the exported matrix -- mat-vec and ULV solve.  Where nothing is cut, or everything is, the
adaptive run must reproduce a fixed-width run bit for bit."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

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


def _low_dim_points(n, r, seed):
    """Points in r = 2 or 3 dimensions (the regime of the paper's low-dimensional sets, where block ranks are
    far below the block sizes) with a smooth label rule."""
    g = np.random.default_rng(seed)
    F = g.uniform(-1.0, 1.0, size=(n, r))
    y = np.where(np.sin(3.0 * F[:, 0]) + F[:, 1] + 0.2 * g.standard_normal(n) >= 0, 1.0, -1.0)
    Om = g.standard_normal((n, 512))
    return F, y, Om


def _compress(F, y, Om, h, leaf, tol, **opts):
    ctx = binding.Context()
    for k, v in opts.items():
        ctx.hss_set_i64(k, v)
    rc = ctx.hss_compress(_dev(F), _dev(y), h, leaf, tol, _dev(Om))
    return ctx, rc


# Gram / pivoted-Cholesky form and Gram-Schmidt form of the decomposition; block ranks reach about 200
@pytest.mark.parametrize("tol,h", [(1e-4, 0.1), (1e-6, 0.15)])
def test_adaptive_width_meets_the_tolerance(tol, h):
    from gpu_helpers import oracle_hss_from_export
    n, r, leaf = 4096, 2, 64
    F, y, Om = _low_dim_points(n, r, 7)
    # fixed width 128: upper nodes are cut by the cap, the tolerance is missed
    ctx0, rc0 = _compress(F, y, Om[:, :128], h, leaf, tol, oversample=10)
    st0 = ctx0.hss_stats()
    assert rc0 & binding.HSS_WRANK and st0["nodes_at_cap"] > 0
    exp0 = ctx0.hss_export()
    perm = exp0["perm"]
    Fp = F[perm]
    K = gaussian_kernel(Fp, Fp, h)
    nrm = np.linalg.norm(K)
    err0 = np.linalg.norm(K - ohss.densify(oracle_hss_from_export(exp0, with_shift=False))) / nrm
    assert err0 > 2 * tol
    ctx0.close()
    # adaptive from 128 columns in steps of 128, up to 512
    ctx, rc = _compress(F, y, Om, h, leaf, tol, oversample=10, adaptive_start=128, adaptive_step=128)
    st = ctx.hss_stats()
    assert not (rc & binding.HSS_WRANK) and st["nodes_at_cap"] == 0
    assert 128 < st["sample_width_used"] < 512 and st["nodes_redone"] > 0
    assert st["rank_max"] < st["sample_width_used"] - 10
    exp = ctx.hss_export()
    assert np.array_equal(exp["perm"], cluster_tree(F, leaf))
    H = oracle_hss_from_export(exp, with_shift=False)
    err = np.linalg.norm(K - ohss.densify(H)) / nrm
    assert err <= tol, (err, st)
    assert ctx.hss_error_estimate(32, 5) <= tol
    # the oracle's adaptive construction on the same Omega: same regime, same width, about the same ranks
    Ho, info = ohss.compress_adaptive(Fp, h, leaf, Om[perm], tol / 10.0, 1e-8, s0=128, step=128, oversample=10)
    err_or = np.linalg.norm(K - ohss.densify(Ho)) / nrm
    assert info["nodes_at_cap"] == 0 and err_or <= tol
    assert abs(st["sample_width_used"] - info["width"]) <= 128
    assert abs(int(exp["ranks"].sum()) - int(Ho.ranks().sum())) <= 0.05 * Ho.ranks().sum() + 4
    assert err <= max(tol, 1.5 * err_or)
    # downstream on the exported matrix (with the guard's shift)
    Hs = oracle_hss_from_export(exp)
    g = np.random.default_rng(1)
    v = g.standard_normal(n)
    mv = ctx.hss_matvec(_dev(v)).cpu().numpy()
    ref = np.empty(n)
    ref[perm] = ohss.matvec(Hs, v[perm])
    assert _rel(mv, ref) <= 1e-12
    ctx.hss_ulv_factor(1.0)
    x = _dev(v)
    ctx.hss_ulv_solve(x)
    Fz = oulv.ulv_factor(Hs, 1.0)
    ref[perm] = oulv.ulv_solve(Fz, v[perm])
    assert _rel(x.cpu().numpy(), ref) <= 1e-10
    ctx.close()


def test_adaptive_with_the_librarys_own_omega():
    n, r, h, leaf, tol = 8192, 3, 0.35, 128, 1e-3
    F, y, _ = _low_dim_points(n, r, 9)
    ctx = binding.Context()
    for k, v in dict(sample_width=1024, oversample=16, max_rank=500, adaptive_start=128, adaptive_step=128).items():
        ctx.hss_set_i64(k, v)
    rc = ctx.hss_compress(_dev(F), _dev(y), h, leaf, tol)
    st = ctx.hss_stats()
    assert not (rc & binding.HSS_WRANK) and st["nodes_at_cap"] == 0
    assert 128 < st["sample_width_used"] < 1024 and st["rank_max"] > 128
    assert ctx.hss_error_estimate(32, 5) <= tol
    # the flops of the sampling launches follow the columns actually sampled
    assert st["sample_flops"] == pytest.approx(
        2.0 * n * n * (st["sample_width_used"] + r * (1 + (st["sample_width_used"] - 128) // 128)), rel=1e-12)
    ctx.close()


def test_adaptive_reproduces_fixed_width_runs_bit_for_bit():
    # (a) nothing is cut at the first width: the further columns are never sampled
    n, h, leaf, tol = 2048, 0.8, 64, 1e-3
    F, y, Om = _low_dim_points(n, 2, 11)
    ctx_a, rc_a = _compress(F, y, Om, h, leaf, tol, oversample=10, adaptive_start=256)
    ctx_f, rc_f = _compress(F, y, Om[:, :256], h, leaf, tol, oversample=10)
    sa, sf = ctx_a.hss_stats(), ctx_f.hss_stats()
    assert sa["sample_width_used"] == 256 and sa["nodes_redone"] == 0 and sa["nodes_at_cap"] == 0
    assert sa["sample_flops"] == sf["sample_flops"]
    ea, ef = ctx_a.hss_export(), ctx_f.hss_export()
    for key in ("ranks", "U", "J", "B", "D"):
        assert np.array_equal(ea[key], ef[key]), key
    ctx_a.close()
    ctx_f.close()
    # (b) saturated workload (cut of workload 1): every level ends at the width the oracle's rule gives, and the
    # ranks are those of the cap
    w = synth.make_workload(1, n=2048, leaf=64, s=512)
    Om = w.omega()
    ctx, rc = _compress(w.F, w.y, Om, w.h, w.leaf, w.tol, adaptive_start=128, adaptive_step=128)
    st = ctx.hss_stats()
    exp = ctx.hss_export()
    perm = exp["perm"]
    Ho, info = ohss.compress_adaptive(w.F[perm], w.h, w.leaf, Om[perm], w.tol / 10.0, 1e-8, s0=128, step=128)
    assert st["sample_width_used"] == info["width"] == 512
    assert np.array_equal(exp["ranks"], Ho.ranks())
    assert st["nodes_redone"] == info["redone"]
    assert bool(rc & binding.HSS_WRANK) == (info["nodes_at_cap"] > 0)
    ctx.close()


def test_adaptive_option_errors():
    w = synth.make_workload(1, n=512, leaf=64, s=256)
    F, y, Om = _dev(w.F), _dev(w.y), _dev(w.omega())
    for opts in (dict(adaptive_start=100), dict(adaptive_start=128, adaptive_step=64)):
        ctx = binding.Context()
        for k, v in opts.items():
            ctx.hss_set_i64(k, v)
        with pytest.raises(binding.HssError) as e:
            ctx.hss_compress(F, y, w.h, w.leaf, w.tol, Om)
        assert e.value.code == binding.HSS_EINVAL
        ctx.close()
    ctx = binding.Context()
    with pytest.raises(binding.HssError):
        ctx.hss_set_i64("adaptive_step", 0)
    ctx.close()
