"""Several right-hand sides through one ULV sweep, and the C-sweep of the ADMM trainer (GPU only).

The hyper-parameter sweep reuses one compression and one factorization per beta (Sec. 3.2); the library runs
up to four values of C in lockstep as interleaved right-hand sides.  Every column must equal the
single-column path and the oracle on the same exported matrix.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import admm as oadmm          # noqa: E402
from oracle import hss as ohss            # noqa: E402
from oracle import ulv as oulv            # noqa: E402
from paper_2108_04167_amd import binding, synth   # noqa: E402

CASES = {
    # name -> (cfg, n, leaf, s, overrides, options)
    "cfg5_small": (5, 2048, 256, 512, {}, {}),                                  # saturated, 16-byte loads
    "lowrank_ragged": (1, 2048, 32, 128, {"h": 20.0, "tol": 1e-6}, {"max_rank": 118}),   # odd sizes: scalar loads
    "one_leaf": (1, 64, 64, 128, {}, {}),
}


def _dev(a):
    import torch
    return torch.tensor(np.ascontiguousarray(a), device="cuda:0")


def _rel(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)


@pytest.fixture(scope="module", params=list(CASES))
def prob(request):
    from gpu_helpers import oracle_hss_from_export
    cfg, n, leaf, s, over, opts = CASES[request.param]
    w = synth.make_workload(cfg, n=n, leaf=leaf, s=s)
    for k, v in over.items():
        setattr(w, k, v)
    ctx = binding.Context()
    for k, v in opts.items():
        ctx.hss_set_i64(k, v)
    ctx.hss_compress(_dev(w.F), _dev(w.y), w.h, w.leaf, w.tol, _dev(w.omega()))
    exp = ctx.hss_export()
    H = oracle_hss_from_export(exp)
    yield w, ctx, exp["perm"], H
    ctx.close()


@pytest.mark.parametrize("nrhs", [1, 2, 3, 4, 5, 7])
def test_multi_rhs_solve(prob, nrhs):
    w, ctx, perm, H = prob
    ctx.hss_ulv_factor(w.beta)
    rng = np.random.default_rng(nrhs)
    Bm = rng.standard_normal((nrhs, w.n))
    X = _dev(Bm)
    ctx.hss_ulv_solve(X)
    X = X.cpu().numpy()
    Fz = oulv.ulv_factor(H, w.beta)
    for j in range(nrhs):
        one = _dev(Bm[j])
        ctx.hss_ulv_solve(one)
        assert _rel(X[j], one.cpu().numpy()) <= 1e-13, j          # same arithmetic per column
        ref = np.empty(w.n)
        ref[perm] = oulv.ulv_solve(Fz, Bm[j][perm])
        assert _rel(X[j], ref) <= 1e-10, j


@pytest.mark.parametrize("Cs", [[0.1, 1.0, 10.0, 100.0], [1.0, 10.0], [0.5, 2.0, 8.0], [3.0], [0.1, 0.3, 1.0, 3.0, 10.0]])
def test_c_sweep_equals_single_runs_and_oracle(prob, Cs):
    w, ctx, perm, H = prob
    iters = 25
    beta = 2.0
    multi = ctx.admm_svm_train_multi(Cs, beta, iters)
    yp = w.y[perm]
    Fz = oulv.ulv_factor(H, beta)
    for j, Cj in enumerate(Cs):
        single = ctx.admm_svm_train(Cj, beta, iters)
        oref = oadmm.admm(lambda t: oulv.ulv_solve(Fz, t), yp, Cj, beta, iters)
        for key in ("x", "z", "mu"):
            got = multi[key][j].cpu().numpy()
            assert _rel(got, single[key].cpu().numpy()) <= 1e-12, (key, j)
            assert _rel(got[perm], oref[key]) <= 1e-6, (key, j)
        assert multi["n_margin"][j] == single["n_margin"]
        assert abs(multi["bias"][j] - single["bias"]) <= 1e-10 * max(1.0, abs(single["bias"]))
        b_ref, cnt = oadmm.bias(oref["z"], yp, Cj, lambda t: ohss.matvec(H, t))
        if cnt == multi["n_margin"][j]:
            assert abs(multi["bias"][j] - b_ref) <= 1e-6 * max(1.0, abs(b_ref))


def test_c_sweep_rejects_bad_arguments(prob):
    w, ctx, perm, H = prob
    for Cs in ([1.0, -1.0], [0.0]):
        with pytest.raises(binding.HssError) as e:
            ctx.admm_svm_train_multi(Cs, 1.0, 3)
        assert e.value.code == binding.HSS_EINVAL
