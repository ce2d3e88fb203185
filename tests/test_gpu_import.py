"""hss_import (GPU only): the exported generators restore the compressed state exactly, and generators
built by the ORACLE's compression run through the library's factorization, solve, mat-vec and ADMM --
the library on a compressed matrix it did not build, against the oracle on the same one."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import admm as oadmm          # noqa: E402
from oracle import hss as ohss            # noqa: E402
from oracle import ulv as oulv            # noqa: E402
from oracle.tree import cluster_tree      # noqa: E402
from paper_2108_04167_amd import binding, synth   # noqa: E402


def _dev(a):
    import torch
    return torch.tensor(np.ascontiguousarray(a), device="cuda:0")


def _rel(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)


def test_export_import_round_trip_is_exact():
    w = synth.make_workload(3, n=2048, leaf=64, s=128)
    F, y = _dev(w.F), _dev(w.y)
    a = binding.Context()
    a.hss_set_i64("sample_width", w.s)
    a.hss_compress(F, y, w.h, w.leaf, w.tol, _dev(w.omega()))
    gen = a.hss_export()
    b = binding.Context()
    rc = b.hss_import(F, y, w.h, w.leaf, gen)
    assert rc == (binding.HSS_WSHIFT if gen["delta"] > 0 else 0)
    back = b.hss_export()
    for key in ("perm", "sizes", "ranks", "D", "U", "J", "B"):
        assert np.array_equal(gen[key], back[key]), key
    assert back["delta"] == gen["delta"]
    rng = np.random.default_rng(0)
    v = rng.standard_normal(w.n)
    assert np.array_equal(a.hss_matvec(_dev(v)).cpu().numpy(), b.hss_matvec(_dev(v)).cpu().numpy())
    xa, xb = _dev(v), _dev(v)
    a.hss_ulv_factor(w.beta)
    b.hss_ulv_factor(w.beta)
    a.hss_ulv_solve(xa)
    b.hss_ulv_solve(xb)
    assert np.array_equal(xa.cpu().numpy(), xb.cpu().numpy())
    oa = a.admm_svm_train(w.C, w.beta, 20)
    ob = b.admm_svm_train(w.C, w.beta, 20)
    for key in ("x", "z", "mu"):
        assert np.array_equal(oa[key].cpu().numpy(), ob[key].cpu().numpy())
    assert oa["bias"] == ob["bias"] and oa["n_margin"] == ob["n_margin"]
    G = _dev(w.F_test[:256])
    assert np.array_equal(a.svm_decision(G, oa["z"], oa["bias"]).cpu().numpy(),
                          b.svm_decision(G, ob["z"], ob["bias"]).cpu().numpy())
    a.close()
    b.close()


@pytest.mark.parametrize("regime", ["low_rank", "saturated"])
def test_library_on_the_oracles_compressed_matrix(regime):
    from gpu_helpers import export_from_oracle_hss
    if regime == "low_rank":      # wide kernel: ranks well below the block size, ragged from node to node
        w = synth.make_workload(1, n=1024, leaf=64, s=128)
        h, tol, kmax = 20.0, 1e-6, 118
    else:                         # the workloads' regime: every node at the cap
        w = synth.make_workload(2, n=1024, leaf=64, s=128)
        h, tol, kmax = w.h, w.tol, 64
    perm = cluster_tree(w.F, w.leaf)
    H = ohss.compress(w.F[perm], h, w.leaf, w.omega()[perm], tol / 10.0, 1e-8, kmax=kmax)
    delta = ohss.psd_shift(H)
    gen = export_from_oracle_hss(H, perm, delta)
    ranks = gen["ranks"][1:]
    if regime == "low_rank":
        assert (ranks < gen["sizes"][1:]).all() and len(set(ranks[-(w.n // w.leaf):].tolist())) > 1
    Hs = ohss.add_diagonal(H, delta)
    ctx = binding.Context()
    ctx.hss_import(_dev(w.F), _dev(w.y), h, w.leaf, gen)
    rng = np.random.default_rng(1)
    v = rng.standard_normal(w.n)
    mv = ctx.hss_matvec(_dev(v)).cpu().numpy()
    ref = np.empty(w.n)
    ref[perm] = ohss.matvec(Hs, v[perm])
    assert _rel(mv, ref) <= 1e-12
    ctx.hss_ulv_factor(w.beta)
    x = _dev(v)
    ctx.hss_ulv_solve(x)
    Fz = oulv.ulv_factor(Hs, w.beta)
    ref[perm] = oulv.ulv_solve(Fz, v[perm])
    assert _rel(x.cpu().numpy(), ref) <= 1e-10
    out = ctx.admm_svm_train(w.C, w.beta, 40)
    yp = w.y[perm]
    oref = oadmm.admm(lambda t: oulv.ulv_solve(Fz, t), yp, w.C, w.beta, 40)
    for key in ("x", "z", "mu"):
        assert _rel(out[key].cpu().numpy()[perm], oref[key]) <= 1e-6, key
    b_ref, cnt = oadmm.bias(oref["z"], yp, w.C, lambda t: ohss.matvec(Hs, t))
    if cnt == out["n_margin"]:
        assert abs(out["bias"] - b_ref) <= 1e-6 * max(1.0, abs(b_ref))
    ctx.close()


def test_import_rejects_inconsistent_generators():
    import torch
    w = synth.make_workload(1, n=512, leaf=64, s=128)
    F, y = _dev(w.F), _dev(w.y)
    a = binding.Context()
    a.hss_compress(F, y, 20.0, w.leaf, 1e-6, _dev(w.omega()))
    good = a.hss_export()
    a.close()
    assert (good["ranks"][1:] < good["sizes"][1:]).all()

    def broken(**kw):
        g = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in good.items()}
        for k, f in kw.items():
            f(g[k])
        return g

    def set_(i, v):
        def f(a):
            a[i] = v
        return f

    k1 = int(good["ranks"][1])
    cases = {
        "perm not a permutation": broken(perm=set_(0, int(good["perm"][1]))),
        "perm out of range": broken(perm=set_(3, w.n)),
        "leaf size": broken(sizes=set_(len(good["sizes"]) - 1, 32)),
        "inner size": broken(sizes=set_(1, int(good["sizes"][1]) + 1)),
        "zero rank": broken(ranks=set_(2, 0)),
        "root rank": broken(ranks=set_(0, 3)),
        "duplicate skeleton row": broken(J=set_(1, int(good["J"][0]))),
        "skeleton row outside the node": broken(J=set_(0, 4096)),
        "basis not interpolative": broken(U=set_(int(good["J"][0]) * k1, 0.5)),
    }
    for name, g in cases.items():
        ctx = binding.Context()
        with pytest.raises(binding.HssError) as e:
            ctx.hss_import(F, y, 20.0, w.leaf, g)
        assert e.value.code == binding.HSS_EINVAL, name
        ctx.n = w.n
        with pytest.raises(binding.HssError) as e:          # still not compressed
            ctx.hss_matvec(torch.zeros(w.n, dtype=torch.float64, device="cuda:0"))
        assert e.value.code == binding.HSS_ESTATE, name
        ctx.close()
    ctx = binding.Context()
    bad = dict(good)
    bad["delta"] = -1.0
    with pytest.raises(binding.HssError):
        ctx.hss_import(F, y, 20.0, w.leaf, bad)
    ybad = y.clone()
    ybad[0] = 2.0
    with pytest.raises(binding.HssError):
        ctx.hss_import(F, ybad, 20.0, w.leaf, good)
    assert ctx.hss_import(F, y, 20.0, w.leaf, good) >= 0     # and the untouched arrays are accepted
    ctx.close()


@pytest.mark.parametrize("seed,leaf,L", [(11, 16, 3), (12, 32, 2), (13, 16, 0), (14, 48, 3), (15, 64, 4)])
def test_library_on_random_generators(seed, leaf, L):
    """Generators that come from no kernel at all (random interpolative bases, ragged ranks down to 1 and up to
    the node size, random coupling blocks): the library's mat-vec and ULV solve as pure HSS linear algebra."""
    from gpu_helpers import export_from_oracle_hss
    from test_oracle_random_generators import random_hss
    H = random_hss(seed, leaf, L)
    n = H.n
    g = np.random.default_rng(seed)
    F = g.standard_normal((n, 3))
    y = np.where(g.random(n) < 0.5, -1.0, 1.0)
    perm = g.permutation(n)
    gen = export_from_oracle_hss(H, perm, 0.0)
    ctx = binding.Context()
    ctx.hss_import(_dev(F), _dev(y), 1.0, leaf, gen)
    V = g.standard_normal((3, n))
    for j in range(3):
        mv = ctx.hss_matvec(_dev(V[j])).cpu().numpy()
        ref = np.empty(n)
        ref[perm] = ohss.matvec(H, V[j][perm])
        assert _rel(mv, ref) <= 1e-12
    for beta in (0.5, 7.0):
        ctx.hss_ulv_factor(beta)
        X = _dev(V)
        ctx.hss_ulv_solve(X)
        X = X.cpu().numpy()
        A = ohss.densify(H) + beta * np.eye(n)
        cond = np.linalg.cond(A)
        for j in range(3):
            ref = np.empty(n)
            ref[perm] = np.linalg.solve(A, V[j][perm])
            assert _rel(X[j], ref) <= max(1e-10, 1e-13 * cond), (beta, j, cond)
    ctx.close()
