"""Pins for oracle.hss and oracle.ulv (CPU only): everything is checked against
dense linear algebra on small inputs, closed forms, or special cases."""
import numpy as np
import pytest

from oracle import hss, ulv
from oracle.kernel import gaussian_kernel
from oracle.tree import cluster_tree


def _points(n, r, seed):
    rng = np.random.default_rng(seed)
    F = rng.standard_normal((n, r))
    return F, rng


def _compress(n, r, h, leaf, s, rel, seed=0, abs_tol=0.0, kmax=None):
    F, rng = _points(n, r, seed)
    perm = cluster_tree(F, leaf)
    Fp = F[perm]
    Om = rng.standard_normal((n, s))
    H = hss.compress(Fp, h, leaf, Om, rel, abs_tol, kmax)
    return Fp, Om, H, rng


def test_sample_is_K_times_omega():
    F, rng = _points(300, 3, 0)
    Om = rng.standard_normal((300, 7))
    S = hss.sample(F, Om, 1.3, block=64)
    assert np.allclose(S, gaussian_kernel(F, F, 1.3) @ Om, rtol=1e-13, atol=1e-13)


def test_row_id_exact_low_rank():
    rng = np.random.default_rng(1)
    A = rng.standard_normal((40, 6)) @ rng.standard_normal((6, 25))
    J, U = hss.row_id(A, 1e-10, 0.0, 25)
    assert J.size == 6 and U.shape == (40, 6)
    assert np.array_equal(U[J], np.eye(6))
    assert np.linalg.norm(A - U @ A[J]) <= 1e-10 * np.linalg.norm(A)
    assert np.abs(U).max() <= 10.0


def test_row_id_tolerance_and_cap():
    rng = np.random.default_rng(2)
    Qa, _ = np.linalg.qr(rng.standard_normal((30, 30)))
    Qb, _ = np.linalg.qr(rng.standard_normal((30, 30)))
    sv = 10.0 ** -np.arange(30)
    A = (Qa * sv) @ Qb.T
    J, U = hss.row_id(A, 1e-5, 0.0, 30)
    err = np.linalg.norm(A - U @ A[J], 2)
    assert 4 <= J.size <= 8
    assert err <= 1e-3                      # ID error is within a modest factor of the cut-off
    J2, _ = hss.row_id(A, 1e-5, 0.0, 3)
    assert J2.size == 3                      # rank cap
    J3, _ = hss.row_id(A, 0.0, 1e-2, 30)     # absolute threshold
    assert 2 <= J3.size <= 4
    J4, U4 = hss.row_id(np.zeros((5, 4)), 1e-3, 0.0, 4)
    assert J4.size == 0 and U4.shape == (5, 0)


@pytest.mark.parametrize("n,r,h,leaf,s,tol", [
    (1024, 2, 1.5, 32, 128, 1e-4),
    (512, 3, 2.0, 64, 128, 1e-6),
    (256, 2, 0.8, 16, 64, 1e-3),
])
def test_reconstruction_error_within_tolerance(n, r, h, leaf, s, tol):
    Fp, Om, H, _ = _compress(n, r, h, leaf, s, tol / 10.0, kmax=s - 10)
    K = gaussian_kernel(Fp, Fp, h)
    Kt = hss.densify(H)
    assert np.array_equal(Kt, Kt.T)
    err = np.linalg.norm(K - Kt) / np.linalg.norm(K)
    assert err <= tol, (err, H.ranks().max())
    assert H.ranks().max() < s - 10          # the sample was wide enough: no saturation
    for i in range(n // leaf):               # diagonal blocks are entries of K itself
        blk = slice(i * leaf, (i + 1) * leaf)
        assert np.array_equal(Kt[blk, blk], K[blk, blk])


def test_exact_when_sample_is_wide_and_tolerance_tiny():
    n, leaf, h = 256, 32, 1.0
    Fp, Om, H, _ = _compress(n, 3, h, leaf, n, 1e-15)
    K = gaussian_kernel(Fp, Fp, h)
    assert np.linalg.norm(K - hss.densify(H)) <= 1e-10 * np.linalg.norm(K)


def test_rank_one_limit():
    Fp, Om, H, _ = _compress(256, 3, 1e7, 32, 32, 1e-8)
    rk = H.ranks()
    assert np.all(rk[1:] == 1)
    assert np.allclose(hss.densify(H), 1.0, atol=1e-10)


def test_identity_limit_gives_zero_ranks():
    Fp, Om, H, _ = _compress(128, 3, 1e-4, 16, 32, 1e-8)
    assert np.all(H.ranks() == 0)
    assert np.array_equal(hss.densify(H), np.eye(128))


def test_matvec_equals_dense_product():
    for (n, leaf, tol) in [(512, 32, 1e-3), (256, 64, 1e-1), (64, 64, 1e-3)]:
        Fp, Om, H, rng = _compress(n, 3, 1.2, leaf, min(n, 96), tol)
        x = rng.standard_normal(n)
        ref = hss.densify(H) @ x
        assert np.linalg.norm(hss.matvec(H, x) - ref) <= 1e-12 * np.linalg.norm(ref)


@pytest.mark.parametrize("n,r,h,leaf,s,tol,beta", [
    (1024, 3, 1.5, 32, 96, 1e-5, 1.0),
    (512, 4, 1.0, 64, 64, 1e-1, 0.5),     # loose: K~ is a poor copy of K, the solve must still be exact for K~
    (256, 2, 2.0, 16, 64, 1e-8, 2.0),
    (512, 6, 0.7, 32, 128, 1e-12, 1.0),   # leaves are full rank (k = m): nothing eliminated there
])
def test_ulv_solve_equals_dense_solve(n, r, h, leaf, s, tol, beta):
    Fp, Om, H, rng = _compress(n, r, h, leaf, s, tol, kmax=s - 8)
    A = hss.densify(H) + beta * np.eye(n)
    Fz = ulv.ulv_factor(H, beta)
    b = rng.standard_normal(n)
    x = ulv.ulv_solve(Fz, b)
    ref = np.linalg.solve(A, b)
    assert np.linalg.norm(x - ref) <= 1e-10 * np.linalg.norm(ref)
    B = rng.standard_normal((n, 3))
    X = ulv.ulv_solve(Fz, B)
    assert np.linalg.norm(X - np.linalg.solve(A, B)) <= 1e-10 * np.linalg.norm(X)


def test_ulv_full_rank_leaves_case_really_has_them():
    Fp, Om, H, _ = _compress(512, 6, 0.7, 32, 128, 1e-12, kmax=120)
    fl = H.first_leaf()
    assert all(H.rank(t) == 32 for t in range(fl, H.nnodes))


def test_ulv_one_leaf_is_dense_lu():
    n = 64
    Fp, Om, H, rng = _compress(n, 3, 1.0, n, 16, 1e-3)
    assert H.L == 0 and H.nnodes == 1
    K = gaussian_kernel(Fp, Fp, 1.0)
    b = rng.standard_normal(n)
    x = ulv.ulv_solve(ulv.ulv_factor(H, 0.3), b)
    assert np.allclose(x, np.linalg.solve(K + 0.3 * np.eye(n), b), rtol=1e-11, atol=1e-12)


def test_ulv_sherman_morrison_limit():
    # h -> infinity: K = e e^T, (e e^T + beta I)^{-1} = (I - e e^T/(beta + n))/beta
    n, beta = 256, 0.7
    Fp, Om, H, rng = _compress(n, 3, 1e7, 32, 32, 1e-8)
    b = rng.standard_normal(n)
    x = ulv.ulv_solve(ulv.ulv_factor(H, beta), b)
    ref = (b - b.sum() / (beta + n)) / beta
    assert np.linalg.norm(x - ref) <= 1e-9 * np.linalg.norm(ref)


def test_ulv_identity_limit():
    n, beta = 128, 2.0
    Fp, Om, H, rng = _compress(n, 3, 1e-4, 16, 32, 1e-8)
    b = rng.standard_normal(n)
    x = ulv.ulv_solve(ulv.ulv_factor(H, beta), b)
    assert np.allclose(x, b / (1.0 + beta), rtol=1e-14)


def test_planted_mistakes_are_caught():
    """A transposed B or a dropped Schur term must move the answers by far more
    than the pins' tolerances (guards the pins' sensitivity, on the CPU)."""
    n, beta = 256, 1.0
    Fp, Om, H, rng = _compress(n, 3, 1.5, 32, 64, 1e-6)
    A = hss.densify(H) + beta * np.eye(n)
    b = rng.standard_normal(n)
    ref = np.linalg.solve(A, b)
    # transpose one B generator (k_a == k_b needed for shapes to stay valid)
    t = next(t for t in range(H.first_leaf()) if H.B[t].shape[0] == H.B[t].shape[1])
    keep = H.B[t]
    H.B[t] = keep.T.copy()
    x_bad = ulv.ulv_solve(ulv.ulv_factor(H, beta), b)
    y_bad = hss.matvec(H, b)
    H.B[t] = keep
    assert np.linalg.norm(x_bad - ref) > 1e-6 * np.linalg.norm(ref)
    assert np.linalg.norm(y_bad - (A - beta * np.eye(n)) @ b) > 1e-6 * np.linalg.norm(b)


def test_psd_shift_restores_definiteness_and_is_zero_when_not_needed():
    # saturated ranks: the compressed matrix is indefinite, the guard repairs it
    Fp, Om, H, _ = _compress(1024, 8, 1.5, 64, 64, 1e-5, kmax=54)
    lam = np.linalg.eigvalsh(hss.densify(H))[0]
    assert lam < -1.0
    delta = hss.psd_shift(H)
    assert -lam <= delta <= 1.2 * -lam
    hss.add_diagonal(H, delta)
    assert np.linalg.eigvalsh(hss.densify(H))[0] >= 0.0
    # accurate compression of a well-conditioned kernel: no shift
    Fp, Om, H2, _ = _compress(512, 2, 0.05, 32, 128, 1e-8, kmax=118)
    assert np.linalg.eigvalsh(hss.densify(H2))[0] > 0
    assert hss.psd_shift(H2) == 0.0


# ---- adaptive sample width (oversampling / truncation to the tolerance, end of Sec. 3.2) ----

def _adaptive_case(n, r, h, leaf, s, seed=0):
    F, rng = _points(n, r, seed)
    perm = cluster_tree(F, leaf)
    Fp = F[perm]
    Om = rng.standard_normal((n, s))
    return Fp, Om, gaussian_kernel(Fp, Fp, h)


def test_adaptive_equals_fixed_width_when_it_starts_at_the_full_width():
    Fp, Om, K = _adaptive_case(512, 3, 1.5, 32, 96)
    H0 = hss.compress(Fp, 1.5, 32, Om, 1e-5, 0.0, 96 - 48)
    H1, info = hss.compress_adaptive(Fp, 1.5, 32, Om, 1e-5, 0.0)
    assert info["width"] == 96 and info["redone"] == 0
    assert np.array_equal(H0.ranks(), H1.ranks())
    assert np.array_equal(hss.densify(H0), hss.densify(H1))
    # ... and when the first width is already enough (nothing is cut), the extra columns are never looked at
    H2, info2 = hss.compress_adaptive(Fp, 1.5, 32, Om, 1e-2, 0.0, s0=64, step=16, oversample=10)
    H3 = hss.compress(Fp, 1.5, 32, Om[:, :64], 1e-2, 0.0, 54)
    assert info2["width"] == 64 and info2["redone"] == 0 and info2["nodes_at_cap"] == 0
    assert np.array_equal(hss.densify(H2), hss.densify(H3))


def test_adaptive_width_meets_the_tolerance_where_the_first_width_cannot():
    n, r, h, leaf, tol = 1024, 2, 1.0, 32, 1e-6
    Fp, Om, K = _adaptive_case(n, r, h, leaf, 256, seed=3)
    nrm = np.linalg.norm(K)
    # first width alone: every upper node is cut by the cap, the tolerance is missed by orders of magnitude
    Hf = hss.compress(Fp, h, leaf, Om[:, :32], tol / 10.0, 0.0, 22)
    err_fixed = np.linalg.norm(K - hss.densify(Hf)) / nrm
    assert err_fixed > 100 * tol
    Ha, info = hss.compress_adaptive(Fp, h, leaf, Om, tol / 10.0, 0.0, s0=32, step=32, oversample=10)
    err = np.linalg.norm(K - hss.densify(Ha)) / nrm
    assert info["nodes_at_cap"] == 0 and info["redone"] > 0
    assert err <= tol, (err, info)
    assert 32 < info["width"] < 256                      # it grew, and stopped before using every column
    assert Ha.ranks().max() < info["width"] - 10         # every rank is below the cap of the final width
    widths = [info["level_width"][l] for l in range(Ha.L, 0, -1)]
    assert widths == sorted(widths)                      # never shrinks on the way up
    for i in range(n // leaf):
        blk = slice(i * leaf, (i + 1) * leaf)
        assert np.array_equal(hss.densify(Ha)[blk, blk], K[blk, blk])


def test_adaptive_width_trajectory_on_known_ranks():
    """h -> infinity: K = e e^T up to 1e-14, every block has rank one; with oversampling p = 3 a first width of
    4 (cap 1) cuts every node although its rank IS one (a cap that is reached counts as a cut), one step to
    width 6 (cap 3) settles it: all ranks 1, exactly one widening, at the leaf level only."""
    Fp, Om, K = _adaptive_case(256, 3, 1e7, 32, 12)
    H, info = hss.compress_adaptive(Fp, 1e7, 32, Om, 1e-8, 0.0, s0=4, step=2, oversample=3)
    assert np.all(H.ranks()[1:] == 1)
    assert info["width"] == 6 and info["redone"] == 8 and info["nodes_at_cap"] == 0
    assert info["level_width"] == {3: 6, 2: 6, 1: 6}
    assert np.allclose(hss.densify(H), 1.0, atol=1e-10)


def test_adaptive_width_stops_at_the_last_column_and_reports_the_cut():
    Fp, Om, K = _adaptive_case(512, 6, 1.0, 32, 64, seed=5)      # ranks far above what 64 columns can show
    H, info = hss.compress_adaptive(Fp, 1.0, 32, Om, 1e-9, 0.0, s0=32, step=16)
    assert info["width"] == 64 and info["nodes_at_cap"] > 0
    assert H.ranks().max() == 32                                   # cap at the full width: 64 - 64 // 2
    # identical to the fixed-width construction at the full width for the nodes of the last level decomposed
    Hf = hss.compress(Fp, 1.0, 32, Om, 1e-9, 0.0, 32)
    assert np.array_equal(H.ranks(), Hf.ranks())
