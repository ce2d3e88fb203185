"""Pins for oracle.admm and oracle.qp (CPU only)."""
import numpy as np
import pytest

from oracle import admm, hss, qp, ulv
from oracle.kernel import gaussian_kernel
from oracle.tree import cluster_tree


def _problem(n, r, h, seed, noise=0.3):
    rng = np.random.default_rng(seed)
    F = rng.standard_normal((n, r))
    y = np.where(np.sin(F[:, 0]) + F[:, 1] * F[:, 2 % r] + noise * rng.standard_normal(n) >= 0, 1.0, -1.0)
    return F, y, gaussian_kernel(F, F, h), rng


def test_x_update_solves_the_bordered_kkt_system():
    """Sec. 2.1: x^{k+1} is the x-part of  [[Y K_beta Y, -y], [-y^T, 0]] [x; lambda] = [q^k; 0]  with
    q^k = e + mu^k + beta z^k.  The oracle's own trajectory is used: k iterations give (z^k, mu^k), k + 1
    iterations give x^{k+1}; the bordered system is solved densely, with no use of the closed form."""
    n, beta, C = 96, 0.8, 0.6
    F, y, K, rng = _problem(n, 3, 1.5, 0)
    Kb = K + beta * np.eye(n)
    big = np.zeros((n + 1, n + 1))
    big[:n, :n] = (y[:, None] * Kb) * y[None, :]
    big[:n, n] = -y
    big[n, :n] = -y
    for k in (0, 1, 2, 7, 30):
        prev = admm.admm_dense(K, y, C, beta, k)
        nxt = admm.admm_dense(K, y, C, beta, k + 1)
        q = 1.0 + prev["mu"] + beta * prev["z"]
        ref = np.linalg.solve(big, np.concatenate([q, [0.0]]))[:n]
        assert np.allclose(nxt["x"], ref, rtol=1e-10, atol=1e-11), k
        assert abs(y @ nxt["x"]) < 1e-10
        # the other two updates of Algorithm 2, from the same pair of states
        assert np.array_equal(nxt["z"], np.clip(nxt["x"] - prev["mu"] / beta, 0.0, C))          # eq. (6)
        assert np.allclose(nxt["mu"], prev["mu"] - beta * (nxt["x"] - nxt["z"]), rtol=0, atol=1e-15)
    assert np.abs(prev["mu"]).max() > 1e-3 and (prev["z"] > 0).any()     # the states fed back are not trivial
    # a trajectory that ignored the feedback of z and mu (the misprint in Algorithm 3) would fail this
    stale = 1.0 + 0.0 * prev["mu"]
    bad = np.linalg.solve(big, np.concatenate([stale, [0.0]]))[:n]
    assert not np.allclose(nxt["x"], bad, rtol=1e-3, atol=1e-4)


def test_first_iteration_matches_hand_formula_and_invariants():
    n, beta, C = 80, 1.0, 0.7
    F, y, K, _ = _problem(n, 3, 1.2, 1)
    out1 = admm.admm_dense(K, y, C, beta, 1)
    Kb = K + beta * np.eye(n)
    e = np.ones(n)
    Kinv_e = np.linalg.solve(Kb, e)
    Kinv_y = np.linalg.solve(Kb, y)          # q^0 = e, Y e = y
    x1 = y * Kinv_y - (e @ Kinv_y) / (e @ Kinv_e) * (y * Kinv_e)
    assert np.allclose(out1["x"], x1, rtol=1e-12, atol=1e-13)
    z1 = np.clip(x1, 0.0, C)                  # mu^0 = 0
    assert np.array_equal(out1["z"], z1) or np.allclose(out1["z"], z1, atol=1e-15)
    assert np.allclose(out1["mu"], -beta * (x1 - z1), atol=1e-14)
    out = admm.admm_dense(K, y, C, beta, 60, history=True)
    assert np.max(np.abs(out["ytx"])) < 1e-10           # y^T x^k = 0 every iteration
    assert out["z"].min() >= 0.0 and out["z"].max() <= C


def test_exact_qp_solver_is_certified_by_kkt():
    n, C = 120, 1.0
    F, y, K, _ = _problem(n, 3, 1.5, 2)
    x, b, it = qp.solve_qp(K, y, C, eps=1e-12)
    res = qp.kkt_residuals(K, y, C, x, b)
    assert res["eq"] < 1e-11 and res["box"] == 0.0 and res["stat"] < 1e-10
    free = (x > 0) & (x < C)
    assert free.sum() >= 3
    # margin identity: decision value on every margin support vector is exactly y_j
    dec = K @ (y * x) + b
    assert np.max(np.abs(y[free] * dec[free] - 1.0)) < 1e-9
    # a wrong-signed bias breaks the certificate
    assert qp.kkt_residuals(K, y, C, x, -b)["stat"] > 1e-3 or abs(b) < 1e-3


def test_qp_agrees_with_an_independent_library_solver():
    sklearn_svm = pytest.importorskip("sklearn.svm")
    n, C = 100, 1.0
    F, y, K, _ = _problem(n, 3, 1.5, 3)
    x, b, _ = qp.solve_qp(K, y, C, eps=1e-12)
    clf = sklearn_svm.SVC(C=C, kernel="precomputed", tol=1e-10, shrinking=False)
    clf.fit(K, y)
    xs = np.zeros(n)
    xs[clf.support_] = np.abs(clf.dual_coef_[0])
    assert np.max(np.abs(xs - x)) < 2e-5      # the library stops at its own, looser, criterion
    assert abs(clf.intercept_[0] - b) < 2e-5


def test_admm_converges_to_the_qp_solution_and_bias_sign():
    n, C, beta = 120, 1.0, 1.0
    F, y, K, _ = _problem(n, 3, 1.5, 2)
    xq, bq, _ = qp.solve_qp(K, y, C, eps=1e-12)
    out = admm.admm_dense(K, y, C, beta, 20000)
    assert np.max(np.abs(out["z"] - xq)) < 5e-6
    assert np.max(np.abs(out["x"] - out["z"])) < 1e-6
    b, cnt = admm.bias(out["z"], y, C, lambda v: K @ v)
    assert cnt == int(((out["z"] > 0) & (out["z"] < C)).sum())
    assert abs(b - bq) < 1e-4
    # the formula as printed in eq. (2)/(7) has the opposite sign
    M = admm.margin_set(out["z"], C)
    printed = ((y * out["z"]) @ (K @ M.astype(float)) - y[M].sum()) / M.sum()
    assert abs(printed + bq) < 1e-4 and abs(bq) > 1e-3


def test_bias_empty_margin_set():
    b, cnt = admm.bias(np.array([0.0, 1.0, 1.0]), np.array([1.0, -1.0, 1.0]), 1.0, lambda v: v)
    assert (b, cnt) == (0.0, 0)


def test_identity_kernel_closed_form():
    # h -> 0: K = I, x-update = (q - y (y^T q)/n)/(1+beta)
    n, beta, C = 64, 0.5, 2.0
    rng = np.random.default_rng(5)
    y = np.where(rng.random(n) < 0.5, -1.0, 1.0)
    out = admm.admm_dense(np.eye(n), y, C, beta, 1)
    q = np.ones(n)
    assert np.allclose(out["x"], (q - y * (y @ q) / n) / (1 + beta), rtol=1e-13, atol=1e-14)


def test_error_bound_eq9():
    """|f(xbar) - f~(xtilde)| <= 1/2 max(|xtilde|^2, |xbar|^2) ||K~ - K||_2.  The bound needs
    both problems convex; a loose K~ is indefinite, so both matrices get the same
    ridge (which leaves K~ - K unchanged and keeps K a valid kernel matrix)."""
    n, C, h, ridge = 128, 1.0, 0.5, 0.2
    rng = np.random.default_rng(6)
    F = rng.standard_normal((n, 3))
    perm = cluster_tree(F, 16)
    Fp = F[perm]
    y = np.where(np.sin(Fp[:, 0]) + Fp[:, 1] * Fp[:, 2] >= 0, 1.0, -1.0)
    K = gaussian_kernel(Fp, Fp, h) + ridge * np.eye(n)
    H = hss.compress(Fp, h, 16, rng.standard_normal((n, 48)), 3e-2, 0.0, 40)
    Kt = hss.densify(H) + ridge * np.eye(n)
    assert np.linalg.norm(K - Kt, 2) > 1e-2          # a genuinely inexact approximation
    assert np.linalg.eigvalsh(Kt).min() > 0.0
    xb, _, _ = qp.solve_qp(K, y, C, eps=1e-11)
    xt, _, _ = qp.solve_qp(Kt, y, C, eps=1e-11)
    f = lambda KK, x: 0.5 * (y * x) @ KK @ (y * x) - x.sum()
    lhs = abs(f(K, xb) - f(Kt, xt))
    rhs = 0.5 * max(xt @ xt, xb @ xb) * np.linalg.norm(Kt - K, 2)
    assert lhs > 1e-6                                 # the two problems really differ
    assert lhs <= rhs * (1 + 1e-9)


def test_admm_through_ulv_equals_dense_cholesky_admm_when_compression_is_exact():
    n, leaf, h, C, beta = 256, 32, 1.0, 1.0, 1.0
    rng = np.random.default_rng(7)
    F = rng.standard_normal((n, 3))
    perm = cluster_tree(F, leaf)
    Fp = F[perm]
    y = np.where(np.sin(Fp[:, 0]) + Fp[:, 1] * Fp[:, 2] >= 0, 1.0, -1.0)
    H = hss.compress(Fp, h, leaf, rng.standard_normal((n, n)), 1e-15)
    Fz = ulv.ulv_factor(H, beta)
    a = admm.admm(lambda v: ulv.ulv_solve(Fz, v), y, C, beta, 100)
    d = admm.admm_dense(gaussian_kernel(Fp, Fp, h), y, C, beta, 100)
    for key in ("x", "z", "mu"):
        assert np.linalg.norm(a[key] - d[key]) <= 1e-8 * max(1.0, np.linalg.norm(d[key]))


def test_decision_on_separable_toy_set():
    rng = np.random.default_rng(8)
    n = 80
    F = np.vstack([rng.normal(-2.0, 0.4, (n // 2, 2)), rng.normal(2.0, 0.4, (n // 2, 2))])
    y = np.concatenate([-np.ones(n // 2), np.ones(n // 2)])
    K = gaussian_kernel(F, F, 1.0)
    out = admm.admm_dense(K, y, 10.0, 1.0, 3000)
    b, _ = admm.bias(out["z"], y, 10.0, lambda v: K @ v)
    G = np.vstack([rng.normal(-2.0, 0.4, (50, 2)), rng.normal(2.0, 0.4, (50, 2))])
    yt = np.concatenate([-np.ones(50), np.ones(50)])
    dec = admm.decision(F, y, out["z"], b, G, 1.0, block=32)
    assert admm.accuracy(dec, yt) == 100.0
    # direct evaluation of the classifier, one test point at a time
    j = 7
    direct = sum(y[i] * out["z"][i] * np.exp(-np.sum((F[i] - G[j]) ** 2) / 2.0) for i in range(n)) + b
    assert dec[j] == pytest.approx(direct, rel=1e-12)
