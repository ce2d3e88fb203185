"""Oracle pins on HSS matrices that come from NO compression: random generators with ragged ranks (including
nodes that keep all their rows and ranks of one), so that the mat-vec, densify and the ULV factorization/solve
are checked as linear algebra on the HSS form itself -- densify is the definition written out (nested bases,
K~(I_a, I_b) = Uh_a B_ab Uh_b^T), the ULV solve must equal a dense solve of it."""
import numpy as np
import pytest

from oracle import hss as ohss
from oracle import ulv as oulv


def random_hss(seed, leaf, L, dense_bases=False):
    g = np.random.default_rng(seed)
    n = leaf << L
    H = ohss.HSS(n, leaf)
    H.D = []
    for _ in range(n // leaf):
        A = g.standard_normal((leaf, leaf))
        H.D.append(A + A.T + 2.0 * leaf * np.eye(leaf))        # symmetric, diagonally dominant
    for t in range(H.nnodes - 1, 0, -1):
        m = H.size(t)
        k = int(g.integers(1, m + 1)) if g.random() < 0.8 else m      # sometimes the node keeps everything
        if dense_bases:
            H.U[t] = g.standard_normal((m, k)) / np.sqrt(m)
            H.J[t] = np.arange(k)
        else:
            J = g.permutation(m)[:k]
            U = g.uniform(-1.0, 1.0, size=(m, k)) * 0.5
            U[J] = np.eye(k)
            H.U[t], H.J[t] = U, J
    for t in range(H.first_leaf()):
        ka, kb = H.rank(2 * t + 1), H.rank(2 * t + 2)
        H.B[t] = g.standard_normal((ka, kb)) * 0.3
    return H


@pytest.mark.parametrize("seed,leaf,L,dense", [(0, 8, 0, False), (1, 8, 1, False), (2, 6, 3, False), (3, 16, 2, True),
                                               (4, 5, 4, False), (5, 12, 3, True), (6, 32, 2, False)])
def test_matvec_and_ulv_on_random_generators(seed, leaf, L, dense):
    H = random_hss(seed, leaf, L, dense)
    A = ohss.densify(H)
    assert np.allclose(A, A.T, atol=0, rtol=0)
    # densify is the definition: check one off-diagonal block against the nested bases by hand
    if L >= 2:
        Ua, Ub = ohss.nested_basis(H, 3), ohss.nested_basis(H, 4)
        w = H.n >> 2
        assert np.allclose(A[:w, w:2 * w], Ua @ H.B[1] @ Ub.T, atol=1e-14)
    g = np.random.default_rng(100 + seed)
    X = g.standard_normal((H.n, 3))
    for j in range(3):
        assert np.allclose(ohss.matvec(H, X[:, j]), A @ X[:, j], rtol=1e-12, atol=1e-12 * np.abs(A).sum(axis=1).max())
    for beta in (0.5, 7.0):
        M = A + beta * np.eye(H.n)
        cond = np.linalg.cond(M)
        F = oulv.ulv_factor(H, beta)
        ref = np.linalg.solve(M, X)
        got = oulv.ulv_solve(F, X)
        assert np.linalg.norm(got - ref) <= 1e-13 * cond * np.linalg.norm(ref)
        one = oulv.ulv_solve(F, X[:, 0])
        assert one.shape == (H.n,) and np.allclose(one, got[:, 0], rtol=1e-12, atol=1e-14)


def test_add_diagonal_shifts_only_the_leaf_blocks():
    H = random_hss(9, 8, 2)
    A = ohss.densify(H)
    H2 = ohss.add_diagonal(H, 2.5)
    assert np.allclose(ohss.densify(H2), A + 2.5 * np.eye(H.n), atol=1e-14)
