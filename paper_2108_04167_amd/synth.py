"""Seeded synthetic inputs shaped like the paper's workloads (Table 1 of the paper).

This module only draws random numbers and labels; it contains none of the
method's arithmetic (no kernel, no HSS, no ADMM).  It is the one module that
both the CPU oracle's tests and the HIP path's tests/bench are allowed to
share, so that both sides see byte-identical inputs.

The five workloads stand in for the LIBSVM-site datasets the paper uses
(cod.rna's 8 features, ijcnn1's 22 features / ~5e4 points, susy's 18 features,
webspam.uni's ~2.5e5 points); no record of any of those datasets is reproduced.
"""
from __future__ import annotations

import dataclasses

import numpy as np


@dataclasses.dataclass
class Workload:
    name: str
    F: np.ndarray          # (n, r) training features, float64, point-major
    y: np.ndarray          # (n,) labels in {-1.0, +1.0}
    F_test: np.ndarray     # (n_test, r)
    y_test: np.ndarray     # (n_test,)
    h: float               # Gaussian kernel width
    C: float               # box bound of the dual QP
    leaf: int              # HSS leaf size m
    tol: float             # HSS relative tolerance
    s: int                 # random sample width
    beta: float            # ADMM penalty
    maxit: int             # ADMM iterations
    seed: int
    C_grid: tuple = ()     # hyper-parameter sweep (workload 5)
    beta_grid: tuple = ()

    @property
    def n(self) -> int:
        return self.F.shape[0]

    @property
    def r(self) -> int:
        return self.F.shape[1]

    def omega(self) -> np.ndarray:
        """The (n, s) Gaussian test matrix of this workload (own stream)."""
        rng = np.random.Generator(np.random.PCG64([self.seed, 0x5EED, 4]))
        return rng.standard_normal((self.n, self.s))


def _sign(v: np.ndarray) -> np.ndarray:
    """sign with sign(0) = +1, as float64."""
    return np.where(v >= 0.0, 1.0, -1.0)


def _streams(seed: int, cfg: int):
    """Independent streams: train features, train label noise, test features,
    test label noise, model parameters."""
    ss = np.random.SeedSequence([seed, cfg])
    return [np.random.Generator(np.random.PCG64(c)) for c in ss.spawn(5)]


def _n_test(n: int) -> int:
    return max(16, min(n // 4, 16384))


def _cfg1(n, seed):
    g = _streams(seed, 1)
    r = 8

    def draw(gf, gn, k):
        F = gf.standard_normal((k, r))
        y = _sign(np.sin(F[:, 0]) + F[:, 1] * F[:, 2] + 0.3 * gn.standard_normal(k))
        return F, y

    F, y = draw(g[0], g[1], n)
    Ft, yt = draw(g[2], g[3], _n_test(n))
    return Workload("cfg1", F, y, Ft, yt, h=1.5, C=1.0, leaf=64, tol=1e-4, s=128,
                    beta=1.0, maxit=200, seed=seed)


def _cfg2(n, seed):
    g = _streams(seed, 2)
    r = 22

    def draw(gf, gn, k):
        c = np.where(gf.random(k) < 0.5, -1.0, 1.0)
        F = 0.5 * c[:, None] + gf.standard_normal((k, r))
        flip = gn.random(k) < 0.05
        return F, np.where(flip, -c, c)

    F, y = draw(g[0], g[1], n)
    Ft, yt = draw(g[2], g[3], _n_test(n))
    mu = F.mean(axis=0)
    sd = F.std(axis=0)
    F = (F - mu) / sd
    Ft = (Ft - mu) / sd
    return Workload("cfg2", F, y, Ft, yt, h=2.0, C=10.0, leaf=128, tol=1e-3, s=256,
                    beta=1.0, maxit=500, seed=seed)


def _cfg3(n, seed):
    g = _streams(seed, 3)
    r, rc = 54, 10
    W1 = g[4].standard_normal((16, r))
    w2 = g[4].standard_normal(16)

    def draw(gf, gn, k):
        F = np.empty((k, r))
        F[:, :rc] = gf.standard_normal((k, rc))
        F[:, rc:] = (gf.random((k, r - rc)) < 0.1).astype(np.float64)
        lab = _sign(np.tanh(F @ W1.T) @ w2)
        flip = gn.random(k) < 0.03
        return F, np.where(flip, -lab, lab)

    F, y = draw(g[0], g[1], n)
    Ft, yt = draw(g[2], g[3], _n_test(n))
    return Workload("cfg3", F, y, Ft, yt, h=3.0, C=1.0, leaf=256, tol=1e-3, s=512,
                    beta=1.0, maxit=500, seed=seed)


def _cfg4(n, seed):
    g = _streams(seed, 4)
    r = 18

    def draw(gf, gn, k):
        F = gf.uniform(-1.0, 1.0, size=(k, r))
        y = _sign((F[:, :4] ** 2).sum(axis=1) - 1.33 + 0.2 * gn.standard_normal(k))
        return F, y

    F, y = draw(g[0], g[1], n)
    Ft, yt = draw(g[2], g[3], _n_test(n))
    return Workload("cfg4", F, y, Ft, yt, h=1.0, C=10.0, leaf=256, tol=1e-2, s=512,
                    beta=1.0, maxit=300, seed=seed)


def _cfg5(n, seed):
    g = _streams(seed, 5)
    r = 90
    a = g[4].standard_normal(r)

    def draw(gf, gn, k):
        F = gf.standard_normal((k, r))
        lab = _sign(F @ a / np.sqrt(r) + 0.5 * (F[:, 0] * F[:, 1] + F[:, 2] ** 2 - 1.0))
        flip = gn.random(k) < 0.05
        return F, np.where(flip, -lab, lab)

    F, y = draw(g[0], g[1], n)
    Ft, yt = draw(g[2], g[3], _n_test(n))
    return Workload("cfg5", F, y, Ft, yt, h=4.0, C=1.0, leaf=256, tol=1e-3, s=512,
                    beta=1.0, maxit=300, seed=seed,
                    C_grid=(0.1, 1.0, 10.0, 100.0), beta_grid=(0.5, 1.0, 2.0))


_FULL_N = {1: 2048, 2: 65536, 3: 262144, 4: 1048576, 5: 262144}
_MAKERS = {1: _cfg1, 2: _cfg2, 3: _cfg3, 4: _cfg4, 5: _cfg5}


def make_workload(cfg: int, n: int | None = None, seed: int = 0, *,
                  leaf: int | None = None, s: int | None = None) -> Workload:
    """Workload `cfg` (1..5).  `n`, `leaf`, `s` shrink it for parity tests that
    must finish in seconds; the default is the full size."""
    if cfg not in _MAKERS:
        raise ValueError(f"cfg must be 1..5, got {cfg}")
    w = _MAKERS[cfg](_FULL_N[cfg] if n is None else int(n), seed)
    if leaf is not None:
        w.leaf = int(leaf)
    if s is not None:
        w.s = int(s)
    w.F = np.ascontiguousarray(w.F, dtype=np.float64)
    w.F_test = np.ascontiguousarray(w.F_test, dtype=np.float64)
    w.y = np.ascontiguousarray(w.y, dtype=np.float64)
    w.y_test = np.ascontiguousarray(w.y_test, dtype=np.float64)
    return w
