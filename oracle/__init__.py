"""CPU oracle for the ADMM + HSS nonlinear-SVM shifted-kernel-solve path.

THIS PACKAGE IS TEST INFRASTRUCTURE.  It is a plain, slow, float64 NumPy/SciPy
statement of what the path computes, written from the paper (Cipolla & Gondzio,
"Training very large scale nonlinear SVMs using ADMM coupled with HSS kernel
approximations") and from the textbook definitions of the methods the paper
names but does not spell out (randomized HSS compression with interpolative
decompositions, ULV factorization/solve).  Only the tests, the smoke check and
the benchmark's CPU-baseline leg may import it.  It shares no code with the HIP
library and imports nothing from it.

Modules
-------
kernel    Gaussian kernel by direct differences (Sec. 1.1, kernel definition).
tree      balanced coordinate-bisection cluster tree (clustering preprocess).
hss       random sampling S = K*Omega, row interpolative decomposition,
          bottom-up HSS construction, densify, HSS mat-vec.
ulv       ULV factorization of K~ + beta*I and its forward/backward solve.
admm      closed-form ADMM (Algorithm 2 with the precomputation of Algorithm 3),
          averaged bias (eq. 7, sign per the margin identity), label assignment.
qp        exact dual-SVM QP by two-variable analytic updates (pin for ADMM/bias).

Parity status: every function here is pinned by tests/test_oracle_*.py to
something other than itself (dense solves, closed forms, KKT certificates,
special cases).  The *entries* of a compressed matrix (which skeleton rows,
exact ranks) are not unique and are deliberately "parity unpinned": only the
reconstruction error and everything computed from a shared compressed matrix
are compared.
"""
