"""Gaussian kernel, written out from its definition (oracle; test infrastructure).

K(f, g) = exp(-||f - g||^2 / (2 h^2))  -- the kernel the paper's experiments use
(Sec. 1.1 and Sec. 3.3; the printed subscript "f_i - f_i" is a typo for
"f_i - f_j": K_ii = 1 and K is symmetric).
"""
import numpy as np


def gaussian_kernel(F, G, h, block=1024):
    """K[i, j] = exp(-sum_f (F[i,f]-G[j,f])^2 / (2 h^2)) by direct differences.

    F: (a, r), G: (b, r) float64.  Returns (a, b) float64.  Row-blocked only to
    bound memory; the arithmetic is the definition, one feature at a time.
    """
    F = np.asarray(F, dtype=np.float64)
    G = np.asarray(G, dtype=np.float64)
    a, r = F.shape
    b = G.shape[0]
    out = np.empty((a, b), dtype=np.float64)
    inv = 1.0 / (2.0 * h * h)
    for i0 in range(0, a, block):
        i1 = min(a, i0 + block)
        d2 = np.zeros((i1 - i0, b), dtype=np.float64)
        for f in range(r):
            diff = F[i0:i1, f][:, None] - G[:, f][None, :]
            d2 += diff * diff
        out[i0:i1] = np.exp(-d2 * inv)
    return out
