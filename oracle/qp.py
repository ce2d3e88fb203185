"""Exact solution of the dual SVM QP on tiny inputs (oracle; test infrastructure).

   min 1/2 x^T Y K Y x - e^T x   s.t.  y^T x = 0,  0 <= x <= C          (eq. 1)

Method: repeated exact minimisation over the most-violating pair of variables
(two-variable analytic updates keep y^T x = 0 and the box), run until the KKT
gap is below `eps`.  This is only a pin for the ADMM fixed point and for the
sign of the bias; its own optimality is certified independently by
`kkt_residuals`, which checks the optimality conditions from their definition.
"""
import numpy as np


def solve_qp(K, y, C, eps=1e-12, max_iter=2_000_000, refresh=2000):
    """Returns (x, b, iters).  b is the bias of the classifier
    sign(sum_i y_i x_i K(f_i, .) + b), i.e. minus the multiplier of y^T x = 0."""
    y = np.asarray(y, dtype=np.float64)
    n = y.size
    Q = (y[:, None] * K) * y[None, :]
    x = np.zeros(n)
    g = -np.ones(n)                       # gradient Qx - e
    it = 0
    b = 0.0
    while it < max_iter:
        v = -y * g
        up = ((y > 0) & (x < C)) | ((y < 0) & (x > 0))
        low = ((y > 0) & (x > 0)) | ((y < 0) & (x < C))
        if not up.any() or not low.any():
            break
        i = int(np.argmax(np.where(up, v, -np.inf)))
        j = int(np.argmin(np.where(low, v, np.inf)))
        gap = v[i] - v[j]
        b = 0.5 * (v[i] + v[j])
        if gap <= eps:
            break
        eta = K[i, i] + K[j, j] - 2.0 * K[i, j]
        t = gap / max(eta, 1e-300)
        # x_i += y_i t, x_j -= y_j t, both must stay in [0, C]
        t = min(t, (C - x[i]) if y[i] > 0 else x[i])
        t = min(t, x[j] if y[j] > 0 else (C - x[j]))
        di, dj = y[i] * t, -y[j] * t
        x[i] = min(max(x[i] + di, 0.0), C)
        x[j] = min(max(x[j] + dj, 0.0), C)
        g += Q[:, i] * di + Q[:, j] * dj
        it += 1
        if it % refresh == 0:
            g = Q @ x - 1.0               # remove accumulated rounding drift
    return x, b, it


def kkt_residuals(K, y, C, x, b):
    """Optimality certificate, straight from the conditions of eq. (1).

    With g = Y K Y x - e and bias b (multiplier of y^T x = 0 is -b):
      free   0 < x_i < C :  g_i + b y_i  = 0
      lower  x_i = 0     :  g_i + b y_i >= 0
      upper  x_i = C     :  g_i + b y_i <= 0
    Returns dict(eq=|y^T x|, box=max box violation, stat=max violation of the
    three sign conditions)."""
    y = np.asarray(y, dtype=np.float64)
    g = y * (K @ (y * x)) - 1.0
    r = g + b * y
    free = (x > 0) & (x < C)
    lower = x <= 0
    upper = x >= C
    stat = 0.0
    if free.any():
        stat = max(stat, float(np.abs(r[free]).max()))
    if lower.any():
        stat = max(stat, float(np.maximum(-r[lower], 0).max()))
    if upper.any():
        stat = max(stat, float(np.maximum(r[upper], 0).max()))
    box = float(max(np.maximum(-x, 0).max(), np.maximum(x - C, 0).max()))
    return {"eq": abs(float(y @ x)), "box": box, "stat": stat}
