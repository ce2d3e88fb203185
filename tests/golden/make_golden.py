"""Writes tests/golden/tiny_admm.json from the oracle only (never from the HIP path)."""
import json
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
from oracle import admm, hss, ulv            # noqa: E402
from oracle.tree import cluster_tree          # noqa: E402


def build():
    rng = np.random.Generator(np.random.PCG64(2108))
    n, r, leaf, h, C, beta = 64, 2, 16, 1.0, 1.0, 1.0
    F = rng.standard_normal((n, r))
    y = np.where(F[:, 0] * F[:, 1] >= 0, 1.0, -1.0)
    perm = cluster_tree(F, leaf)
    Fp, yp = F[perm], y[perm]
    H = hss.compress(Fp, h, leaf, rng.standard_normal((n, 32)), 1e-8, 0.0, 32)
    Fz = ulv.ulv_factor(H, beta)
    out = admm.admm(lambda v: ulv.ulv_solve(Fz, v), yp, C, beta, 25)
    b, cnt = admm.bias(out["z"], yp, C, lambda v: hss.matvec(H, v))
    return {"perm_head": perm[:8].tolist(), "ranks": H.ranks().tolist(),
            "z_head": out["z"][:6].tolist(), "x_norm": float(np.linalg.norm(out["x"])),
            "bias": b, "n_margin": cnt}


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_admm.json")
    with open(path, "w") as f:
        json.dump(build(), f, indent=1)
    print("wrote", path)
