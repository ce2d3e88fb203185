"""Helpers shared by the GPU tests: access to the library's internal test entry points and the
bridge from an exported compressed matrix to the oracle's HSS container."""
import ctypes as C

import numpy as np

from oracle import hss as ohss
from paper_2108_04167_amd import binding


_hooks = None


def lib():
    """The unit tests' hook library (building blocks of the product library, one call each)."""
    global _hooks
    if _hooks is None:
        import os
        binding.load()
        _hooks = C.CDLL(os.path.join(os.path.dirname(binding.LIB_PATH), "libhsssvm_hooks.so"))
    return _hooks


def dev(a):
    import torch
    return torch.tensor(np.ascontiguousarray(a), device="cuda:0")


def ptr(t):
    return C.c_void_p(t.data_ptr())


def hptr(a):
    return C.c_void_p(a.ctypes.data)


def oracle_hss_from_export(exp, with_shift=True):
    """Oracle HSS container holding exactly the generators the library exported (plus the guard's
    diagonal shift when with_shift)."""
    n, leaf = int(exp["n"]), int(exp["leaf"])
    H = ohss.HSS(n, leaf)
    sizes, ranks = exp["sizes"], exp["ranks"]
    uo = jo = bo = 0
    for t in range(1, H.nnodes):
        m, k = int(sizes[t]), int(ranks[t])
        H.U[t] = exp["U"][uo:uo + m * k].reshape(m, k).copy()
        H.J[t] = exp["J"][jo:jo + k].astype(np.int64)
        uo += m * k
        jo += k
    for t in range(H.first_leaf()):
        ka, kb = int(ranks[2 * t + 1]), int(ranks[2 * t + 2])
        H.B[t] = exp["B"][bo:bo + ka * kb].reshape(ka, kb).copy()
        bo += ka * kb
    shift = exp["delta"] if with_shift else 0.0
    H.D = [exp["D"][i] + shift * np.eye(exp["D"][i].shape[0]) for i in range(len(exp["D"]))]
    assert [d.shape[0] for d in H.D] == list(np.diff(H.loff))
    assert uo == exp["U"].size and bo == exp["B"].size
    return H


def export_from_oracle_hss(H, perm, delta=0.0):
    """The oracle's generators in the layout hss_export writes / hss_import reads (D without the shift)."""
    nn = H.nnodes
    sizes = np.array([H.size(t) for t in range(nn)], dtype=np.int32)
    ranks = np.array([H.rank(t) for t in range(nn)], dtype=np.int32)
    U = [H.U[t].reshape(-1) for t in range(1, nn)]
    J = [np.asarray(H.J[t], dtype=np.int32) for t in range(1, nn)]
    B = [H.B[t].reshape(-1) for t in range(H.first_leaf())]
    cat = lambda xs, dt: np.concatenate(xs).astype(dt) if xs else np.zeros(0, dtype=dt)
    return {"n": H.n, "leaf": H.leaf, "perm": np.asarray(perm, dtype=np.int64), "sizes": sizes, "ranks": ranks,
            "D": np.stack(H.D) if len({d.shape for d in H.D}) == 1 else list(H.D), "U": cat(U, np.float64), "J": cat(J, np.int32), "B": cat(B, np.float64),
            "delta": float(delta)}
