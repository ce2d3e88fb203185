"""Thin ctypes binding of libhsssvm.so: argument marshalling only.  torch is used for device
memory and the current HIP stream; every step of the path runs inside the library."""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhsssvm.so")
_lib = None

HSS_OK, HSS_EINVAL, HSS_ESTATE, HSS_ENOMEM, HSS_EHIP, HSS_EUNSUPPORTED = 0, -1, -2, -3, -4, -5
HSS_WRANK, HSS_WPIVOT, HSS_WNOMARGIN, HSS_WSHIFT = 1, 2, 4, 8

c_dp = C.c_void_p     # device or host pointer passed as an address


class HssStats(C.Structure):
    _fields_ = [("n", C.c_int64), ("r", C.c_int64), ("leaf", C.c_int64), ("levels", C.c_int64),
                ("sample_width", C.c_int64), ("rank_cap", C.c_int64),
                ("rank_max", C.c_int64), ("rank_sum", C.c_int64), ("nodes_at_cap", C.c_int64),
                ("generator_bytes", C.c_int64), ("factor_bytes", C.c_int64), ("factor_bytes_compact", C.c_int64),
                ("sample_flops", C.c_double), ("delta", C.c_double), ("beta", C.c_double),
                ("t_tree", C.c_double), ("t_sample", C.c_double), ("t_levels", C.c_double),
                ("t_guard", C.c_double), ("t_factor", C.c_double), ("t_sample_kernel", C.c_double),
                ("warnings", C.c_int32), ("reserved", C.c_int32),
                ("sample_width_used", C.c_int64), ("nodes_redone", C.c_int64)]


# name -> (restype, argtypes): every symbol include/hss_svm.h declares
ABI = {
    "hss_strerror": (C.c_char_p, [C.c_int]),
    "hss_create": (C.c_int, [C.POINTER(C.c_void_p), C.c_void_p]),
    "hss_destroy": (None, [C.c_void_p]),
    "hss_set_i64": (C.c_int, [C.c_void_p, C.c_char_p, C.c_int64]),
    "hss_set_f64": (C.c_int, [C.c_void_p, C.c_char_p, C.c_double]),
    "hss_kernel_sample": (C.c_int, [C.c_void_p, c_dp, C.c_int64, C.c_int32, C.c_double, c_dp, C.c_int32, c_dp]),
    "hss_kernel_sample_noalloc": (C.c_int, [C.c_void_p, c_dp, C.c_int64, C.c_int32, C.c_double, c_dp, C.c_int32, c_dp]),
    "hss_compress": (C.c_int, [C.c_void_p, c_dp, c_dp, C.c_int64, C.c_int32, C.c_double, C.c_int32, C.c_double]),
    "hss_compress_with_samples": (C.c_int, [C.c_void_p, c_dp, c_dp, C.c_int64, C.c_int32, C.c_double, C.c_int32,
                                            C.c_double, c_dp, C.c_int32]),
    "hss_error_estimate": (C.c_int, [C.c_void_p, C.c_int32, C.c_uint64, C.POINTER(C.c_double)]),
    "hss_ulv_factor": (C.c_int, [C.c_void_p, C.c_double]),
    "hss_ulv_solve": (C.c_int, [C.c_void_p, c_dp, C.c_int32]),
    "hss_matvec": (C.c_int, [C.c_void_p, c_dp, c_dp]),
    "admm_svm_train": (C.c_int, [C.c_void_p, C.c_double, C.c_double, C.c_int32, c_dp, c_dp, c_dp,
                                 C.POINTER(C.c_double), C.POINTER(C.c_int64)]),
    "admm_svm_train_multi": (C.c_int, [C.c_void_p, C.POINTER(C.c_double), C.c_int32, C.c_double, C.c_int32, c_dp, c_dp,
                                       c_dp, C.POINTER(C.c_double), C.POINTER(C.c_int64)]),
    "svm_decision": (C.c_int, [C.c_void_p, c_dp, C.c_int64, c_dp, C.c_double, c_dp]),
    "hss_stream_copy": (C.c_int, [C.c_void_p, c_dp, c_dp, C.c_int64]),
    "hss_stats": (C.c_int, [C.c_void_p, C.POINTER(HssStats)]),
    "hss_export_sizes": (C.c_int, [C.c_void_p] + [C.POINTER(C.c_int64)] * 4),
    "hss_export": (C.c_int, [C.c_void_p, c_dp, c_dp, c_dp, c_dp, c_dp, c_dp, c_dp, C.POINTER(C.c_double)]),
    "hss_export_neighbours": (C.c_int, [C.c_void_p, C.POINTER(C.c_int32), c_dp, c_dp]),
    "hss_import": (C.c_int, [C.c_void_p, c_dp, c_dp, C.c_int64, C.c_int32, C.c_double, C.c_int32,
                             c_dp, c_dp, c_dp, c_dp, c_dp, c_dp, c_dp, C.c_double]),
}


class HssError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        msg = _lib.hss_strerror(code).decode() if _lib is not None else "?"
        super().__init__(f"{where}: {msg} ({code})")


def load():
    """dlopen the in-tree library and declare every ABI symbol.  Raises if the library has not
    been built: there is no fallback path."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: run `python __graft_entry__.py` (build()) first")
    lib = C.CDLL(LIB_PATH)
    for name, (res, args) in ABI.items():
        fn = getattr(lib, name)          # AttributeError if a declared symbol is not exported
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def _check(code, where):
    if code < 0:
        raise HssError(code, where)
    return code


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _dev_f64(t, name, numel=None):
    import torch
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float64 and t.is_contiguous()):
        raise TypeError(f"{name} must be a contiguous float64 CUDA tensor")
    if numel is not None and t.numel() != numel:
        raise ValueError(f"{name} must hold {numel} doubles, got {t.numel()}")
    return t


class Context:
    """Owns one hss_ctx.  Methods carry the names of the C calls."""

    def __init__(self, stream=None):
        import torch
        lib = load()
        if stream is None:
            stream = torch.cuda.current_stream().cuda_stream
        self._h = C.c_void_p()
        _check(lib.hss_create(C.byref(self._h), C.c_void_p(stream)), "hss_create")
        self.n = 0
        self.r = 0

    def close(self):
        if self._h:
            _lib.hss_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def hss_set_i64(self, key, v):
        return _check(_lib.hss_set_i64(self._h, key.encode(), int(v)), "hss_set_i64")

    def hss_set_f64(self, key, v):
        return _check(_lib.hss_set_f64(self._h, key.encode(), float(v)), "hss_set_f64")

    def hss_kernel_sample(self, F, h, Omega):
        import torch
        n, r = F.shape
        s = Omega.shape[1]
        _dev_f64(F, "F")
        _dev_f64(Omega, "Omega", n * s)
        S = torch.empty((n, s), dtype=torch.float64, device=F.device)
        _check(_lib.hss_kernel_sample(self._h, _ptr(F), n, r, float(h), _ptr(Omega), s, _ptr(S)), "hss_kernel_sample")
        return S

    def hss_kernel_sample_noalloc(self, F, h, Omega, S_out):
        """Allocation-free variant: the caller brings S_out (n x s); asynchronous on the context's stream."""
        n, r = F.shape
        s = Omega.shape[1]
        _dev_f64(F, "F")
        _dev_f64(Omega, "Omega", n * s)
        _dev_f64(S_out, "S_out", n * s)
        return _check(_lib.hss_kernel_sample_noalloc(self._h, _ptr(F), n, r, float(h), _ptr(Omega), s, _ptr(S_out)),
                      "hss_kernel_sample_noalloc")

    def hss_compress(self, F, y, h, leaf, tol, Omega=None):
        n, r = F.shape
        _dev_f64(F, "F")
        _dev_f64(y, "y", n)
        if Omega is None:
            rc = _lib.hss_compress(self._h, _ptr(F), _ptr(y), n, r, float(h), int(leaf), float(tol))
        else:
            _dev_f64(Omega, "Omega", n * Omega.shape[1])
            rc = _lib.hss_compress_with_samples(self._h, _ptr(F), _ptr(y), n, r, float(h), int(leaf), float(tol),
                                                _ptr(Omega), int(Omega.shape[1]))
        _check(rc, "hss_compress")
        self.n, self.r = n, r
        return rc

    def hss_ulv_factor(self, beta):
        return _check(_lib.hss_ulv_factor(self._h, float(beta)), "hss_ulv_factor")

    def hss_ulv_solve(self, rhs):
        """In place; rhs is (n,) or (nrhs, n) contiguous (each right-hand side contiguous)."""
        _dev_f64(rhs, "rhs")
        nrhs = 1 if rhs.dim() == 1 else rhs.shape[0]
        if rhs.numel() != nrhs * self.n:
            raise ValueError("rhs has the wrong size")
        return _check(_lib.hss_ulv_solve(self._h, _ptr(rhs), nrhs), "hss_ulv_solve")

    def hss_matvec(self, x):
        import torch
        _dev_f64(x, "x", self.n)
        y = torch.empty_like(x)
        _check(_lib.hss_matvec(self._h, _ptr(x), _ptr(y)), "hss_matvec")
        return y

    def admm_svm_train(self, Cbox, beta, maxit):
        import torch
        dev = torch.device("cuda", torch.cuda.current_device())
        x = torch.empty(self.n, dtype=torch.float64, device=dev)
        z = torch.empty_like(x)
        mu = torch.empty_like(x)
        b = C.c_double(0.0)
        cnt = C.c_int64(0)
        rc = _check(_lib.admm_svm_train(self._h, float(Cbox), float(beta), int(maxit), _ptr(x), _ptr(z), _ptr(mu),
                                        C.byref(b), C.byref(cnt)), "admm_svm_train")
        return {"x": x, "z": z, "mu": mu, "bias": b.value, "n_margin": cnt.value, "rc": rc}

    def svm_decision(self, G, z, bias):
        import torch
        _dev_f64(G, "G")
        _dev_f64(z, "z", self.n)
        if G.shape[1] != self.r:
            raise ValueError("G has the wrong feature count")
        dec = torch.empty(G.shape[0], dtype=torch.float64, device=G.device)
        _check(_lib.svm_decision(self._h, _ptr(G), G.shape[0], _ptr(z), float(bias), _ptr(dec)), "svm_decision")
        return dec

    def hss_stream_copy(self, src, dst):
        _dev_f64(src, "src")
        _dev_f64(dst, "dst", src.numel())
        return _check(_lib.hss_stream_copy(self._h, _ptr(src), _ptr(dst), src.numel()), "hss_stream_copy")

    def hss_stats(self):
        st = HssStats()
        _check(_lib.hss_stats(self._h, C.byref(st)), "hss_stats")
        return {k: getattr(st, k) for k, _ in HssStats._fields_}

    def hss_export(self):
        """Generators on the host as numpy arrays (see include/hss_svm.h for the layout)."""
        import numpy as np
        nn, ul, jl, bl = C.c_int64(), C.c_int64(), C.c_int64(), C.c_int64()
        _check(_lib.hss_export_sizes(self._h, C.byref(nn), C.byref(ul), C.byref(jl), C.byref(bl)), "hss_export_sizes")
        st = self.hss_stats()
        n, leaf = st["n"], st["leaf"]
        perm = np.empty(n, dtype=np.int64)
        sizes = np.empty(nn.value, dtype=np.int32)
        ranks = np.empty(nn.value, dtype=np.int32)
        D = np.empty(n * leaf, dtype=np.float64)
        U = np.empty(max(ul.value, 1), dtype=np.float64)
        J = np.empty(max(jl.value, 1), dtype=np.int32)
        B = np.empty(max(bl.value, 1), dtype=np.float64)
        delta = C.c_double(0.0)
        p = lambda a: C.c_void_p(a.ctypes.data)
        _check(_lib.hss_export(self._h, p(perm), p(sizes), p(ranks), p(D), p(U), p(J), p(B), C.byref(delta)),
               "hss_export")
        # leaf blocks: compact, one after the other; a (leaves, m, m) array when all leaves have one size, else a list
        msz = sizes[(nn.value + 1) // 2 - 1:].astype(np.int64)
        if (msz == msz[0]).all():
            Dl = D[:msz.size * int(msz[0]) ** 2].reshape(msz.size, int(msz[0]), int(msz[0]))
        else:
            off = np.concatenate([[0], np.cumsum(msz * msz)])
            Dl = [D[off[i]:off[i + 1]].reshape(int(msz[i]), int(msz[i])) for i in range(msz.size)]
        return {"n": n, "leaf": leaf, "perm": perm, "sizes": sizes, "ranks": ranks,
                "D": Dl, "U": U[:ul.value], "J": J[:jl.value], "B": B[:bl.value], "delta": delta.value}

    def hss_export_neighbours(self):
        """(idx, dist) of the last neighbour-based compression: (n, k) int32 / float64, cluster-tree order."""
        import numpy as np
        k = C.c_int32(0)
        _check(_lib.hss_export_neighbours(self._h, C.byref(k), None, None), "hss_export_neighbours")
        idx = np.empty((self.n, k.value), dtype=np.int32)
        dist = np.empty((self.n, k.value), dtype=np.float64)
        _check(_lib.hss_export_neighbours(self._h, C.byref(k), C.c_void_p(idx.ctypes.data), C.c_void_p(dist.ctypes.data)),
               "hss_export_neighbours")
        return idx, dist

    def hss_import(self, F, y, h, leaf, gen):
        """Compressed state from host generators `gen` (a dict laid out like hss_export's result)."""
        import numpy as np
        n, r = F.shape
        keep = [np.ascontiguousarray(gen["perm"], dtype=np.int64), np.ascontiguousarray(gen["sizes"], dtype=np.int32),
                np.ascontiguousarray(gen["ranks"], dtype=np.int32),
                (np.concatenate([np.asarray(d, dtype=np.float64).reshape(-1) for d in gen["D"]])
                 if isinstance(gen["D"], (list, tuple)) else np.ascontiguousarray(gen["D"], dtype=np.float64).reshape(-1)),
                np.ascontiguousarray(gen["U"], dtype=np.float64), np.ascontiguousarray(gen["J"], dtype=np.int32),
                np.ascontiguousarray(gen["B"], dtype=np.float64)]
        keep = [a if a.size else np.zeros(1, dtype=a.dtype) for a in keep]
        p = lambda a: C.c_void_p(a.ctypes.data)
        rc = _check(_lib.hss_import(self._h, _ptr(F), _ptr(y), n, r, float(h), int(leaf), *[p(a) for a in keep],
                                    float(gen.get("delta", 0.0))), "hss_import")
        self.n, self.r = n, r
        return rc

    def admm_svm_train_multi(self, C_list, beta, maxit):
        """One ADMM run per box bound in C_list (same beta); x, z, mu come back as (len(C_list), n)."""
        import torch
        nC = len(C_list)
        cl = (C.c_double * nC)(*[float(v) for v in C_list])
        dev = torch.device("cuda", torch.cuda.current_device())
        x = torch.empty((nC, self.n), dtype=torch.float64, device=dev)
        z = torch.empty_like(x)
        mu = torch.empty_like(x)
        bias = (C.c_double * nC)()
        cnt = (C.c_int64 * nC)()
        rc = _check(_lib.admm_svm_train_multi(self._h, cl, nC, float(beta), int(maxit), _ptr(x), _ptr(z), _ptr(mu),
                                              bias, cnt), "admm_svm_train_multi")
        return {"x": x, "z": z, "mu": mu, "bias": list(bias), "n_margin": list(cnt), "warnings": rc}

    def hss_error_estimate(self, nprobe=16, seed=1):
        out = C.c_double(0.0)
        _check(_lib.hss_error_estimate(self._h, int(nprobe), int(seed), C.byref(out)), "hss_error_estimate")
        return out.value
