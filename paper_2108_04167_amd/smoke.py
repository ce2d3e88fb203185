"""One small invocation of the whole hot path on cuda:0, checked against the CPU oracle."""
import numpy as np


def run():
    import torch
    from oracle import admm as oadmm
    from oracle import hss as ohss
    from oracle import ulv as oulv
    from . import binding, synth

    if not torch.cuda.is_available():
        raise RuntimeError("smoke() needs a GPU")
    w = synth.make_workload(1, n=1024, leaf=64, s=128)
    dev = torch.device("cuda:0")
    ctx = binding.Context()
    F, y = torch.tensor(w.F, device=dev), torch.tensor(w.y, device=dev)
    Om = w.omega()
    ctx.hss_compress(F, y, w.h, w.leaf, w.tol, torch.tensor(Om, device=dev))
    exp = ctx.hss_export()
    perm = exp["perm"]
    # the oracle's view of the exported compressed matrix
    H = ohss.HSS(w.n, w.leaf)
    uo = jo = bo = 0
    for t in range(1, H.nnodes):
        m, k = int(exp["sizes"][t]), int(exp["ranks"][t])
        H.U[t] = exp["U"][uo:uo + m * k].reshape(m, k)
        uo += m * k
    for t in range(H.first_leaf()):
        ka, kb = int(exp["ranks"][2 * t + 1]), int(exp["ranks"][2 * t + 2])
        H.B[t] = exp["B"][bo:bo + ka * kb].reshape(ka, kb)
        bo += ka * kb
    H.D = [exp["D"][i] + exp["delta"] * np.eye(w.leaf) for i in range(w.n // w.leaf)]
    ctx.hss_ulv_factor(w.beta)
    b = np.random.default_rng(0).standard_normal(w.n)
    x = torch.tensor(b, device=dev)
    ctx.hss_ulv_solve(x)
    Fz = oulv.ulv_factor(H, w.beta)
    ref = np.empty(w.n)
    ref[perm] = oulv.ulv_solve(Fz, b[perm])
    err = np.linalg.norm(x.cpu().numpy() - ref) / np.linalg.norm(ref)
    assert err <= 1e-10, f"ULV solve differs from the oracle: {err}"
    out = ctx.admm_svm_train(w.C, w.beta, 30)
    oref = oadmm.admm(lambda v: oulv.ulv_solve(Fz, v), w.y[perm], w.C, w.beta, 30)
    ez = np.linalg.norm(out["z"].cpu().numpy()[perm] - oref["z"]) / max(np.linalg.norm(oref["z"]), 1e-300)
    assert ez <= 1e-6, f"ADMM iterate differs from the oracle: {ez}"
    ctx.close()
    print(f"smoke ok: ulv rel err {err:.2e}, admm z rel err {ez:.2e}")
