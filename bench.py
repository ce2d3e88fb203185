"""Benchmark of the shifted-kernel-solve hot path on one MI355X.

A step is one pass of the whole path on one batch of synthetic input already resident in HBM:
HSS compression (cluster tree, K*Omega sampling, interpolative decompositions, definiteness guard),
ULV factorization of K~ + beta I, and the ADMM run (maxit iterations, one ULV solve each) with the
bias.  Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
FP64_MFMA_PEAK_TFLOPS = 78.6
# (workload, n) -> HBM bytes per launch (sample_kernel) / per solve (all launches of one ULV solve), read + written,
# from the FETCH_SIZE / WRITE_SIZE counter runs summarised in profiles/sample_kernel_cfg3_counters.txt and
# profiles/solve_gemv_kernel_cfg3_counters.txt, each with the SHA-256 (first 16 hex digits) of the kernel source the
# counters were taken on: a figure is reported only while that source is unchanged, null otherwise.
MEASURED_TRAFFIC_BYTES = {(3, 262144): {"sample_kernel": (7.950e11, "sample.hip", "d441294bdb34d313"),
                                        "solve": (4.393e9, "solve.hip", "9b26fe6d70520f64")}}


def measured_traffic(cfg, n, which):
    import hashlib
    ent = MEASURED_TRAFFIC_BYTES.get((cfg, n), {}).get(which)
    if ent is None:
        return None, "no counter run for this workload"
    nbytes, src, sha = ent
    path = os.path.join(ROOT, "paper_2108_04167_amd", "csrc", src)
    cur = hashlib.sha256(open(path, "rb").read()).hexdigest()[:16]
    if cur != sha:
        return None, f"{src} changed since the counters were taken (profiles/): retake them"
    return nbytes, f"rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on {src} {sha}, see profiles/"


def cpu_baseline(cfg, n_small, maxit):
    """The oracle, as it stands, on a bounded cut of the same workload (host cores of this machine)."""
    import numpy as np
    from oracle import admm as oadmm
    from oracle import hss as ohss
    from oracle import ulv as oulv
    from oracle.tree import cluster_tree
    from paper_2108_04167_amd import synth
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    w = synth.make_workload(cfg, n=n_small)
    t0 = time.time()
    perm = cluster_tree(w.F, w.leaf)
    Fp, yp = w.F[perm], w.y[perm]
    Om = w.omega()[perm]
    t1 = time.time()
    S = ohss.sample(Fp, Om, w.h)
    t2 = time.time()
    H = ohss.compress(Fp, w.h, w.leaf, Om, w.tol / 10.0, 1e-8, w.s // 2, S=S)
    ohss.add_diagonal(H, ohss.psd_shift(H))
    Fz = oulv.ulv_factor(H, w.beta)
    out = oadmm.admm(lambda v: oulv.ulv_solve(Fz, v), yp, w.C, w.beta, maxit)
    oadmm.bias(out["z"], yp, w.C, lambda v: ohss.matvec(H, v))
    t3 = time.time()
    return {"n": n_small, "t_sampling": t2 - t1, "t_rest": (t1 - t0) + (t3 - t2), "threads": threads}


def sweep(args, w, ctx, F, y):
    """The hyper-parameter grid of a workload (Sec. 3.2: compress once per h, factor once per beta, one ADMM run
    per (C, beta)): lockstep C runs against the same grid as separate runs."""
    import torch
    Cs = list(w.C_grid) if w.C_grid else [w.C]
    betas = list(w.beta_grid) if w.beta_grid else [w.beta]

    def timed(f):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        out = f()
        torch.cuda.synchronize()
        return time.perf_counter() - t0, out

    t_compress, _ = timed(lambda: ctx.hss_compress(F, y, w.h, w.leaf, w.tol))
    rows = []
    t_factor = t_lock = t_sep = 0.0
    t_factor_each = []
    for beta in betas:
        tf, _ = timed(lambda: ctx.hss_ulv_factor(beta))
        t_factor_each.append(tf)
        tl, multi = timed(lambda: ctx.admm_svm_train_multi(Cs, beta, w.maxit))
        ts = 0.0
        for j, Cj in enumerate(Cs):
            t1, single = timed(lambda: ctx.admm_svm_train(Cj, beta, w.maxit))
            ts += t1
            dz = float((multi["z"][j] - single["z"]).abs().max().item())
            rows.append({"C": Cj, "beta": beta, "bias": multi["bias"][j], "n_margin": multi["n_margin"][j],
                         "max_abs_diff_z_vs_separate_run": dz})
        t_factor += tf
        t_lock += tl
        t_sep += ts
    st = ctx.hss_stats()
    npairs = len(Cs) * len(betas)
    rec = {"metric": "admm_hss_sweep_seconds", "value": t_compress + t_factor + t_lock, "unit": "s", "n_gpus": 1,
           "higher_is_better": False, "dtype": "f64", "data": "synthetic",
           "config": {"workload": f"cfg{args.cfg}" + (f" cut to n={w.n}" if args.n else ""), "n": w.n, "r": w.r,
                      "h": w.h, "leaf": w.leaf, "sample_width": w.s, "C_grid": Cs, "beta_grid": betas,
                      "admm_iterations": w.maxit},
           "factor_s_per_beta": t_factor_each,     # the first builds the beta-independent parts, the others reuse them
           "phases_s": {"compress": t_compress, "factor_all_betas": t_factor, "admm_lockstep_all_pairs": t_lock,
                        "admm_separate_runs_all_pairs": t_sep},
           "seconds_per_pair_lockstep": t_lock / npairs, "seconds_per_pair_separate": t_sep / npairs,
           "solve_bytes": st["factor_bytes"], "pairs": rows}
    print(json.dumps(rec))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--cfg", type=int, default=3, help="workload 1..5 (default 3: n=262144, the metric's config)")
    ap.add_argument("--n", type=int, default=0, help="cut the workload to n points (profiling runs only; 0 = full size)")
    ap.add_argument("--copy-probe", type=int, default=0,
                    help="also run one plain device-to-device copy of this many bytes (reference for HBM counters)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-neighbour-leg", action="store_true", help="skip the extra pass with neighbour-based sampling")
    ap.add_argument("--sample-width", type=int, default=0, help="override the workload's sample width s (largest width "
                    "with --adaptive-start)")
    ap.add_argument("--adaptive-start", type=int, default=0, help="adaptive sample width: first width (0 = off)")
    ap.add_argument("--adaptive-step", type=int, default=128)
    ap.add_argument("--oversample", type=int, default=-1, help="oversampling p (rank cap = width - p; default width/2)")
    ap.add_argument("--max-rank", type=int, default=0)
    ap.add_argument("--tol", type=float, default=0.0, help="override the workload's tolerance (relative truncation "
                    "threshold = tol / 10)")
    ap.add_argument("--abs-tol", type=float, default=-1.0, help="absolute truncation threshold (default 1e-8)")
    ap.add_argument("--leaf", type=int, default=0, help="override the workload's largest leaf size")
    ap.add_argument("--paper-table1", action="store_true",
                    help="the parameter set under the paper's first results table: relative threshold 1, absolute 0.1, "
                         "rank cap 200, 64 approximate neighbours (neighbour-based sampling), leaf 128")
    ap.add_argument("--neighbours", action="store_true",
                    help="neighbour-based sampling (the paper's own compressor) instead of the random sample K*Omega")
    ap.add_argument("--ann-trees", type=int, default=3)
    ap.add_argument("--clustering", type=int, default=0, help="cluster tree rule: 0 coordinate bisection, 1 two-means")
    ap.add_argument("--graph", action="store_true", help="replay the ADMM iterations from a HIP graph (A/B; default eager)")
    ap.add_argument("--no-merge-top", action="store_true", help="one launch per tree level in the solve (A/B)")
    ap.add_argument("--sweep", action="store_true",
                    help="time the workload's C x beta grid instead (one compression, one factorization per beta, "
                         "the C values of a beta in lockstep); prints its own JSON line")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on ONE GPU; --gpus must be 1 (no collectives, no sharding).", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2108_04167_amd import binding, synth
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    binding.load()
    dev = torch.device("cuda:0")
    w = synth.make_workload(args.cfg, n=args.n or None)
    if args.copy_probe > 0:
        src = torch.ones(args.copy_probe // 8, dtype=torch.float64, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    F = torch.tensor(w.F, device=dev)
    y = torch.tensor(w.y, device=dev)
    ctx = binding.Context()
    if args.paper_table1:
        args.neighbours, args.tol, args.abs_tol, args.max_rank, args.leaf = True, 10.0, 0.1, 200, 128
        args.sample_width = args.sample_width or 256
    if args.tol > 0.0:
        w.tol = args.tol
    if args.leaf:
        w.leaf = args.leaf
    if args.abs_tol >= 0.0:
        ctx.hss_set_f64("abs_tol", args.abs_tol)
    if args.sample_width:
        w.s = args.sample_width
    ctx.hss_set_i64("sample_width", w.s)
    if args.adaptive_start:
        ctx.hss_set_i64("adaptive_start", args.adaptive_start)
        ctx.hss_set_i64("adaptive_step", args.adaptive_step)
    if args.oversample >= 0:
        ctx.hss_set_i64("oversample", args.oversample)
    if args.max_rank:
        ctx.hss_set_i64("max_rank", args.max_rank)
    if args.neighbours:
        ctx.hss_set_i64("sampling", 1)
        ctx.hss_set_i64("ann_trees", args.ann_trees)
    if args.clustering:
        ctx.hss_set_i64("clustering", args.clustering)
    if args.graph:
        ctx.hss_set_i64("graph", 1)
    if args.no_merge_top:
        ctx.hss_set_i64("merge_top", 0)
    if args.sweep:
        sweep(args, w, ctx, F, y)
        return

    def step():
        ctx.hss_compress(F, y, w.h, w.leaf, w.tol)                 # draws Omega in-library
        st = ctx.hss_stats()
        t0 = time.perf_counter()
        out = ctx.admm_svm_train(w.C, w.beta, w.maxit)              # factors, iterates, computes the bias
        torch.cuda.synchronize()
        t_train = time.perf_counter() - t0
        st2 = ctx.hss_stats()
        return st, st2, t_train, out

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    t_kernel = 0.0
    t_solve_iter = 0.0
    last = None
    for _ in range(args.steps):
        st, st2, t_train, out = step()
        t_kernel += st["t_sample_kernel"]
        t_solve_iter += max(t_train - st2["t_factor"], 0.0) / max(w.maxit, 1)
        last = (st, st2, t_train, out)
    torch.cuda.synchronize()
    total = time.perf_counter() - t_begin
    per_step = total / args.steps
    st, st2, t_train, out = last
    t_kernel /= args.steps
    t_solve_iter /= args.steps
    n, r, s = w.n, w.r, w.s
    flops = st["sample_flops"]        # 2 n^2 (columns + r) summed over the sampling launches of one compression
    tf = flops / t_kernel / 1e12 if t_kernel > 0 else 0.0
    solve_gbs = st2["factor_bytes"] / t_solve_iter / 1e9

    # one ULV solve alone: median of 64 back-to-back calls through the C ABI (permutation in and out included),
    # timed with events on the stream the library launches on
    xb = torch.randn(n, dtype=torch.float64, device=dev)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(64)]
    ctx.hss_ulv_solve(xb)
    for e0, e1 in evs:
        e0.record()
        ctx.hss_ulv_solve(xb)
        e1.record()
    torch.cuda.synchronize()
    t_solve_median = sorted(e0.elapsed_time(e1) for e0, e1 in evs)[len(evs) // 2] * 1e-3

    # accuracy of the trained model (exact kernel), reported for context
    dec = ctx.svm_decision(torch.tensor(w.F_test, device=dev), out["z"], out["bias"])
    acc = float((((dec >= 0).double() * 2 - 1) == torch.tensor(w.y_test, device=dev)).double().mean().item() * 100)

    # HBM bytes per launch from the FETCH_SIZE / WRITE_SIZE counter runs summarised under profiles/ (scaled by
    # a plain copy of known size); they hold for the default workload and the kernels they were taken on only.
    default_path = not (args.neighbours or args.sample_width or args.adaptive_start or args.no_merge_top or args.tol > 0.0
                        or args.leaf or args.abs_tol >= 0.0)
    tr_sample, note_sample = measured_traffic(args.cfg, n, "sample_kernel") if default_path else (None, "non-default options")
    tr_solve, note_solve = measured_traffic(args.cfg, n, "solve") if default_path else (None, "non-default options")

    rel_err = ctx.hss_error_estimate(8, 1)     # achieved ||K~ - K||_F / ||K||_F on 8 probe vectors (not timed)

    rec = {
        "metric": "admm_hss_train_seconds", "value": per_step, "unit": "s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": per_step * 1e3,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": f"cfg{args.cfg}" + (f" cut to n={n}" if args.n else ""), "n": n, "r": r, "h": w.h, "C": w.C, "leaf": w.leaf, "tol": w.tol,
                   "sampling": "neighbours" if args.neighbours else "random", "clustering": args.clustering,
                   "sample_width": s, "sample_width_used": st["sample_width_used"], "rank_cap": st["rank_cap"],
                   "beta": w.beta, "admm_iterations": w.maxit},
        "phases_s": {"tree": st["t_tree"], "sampling": st["t_sample"], "levels": st["t_levels"], "guard": st["t_guard"],
                     "factor": st2["t_factor"], "admm_and_bias": t_train - st2["t_factor"]},
        "roofline": {"kernel": "sample_kernel (S = K*Omega, fused Gram+exp+contraction)", "bound": "mfma",
                     "achieved": tf, "peak": FP64_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": tf / FP64_MFMA_PEAK_TFLOPS,
                     "traffic": tr_sample, "traffic_source": note_sample, "flops_per_launch": flops,
                     "seconds_per_launch": t_kernel},
        "roofline_solve": {"kernel": "solve_gemv_kernel (ULV up/down sweeps, per ADMM iteration incl. vector update)",
                           "bound": "hbm", "achieved": solve_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                           "frac": solve_gbs / HBM_PEAK_GBS, "traffic": tr_solve, "traffic_source": note_solve,
                           "bytes_per_solve": st2["factor_bytes"], "bytes_per_solve_compact": st2["factor_bytes_compact"],
                           "seconds_per_iteration": t_solve_iter, "seconds_per_solve_median_of_64": t_solve_median},
        "model": {"delta": st["delta"], "rank_max": st["rank_max"], "nodes_at_cap": st["nodes_at_cap"],
                  "rel_error_estimate": rel_err, "tolerance_met": bool(rel_err <= w.tol and st["nodes_at_cap"] == 0),
                  "bias": out["bias"], "n_margin": out["n_margin"], "test_accuracy_pct": acc, "warnings": st2["warnings"]},
    }
    if not args.neighbours and not args.no_neighbour_leg:
        # the same train with the paper's own neighbour-based sample in place of K*Omega (one pass, not the metric);
        # the first context is done: its device memory goes back before the second one is built
        ctx.close()
        ctx2 = binding.Context()
        ctx2.hss_set_i64("sample_width", w.s)
        ctx2.hss_set_i64("sampling", 1)
        for _ in range(2):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ctx2.hss_compress(F, y, w.h, w.leaf, w.tol)
            o2 = ctx2.admm_svm_train(w.C, w.beta, w.maxit)
            torch.cuda.synchronize()
            t_ann = time.perf_counter() - t0
        s2 = ctx2.hss_stats()
        dec2 = ctx2.svm_decision(torch.tensor(w.F_test, device=dev), o2["z"], o2["bias"])
        acc2 = float((((dec2 >= 0).double() * 2 - 1) == torch.tensor(w.y_test, device=dev)).double().mean().item() * 100)
        rec["neighbour_sampling"] = {"train_seconds": t_ann, "rel_error_estimate": ctx2.hss_error_estimate(8, 1),
                                     "delta": s2["delta"], "test_accuracy_pct": acc2,
                                     "note": "option sampling=1 (Sec. 3.1 of the paper: columns of approximate nearest "
                                             "neighbours instead of the random sample); same width and rank cap"}
        ctx2.close()
    if not args.no_cpu_baseline:
        n_small = min(n, 4096 if args.cfg != 1 else 2048)
        cb = cpu_baseline(args.cfg, n_small, w.maxit)
        scale = n / cb["n"]
        est = cb["t_sampling"] * scale * scale + cb["t_rest"] * scale
        rec["cpu_baseline"] = {
            "value": est, "unit": "s", "cores": cb["threads"], "kind": "oracle",
            "sample": (f"whole oracle train (tree, K*Omega, HSS, guard, ULV, {w.maxit} ADMM iterations, bias) on the "
                       f"cfg{args.cfg} generator cut to n={cb['n']}: sampling {cb['t_sampling']:.2f} s, rest "
                       f"{cb['t_rest']:.2f} s; value extrapolates sampling by (n/n_cut)^2 and the rest by n/n_cut"),
        }
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
