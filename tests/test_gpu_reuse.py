"""One context used for a sequence of different problems (GPU only): sizes up and down, few and many features,
random and neighbour-based sampling, both trees, a factorization and an ADMM run in between.  Every step must give
bit for bit what a fresh context gives for the same problem: nothing of an earlier, larger problem may leak into a
later one (the context's buffers only grow)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from paper_2108_04167_amd import binding   # noqa: E402


def _dev(a):
    import torch
    return torch.tensor(np.ascontiguousarray(a), device="cuda:0")


def _problem(n, r, seed):
    g = np.random.default_rng(seed)
    F = g.standard_normal((n, r)) * (0.3 if r > 20 else 1.0)
    F[:, 0] += 0.5 * g.standard_normal(n)
    y = np.where(g.random(n) < 0.5, 1.0, -1.0)
    G = g.standard_normal((37, r))
    return F, y, G


def _run(ctx, F, y, G, h, leaf, s, opts, beta, C, its):
    """Set every option the sequence touches (so that a reused context carries none over), then the whole path."""
    full = dict(sampling=0, clustering=0, adaptive_start=0, max_rank=0, ann_neighbours=64, ann_trees=3, seed=0)
    full.update(opts)
    ctx.hss_set_i64("sample_width", s)
    for k, v in full.items():
        ctx.hss_set_i64(k, v)
    rc = ctx.hss_compress(_dev(F), _dev(y), h, leaf, 1e-3)
    exp = ctx.hss_export()
    out = ctx.admm_svm_train(C, beta, its)
    dec = ctx.svm_decision(_dev(G), out["z"], out["bias"]).cpu().numpy()
    est = ctx.hss_error_estimate(4, 9)
    st = ctx.hss_stats()
    return dict(rc=rc, perm=exp["perm"], sizes=exp["sizes"], ranks=exp["ranks"], U=exp["U"], B=exp["B"], J=exp["J"],
                D=np.concatenate([np.asarray(d).reshape(-1) for d in exp["D"]]), delta=exp["delta"],
                x=out["x"].cpu().numpy(), z=out["z"].cpu().numpy(), mu=out["mu"].cpu().numpy(), bias=out["bias"],
                dec=dec, est=est, cap=st["rank_cap"], width=st["sample_width_used"])


SEQUENCE = [
    # n, r, h, leaf, s, options, beta, C, iterations
    (1000, 8, 1.5, 64, 128, {}, 1.0, 1.0, 12),
    (3001, 54, 3.0, 256, 512, {}, 0.5, 10.0, 8),
    (500, 3, 0.8, 32, 128, {"sampling": 1, "ann_neighbours": 16}, 1.0, 1.0, 10),
    (2048, 123, 2.0, 64, 128, {"clustering": 1}, 2.0, 1.0, 6),
    (777, 22, 2.0, 128, 256, {"adaptive_start": 128}, 1.0, 0.1, 9),
    (64, 5, 1.0, 64, 128, {}, 1.0, 1.0, 5),                              # a single leaf
    (4099, 18, 1.0, 256, 512, {"sampling": 1, "clustering": 1}, 1.0, 10.0, 6),
    (1000, 8, 1.5, 64, 128, {}, 1.0, 1.0, 12),                           # the first problem again
]


def test_one_context_for_many_problems():
    shared = binding.Context()
    first = None
    for step, (n, r, h, leaf, s, opts, beta, C, its) in enumerate(SEQUENCE):
        F, y, G = _problem(n, r, 100 + step if step != len(SEQUENCE) - 1 else 100)
        got = _run(shared, F, y, G, h, leaf, s, opts, beta, C, its)
        fresh = binding.Context()
        ref = _run(fresh, F, y, G, h, leaf, s, opts, beta, C, its)
        fresh.close()
        for key in ref:
            a, b = got[key], ref[key]
            same = np.array_equal(a, b) if isinstance(b, np.ndarray) else a == b
            assert same, (step, key)
        if step == 0:
            first = got
    for key in first:                      # and the last step repeated the first problem
        a, b = got[key], first[key]
        assert np.array_equal(a, b) if isinstance(b, np.ndarray) else a == b, key
    shared.close()


def test_out_of_memory_is_an_error_and_the_context_stays_usable():
    """A compression whose sample buffers cannot be allocated (2^25 points x 2048 columns = 550 GB per buffer) returns
    HSS_ENOMEM -- no abort, nothing left half-built -- and the same context then compresses a small problem to the
    bits of a fresh context."""
    import torch
    n = 1 << 25
    g = torch.Generator(device="cuda:0")
    g.manual_seed(1)
    F = torch.randn((n, 1), dtype=torch.float64, device="cuda:0", generator=g)
    y = torch.ones(n, dtype=torch.float64, device="cuda:0")
    ctx = binding.Context()
    ctx.hss_set_i64("sample_width", 2048)
    ctx.hss_set_i64("max_rank", 512)
    with pytest.raises(binding.HssError) as e:
        ctx.hss_compress(F, y, 1.0, 256, 1e-2)
    assert e.value.code == binding.HSS_ENOMEM
    del F, y
    torch.cuda.empty_cache()
    with pytest.raises(binding.HssError) as e:                # nothing compressed
        ctx.hss_ulv_factor(1.0)
    assert e.value.code == binding.HSS_ESTATE
    Fs, ys, G = _problem(1000, 8, 5)
    got = _run(ctx, Fs, ys, G, 1.5, 64, 128, {}, 1.0, 1.0, 8)
    fresh = binding.Context()
    ref = _run(fresh, Fs, ys, G, 1.5, 64, 128, {}, 1.0, 1.0, 8)
    for key in ref:
        a, b = got[key], ref[key]
        assert np.array_equal(a, b) if isinstance(b, np.ndarray) else a == b, key
    fresh.close()
    ctx.close()


def test_destroy_returns_the_device_memory():
    """Create, use and destroy 40 contexts: the free device memory afterwards is what it was before (within the
    allocator's granularity), so nothing the library allocates outlives hss_destroy."""
    import torch
    Fs, ys, G = _problem(3001, 20, 3)
    warm = binding.Context()
    _run(warm, Fs, ys, G, 2.0, 128, 256, {"sampling": 1}, 1.0, 1.0, 3)      # first use: code objects, arena, streams
    warm.close()
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    before, _ = torch.cuda.mem_get_info()
    for i in range(40):
        ctx = binding.Context()
        _run(ctx, Fs, ys, G, 2.0, 128, 256, {"sampling": i % 2, "clustering": (i // 2) % 2}, 1.0, 1.0, 3)
        ctx.close()
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    after, _ = torch.cuda.mem_get_info()
    assert before - after < 64 << 20, (before, after)


def test_repeated_trains_on_one_context_settle_and_leave_nothing():
    """The context keeps released device blocks for later allocations of the same size: after the second of several
    identical trains on one context the device's free memory no longer moves (nothing is allocated or freed on the
    way), every train gives the bits of the first, a change of shape does not let the footprint grow beyond what
    the two latest shapes need, and a closed context has returned everything."""
    import torch
    Fs, ys, G = _problem(4099, 20, 11)
    F2, y2, G2 = _problem(1500, 7, 12)
    warm = binding.Context()
    _run(warm, Fs, ys, G, 2.0, 128, 256, {}, 1.0, 1.0, 3)
    warm.close()
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    base, _ = torch.cuda.mem_get_info()
    ctx = binding.Context()
    first = _run(ctx, Fs, ys, G, 2.0, 128, 256, {}, 1.0, 1.0, 3)
    free = []
    for _ in range(4):
        got = _run(ctx, Fs, ys, G, 2.0, 128, 256, {}, 1.0, 1.0, 3)
        for key in first:
            a, b = got[key], first[key]
            assert np.array_equal(a, b) if isinstance(b, np.ndarray) else a == b, key
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
        free.append(torch.cuda.mem_get_info()[0])
    assert max(free[1:]) - min(free[1:]) <= 4 << 20, free      # (the runtime's own small pools may still move)
    held_same_shape = base - free[3]
    # another shape, three times: the blocks of the first shape age out, the footprint follows the new shape
    for _ in range(3):
        _run(ctx, F2, y2, G2, 1.0, 64, 128, {}, 1.0, 1.0, 3)
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    assert base - torch.cuda.mem_get_info()[0] <= held_same_shape + (64 << 20)
    ctx.close()
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    assert base - torch.cuda.mem_get_info()[0] < 64 << 20


def test_failed_allocation_empties_the_caches_of_other_contexts():
    """What one context keeps for reuse must never be the reason another one runs out of memory: an allocation that
    fails in context b empties the block cache of the idle context a as well (its blocks go back to the device), and
    a then still gives the bits it gave before."""
    import torch
    Fs, ys, G = _problem(4099, 20, 31)
    a = binding.Context()
    first = _run(a, Fs, ys, G, 2.0, 128, 256, {}, 1.0, 1.0, 3)
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    free1, _ = torch.cuda.mem_get_info()
    n = 1 << 25
    F = torch.zeros((n, 1), dtype=torch.float64, device="cuda:0")
    F[::2] = 1.0
    y = torch.ones(n, dtype=torch.float64, device="cuda:0")
    b = binding.Context()
    b.hss_set_i64("sample_width", 2048)
    b.hss_set_i64("max_rank", 512)
    with pytest.raises(binding.HssError) as e:
        b.hss_compress(F, y, 1.0, 256, 1e-2)
    code = e.value.code
    del e                                    # (its traceback holds the call's arguments)
    assert code == binding.HSS_ENOMEM
    b.close()
    del F, y
    import gc
    gc.collect()
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    free2, _ = torch.cuda.mem_get_info()
    assert free2 >= free1 + (16 << 20), (free1, free2)          # a's cached work space went back
    again = _run(a, Fs, ys, G, 2.0, 128, 256, {}, 1.0, 1.0, 3)
    for key in first:
        x, z = again[key], first[key]
        assert np.array_equal(x, z) if isinstance(z, np.ndarray) else x == z, key
    a.close()


def test_block_cache_option_changes_no_result():
    """Option block_cache_mib: 0 keeps nothing (the device's free memory after a train is then what a fresh context
    leaves), any value gives the same bits; values out of range are refused."""
    import torch
    Fs, ys, G = _problem(3001, 20, 41)
    ref_ctx = binding.Context()
    ref = _run(ref_ctx, Fs, ys, G, 2.0, 128, 256, {}, 1.0, 1.0, 3)
    ref = _run(ref_ctx, Fs, ys, G, 2.0, 128, 256, {}, 1.0, 1.0, 3)       # second pass: served from the cache
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    free_cached, _ = torch.cuda.mem_get_info()
    ref_ctx.hss_set_i64("block_cache_mib", 0)                           # frees what is kept
    torch.cuda.synchronize()
    free_after_off, _ = torch.cuda.mem_get_info()
    assert free_after_off >= free_cached
    for mib in (0, 1, 64):
        ctx = binding.Context()
        ctx.hss_set_i64("block_cache_mib", mib)
        for _ in range(2):
            got = _run(ctx, Fs, ys, G, 2.0, 128, 256, {}, 1.0, 1.0, 3)
            for key in ref:
                a, b = got[key], ref[key]
                assert np.array_equal(a, b) if isinstance(b, np.ndarray) else a == b, (mib, key)
        ctx.close()
    for bad in (-1, 1 << 25):
        with pytest.raises(binding.HssError) as e:
            ref_ctx.hss_set_i64("block_cache_mib", bad)
        assert e.value.code == binding.HSS_EINVAL
    ref_ctx.close()


def test_two_contexts_on_two_threads():
    """Different contexts may be used by different threads at the same time (one context by one thread at a time):
    two threads, each with a context of its own, train different problems three times over while the other one runs
    (the library calls release the interpreter lock); every result is the bits of the same train run alone."""
    import threading
    probs = [(_problem(3001, 20, 51), 2.0, 128, 256, {}), (_problem(2048, 8, 52), 1.5, 64, 128, {"sampling": 1})]
    refs = []
    for (Fs, ys, G), h, leaf, s, opts in probs:
        c = binding.Context()
        refs.append(_run(c, Fs, ys, G, h, leaf, s, opts, 1.0, 1.0, 4))
        c.close()
    errors = []

    def work(i):
        try:
            (Fs, ys, G), h, leaf, s, opts = probs[i]
            c = binding.Context()
            for _ in range(3):
                got = _run(c, Fs, ys, G, h, leaf, s, opts, 1.0, 1.0, 4)
                for key in refs[i]:
                    a, b = got[key], refs[i][key]
                    if not (np.array_equal(a, b) if isinstance(b, np.ndarray) else a == b):
                        errors.append((i, key))
            c.close()
        except Exception as e:          # noqa: BLE001
            errors.append((i, repr(e)))

    threads = [threading.Thread(target=work, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=120)
    assert not any(t.is_alive() for t in threads)
    assert not errors, errors
