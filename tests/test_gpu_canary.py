"""Race canary (GPU only): the same work split differently over the grid must give the same bits.  A kernel whose
result depended on which workgroup or wavefront got to a value first (a missing barrier, an unordered accumulation)
would differ between two decompositions sooner or later.
  * S = K Omega: one 512-column launch (64 x 512 blocks of S per workgroup) against 256- and 128-column windows
    (128 x 256 and 128 x 128 blocks);
  * row interpolative decomposition, both forms: 32 rows per workgroup (the library's split) against 8 and 64;
  * ULV solve: one right-hand side (two rows per wavefront) against the same column inside two and four lockstep
    columns (other row split, other work list);
  * compression as a whole run twice: identical generators."""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from paper_2108_04167_amd import binding, synth   # noqa: E402


def _dev(a):
    import torch
    return torch.tensor(np.ascontiguousarray(a), device="cuda:0")


@pytest.mark.parametrize("n,r,h", [(4096, 54, 3.0), (2048, 8, 1.5), (1000, 90, 4.0)])
def test_sampling_is_the_same_in_every_launch_shape(n, r, h):
    import torch
    rng = np.random.default_rng(n + r)
    F = _dev(rng.standard_normal((n, r)))
    Om = rng.standard_normal((n, 512))
    ctx = binding.Context()
    whole = ctx.hss_kernel_sample(F, h, _dev(Om))
    for width in (256, 128):
        for c0 in range(0, 512, width):
            part = ctx.hss_kernel_sample(F, h, _dev(Om[:, c0:c0 + width]))
            assert torch.equal(part, whole[:, c0:c0 + width].contiguous()), (width, c0)
    ctx.close()


@pytest.mark.parametrize("gram", [0, 1])
def test_row_id_is_the_same_for_every_row_split(gram):
    import torch
    from gpu_helpers import dev, hptr, lib, ptr
    L = lib()
    rng = np.random.default_rng(8)
    sizes = [64, 100, 33, 256, 16, 200, 512]
    rows = sum(sizes)
    A = np.zeros((rows, 256))
    moff = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    for t, m in enumerate(sizes):
        k = min(m, 256)
        Qa, _ = np.linalg.qr(rng.standard_normal((m, k)))
        Qb, _ = np.linalg.qr(rng.standard_normal((256, k)))
        A[moff[t]:moff[t + 1]] = (Qa * 0.9 ** np.arange(k)) @ Qb.T
    Ad = dev(A)
    L.hsx_row_id_blocks.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_double,
                                    C.c_double, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
    kcap, outs = 200, []
    for rpb in (32, 8, 64):
        ranks = np.zeros(len(sizes), dtype=np.int32)
        J = np.zeros((len(sizes), kcap), dtype=np.int32)
        U = torch.zeros(rows * kcap, dtype=torch.float64, device="cuda:0")
        assert L.hsx_row_id_blocks(None, ptr(Ad), 256, len(sizes), hptr(moff), kcap, 1e-4, 0.0, gram, rpb, hptr(ranks),
                                   hptr(J), ptr(U)) == 0
        outs.append((ranks.copy(), J.copy(), U.cpu().numpy()))
    for o in outs[1:]:
        assert np.array_equal(o[0], outs[0][0]) and np.array_equal(o[1], outs[0][1]) and np.array_equal(o[2], outs[0][2])


def test_solve_columns_do_not_depend_on_their_company():
    import torch
    w = synth.make_workload(3, n=16384)
    ctx = binding.Context()
    ctx.hss_set_i64("sample_width", w.s)
    ctx.hss_compress(_dev(w.F), _dev(w.y), w.h, w.leaf, w.tol)
    ctx.hss_ulv_factor(1.0)
    B = torch.randn((4, w.n), dtype=torch.float64, device="cuda:0")
    four = B.clone()
    ctx.hss_ulv_solve(four)
    two = B[:2].clone()
    ctx.hss_ulv_solve(two)
    for j in range(4):
        one = B[j].clone()
        ctx.hss_ulv_solve(one)
        assert torch.equal(one, four[j])
        if j < 2:
            assert torch.equal(one, two[j])
    ctx.close()


def test_compression_twice_gives_identical_generators():
    w = synth.make_workload(2, n=8192)
    exps = []
    for _ in range(2):
        ctx = binding.Context()
        ctx.hss_set_i64("sample_width", w.s)
        ctx.hss_compress(_dev(w.F), _dev(w.y), w.h, w.leaf, w.tol)
        exps.append(ctx.hss_export())
        ctx.close()
    for key in ("perm", "ranks", "U", "J", "B", "D"):
        assert np.array_equal(exps[0][key], exps[1][key]), key
    assert exps[0]["delta"] == exps[1]["delta"]
