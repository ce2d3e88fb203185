"""GPU tests of the building blocks (matrix-core GEMM, batched LU / Cholesky / inverse, row
interpolative decomposition, kernel sampling, the Omega generator) against NumPy and the oracle."""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def L():
    from gpu_helpers import lib
    return lib()


def test_mfma_f64_lane_layout(L):
    """The layout the kernels assume: A[l%16][l/16], B[l/16][l%16], accumulator v of lane l = D[4v + l/16][l%16]."""
    import torch
    from gpu_helpers import dev, ptr
    rng = np.random.default_rng(0)
    A = rng.standard_normal((16, 4))
    B = rng.standard_normal((4, 16))
    a = np.array([A[l % 16, l // 16] for l in range(64)])
    b = np.array([B[l // 16, l % 16] for l in range(64)])
    d = torch.zeros(256, dtype=torch.float64, device="cuda:0")
    assert L.hsx_probe_mfma(ptr(dev(a)), ptr(dev(b)), ptr(d)) == 0
    d = d.cpu().numpy().reshape(64, 4)
    Dm = A @ B
    for l in range(64):
        for v in range(4):
            assert abs(d[l, v] - Dm[4 * v + l // 16, l % 16]) < 1e-13


def _bgemm(L, shapes, ta, tb, alpha, beta, seed=0):
    from gpu_helpers import dev, hptr, ptr
    rng = np.random.default_rng(seed)
    host, dims, offs, mats = [], [], [], []
    off = 0
    for (M, N, K) in shapes:
        Ah = rng.standard_normal((K, M) if ta else (M, K))
        Bh = rng.standard_normal((N, K) if tb else (K, N))
        Ch = rng.standard_normal((M, N))
        oa, ob, oc = off, off + Ah.size, off + Ah.size + Bh.size
        off = oc + Ch.size
        host += [Ah.ravel(), Bh.ravel(), Ch.ravel()]
        dims += [M, N, K, max(1, Ah.shape[1]), max(1, Bh.shape[1]), max(1, N)]
        offs += [oa, ob, oc]
        mats.append((Ah, Bh, Ch, oc))
    base = dev(np.concatenate(host + [np.zeros(1)]))
    dims = np.array(dims, dtype=np.int32)
    offs = np.array(offs, dtype=np.int64)
    L.hsx_bgemm.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_double, C.c_double]
    assert L.hsx_bgemm(None, len(shapes), hptr(dims), hptr(offs), ptr(base), int(ta), int(tb), alpha, beta) == 0
    out = base.cpu().numpy()
    worst = 0.0
    for (Ah, Bh, Ch, oc), (M, N, K) in zip(mats, shapes):
        if M * N == 0:
            continue
        ref = alpha * ((Ah.T if ta else Ah) @ (Bh.T if tb else Bh)) + beta * Ch
        got = out[oc:oc + M * N].reshape(M, N)
        worst = max(worst, np.abs(got - ref).max() / (np.abs(ref).max() + 1e-300))
    return worst


@pytest.mark.parametrize("ta", [0, 1])
@pytest.mark.parametrize("tb", [0, 1])
def test_batched_gemm(L, ta, tb):
    shapes = [(64, 64, 16), (1, 1, 1), (70, 33, 5), (129, 200, 77), (16, 300, 130), (300, 17, 64), (5, 5, 0),
              (100, 100, 100), (502, 512, 1004)]
    assert _bgemm(L, shapes, ta, tb, 1.0, 0.0) < 1e-13            # items of 128 x 128 and more: the 128 x 128-tile kernel
    assert _bgemm(L, shapes, ta, tb, -0.5, 1.0, seed=1) < 1e-13
    small = [(64, 64, 16), (1, 1, 1), (70, 33, 5), (100, 127, 77), (127, 100, 130), (16, 127, 300), (5, 5, 0)]
    assert _bgemm(L, small, ta, tb, 1.0, 0.0, seed=2) < 1e-13       # the 64 x 64-tile kernel
    assert _bgemm(L, small, ta, tb, 2.0, -1.0, seed=3) < 1e-13


def test_gemm_tile_sizes_give_the_same_bits(L):
    """One 200 x 200 x 77 product as a single item (the 128 x 128-tile kernel) and as four 100 x 100 quadrants (the
    64 x 64-tile kernel) of the same operands: every output element adds its k-steps in the same order."""
    from gpu_helpers import dev, hptr, ptr
    rng = np.random.default_rng(9)
    M = N = 200
    K = 77
    A, B = rng.standard_normal((M, K)), rng.standard_normal((K, N))
    oa, ob, oc1, oc2 = 0, M * K, M * K + K * N, M * K + K * N + M * N
    base = dev(np.concatenate([A.ravel(), B.ravel(), np.zeros(2 * M * N + 1)]))
    L.hsx_bgemm.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_double, C.c_double]
    dims = np.array([M, N, K, K, N, N], dtype=np.int32)
    offs = np.array([oa, ob, oc1], dtype=np.int64)
    assert L.hsx_bgemm(None, 1, hptr(dims), hptr(offs), ptr(base), 0, 0, 1.0, 0.0) == 0
    dims4, offs4 = [], []
    for bi in range(2):
        for bj in range(2):
            dims4 += [100, 100, K, K, N, N]
            offs4 += [oa + bi * 100 * K, ob + bj * 100, oc2 + bi * 100 * N + bj * 100]
    dims4 = np.array(dims4, dtype=np.int32)
    offs4 = np.array(offs4, dtype=np.int64)
    assert L.hsx_bgemm(None, 4, hptr(dims4), hptr(offs4), ptr(base), 0, 0, 1.0, 0.0) == 0
    out = base.cpu().numpy()
    C1, C2 = out[oc1:oc1 + M * N], out[oc2:oc2 + M * N]
    assert np.abs(C1.reshape(M, N) - A @ B).max() < 1e-12
    assert np.array_equal(C1, C2)


def test_batched_inverse_with_pivoting(L):
    from gpu_helpers import dev, hptr, ptr
    rng = np.random.default_rng(2)
    sizes = [1, 2, 5, 31, 32, 33, 64, 100, 257, 502, 1004]
    mats, host, offs = [], [], []
    off = 0
    for n in sizes:
        A = rng.standard_normal((n, n))
        if n >= 5:
            A[0, 0] = 0.0            # forces a row interchange at the first step
            A = A + A.T              # symmetric indefinite, as a loose compressed matrix can be
        mats.append(A)
        host += [A.ravel(), np.zeros(n * n)]
        offs += [off, off + n * n]
        off += 2 * n * n
    base = dev(np.concatenate(host))
    ns = np.array(sizes, dtype=np.int32)
    offs = np.array(offs, dtype=np.int64)
    flag = np.zeros(1, dtype=np.int32)
    assert L.hsx_inverse(None, len(sizes), hptr(ns), hptr(offs), ptr(base), hptr(flag)) == 0
    out = base.cpu().numpy()
    for A, n, i in zip(mats, sizes, range(len(sizes))):
        X = out[offs[2 * i + 1]:offs[2 * i + 1] + n * n].reshape(n, n)
        res = np.linalg.norm(A @ X - np.eye(n)) / (np.linalg.cond(A) * np.sqrt(n))
        assert res < 1e-13, (n, res)
    assert flag[0] == 0


def test_batched_cholesky(L):
    from gpu_helpers import dev, hptr, ptr
    rng = np.random.default_rng(3)
    sizes = [1, 3, 32, 33, 65, 200, 502]
    mats, host, offs = [], [], []
    off = 0
    for n in sizes:
        T = rng.standard_normal((n + 3, n))
        A = np.eye(n) + T.T @ T          # the shape of matrix the factorization meets: I + T^T T
        mats.append(A)
        host.append(A.ravel())
        offs.append(off)
        off += n * n
    base = dev(np.concatenate(host))
    assert L.hsx_chol(None, len(sizes), hptr(np.array(sizes, dtype=np.int32)), hptr(np.array(offs, dtype=np.int64)),
                      ptr(base)) == 0
    out = base.cpu().numpy()
    for A, n, o in zip(mats, sizes, offs):
        Lc = out[o:o + n * n].reshape(n, n)
        assert np.array_equal(np.triu(Lc, 1), np.zeros((n, n)))
        assert np.linalg.norm(Lc @ Lc.T - A) <= 1e-13 * np.linalg.norm(A)
        assert np.allclose(Lc, np.linalg.cholesky(A), rtol=1e-11, atol=1e-12)


def _row_id(L, blocks, ld, kcap, rel, abs_tol, gram=0):
    import torch
    from gpu_helpers import dev, hptr, ptr
    rows = sum(b.shape[0] for b in blocks)
    A = np.zeros((rows, ld))
    moff = [0]
    for b in blocks:
        A[moff[-1]:moff[-1] + b.shape[0], :b.shape[1]] = b
        moff.append(moff[-1] + b.shape[0])
    moff = np.array(moff, dtype=np.int64)
    nn = len(blocks)
    ranks = np.zeros(nn, dtype=np.int32)
    J = np.zeros((nn, kcap), dtype=np.int32)
    U = torch.zeros(rows * kcap, dtype=torch.float64, device="cuda:0")
    L.hsx_row_id.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_double, C.c_double,
                             C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
    assert L.hsx_row_id(None, ptr(dev(A)), ld, nn, hptr(moff), kcap, rel, abs_tol, gram, hptr(ranks), hptr(J),
                        ptr(U)) == 0
    U = U.cpu().numpy()
    out, uo = [], 0
    for t, b in enumerate(blocks):
        m, k = b.shape[0], int(ranks[t])
        out.append((k, J[t, :k].copy(), U[uo:uo + m * k].reshape(m, k)))
        uo += m * k
    return out


def test_row_id_ragged_blocks(L):
    from oracle import hss as ohss
    rng = np.random.default_rng(4)
    blocks = []
    for (m, rank, cols) in [(64, 5, 128), (100, 17, 128), (33, 33, 100), (256, 40, 128), (16, 1, 64), (200, 128, 128)]:
        Qa, _ = np.linalg.qr(rng.standard_normal((m, min(m, rank))))
        Qb, _ = np.linalg.qr(rng.standard_normal((cols, min(m, rank))))
        sv = 2.0 ** -np.arange(min(m, rank))
        blocks.append((Qa * sv) @ Qb.T)
    rel, kcap = 1e-9, 120
    res = _row_id(L, blocks, 128, kcap, rel, 0.0)
    for (k, J, U), b in zip(res, blocks):
        m = b.shape[0]
        Jo, Uo = ohss.row_id(b, rel, 0.0, kcap)
        assert abs(k - Jo.size) <= 2, (k, Jo.size)
        assert len(set(J.tolist())) == k and J.min() >= 0 and J.max() < m
        assert np.array_equal(U[J], np.eye(k))
        err = np.linalg.norm(b - U @ b[J]) / np.linalg.norm(b)
        assert err <= 1e-7, (m, k, err)
        assert np.abs(U).max() <= 20.0


def _decaying_blocks(rng, shapes, decay):
    """Blocks with singular values decay^j (ragged sizes, more columns than the numerical rank)."""
    blocks = []
    for (m, cols) in shapes:
        k = min(m, cols)
        Qa, _ = np.linalg.qr(rng.standard_normal((m, k)))
        Qb, _ = np.linalg.qr(rng.standard_normal((cols, k)))
        blocks.append((Qa * decay ** np.arange(k)) @ Qb.T)
    return blocks


@pytest.mark.parametrize("rel", [1e-2, 1e-3, 1e-4, 3e-5])
@pytest.mark.parametrize("gram", [1, 0])
def test_row_id_meets_the_tolerance_in_both_forms(L, rel, gram):
    """Truncation of a block to a relative threshold (end of Sec. 3.2) where the threshold, not the cap, stops
    the decomposition: the form built on the Gram matrix (the one the compression runs for thresholds of 3e-6
    and above, i.e. on every workload) and the Gram-Schmidt form against the oracle's pivoted Householder QR.
    The first discarded pivot is the largest remaining row norm, so every row of A - U A[J] is at most the
    threshold long; the bound asserted is twice that."""
    from oracle import hss as ohss
    rng = np.random.default_rng(11)
    shapes = [(64, 128), (100, 128), (33, 100), (256, 128), (16, 64), (200, 128), (512, 256), (130, 256)]
    for decay, ld in ((0.8, 256), (0.93, 256)):
        blocks = _decaying_blocks(rng, shapes, decay)
        kcap = 250
        res = _row_id(L, blocks, ld, kcap, rel, 0.0, gram)
        for (k, J, U), b in zip(res, blocks):
            m = b.shape[0]
            Jo, Uo = ohss.row_id(b, rel, 0.0, kcap)
            assert abs(k - Jo.size) <= 2, (m, k, Jo.size)
            assert len(set(J.tolist())) == k and J.min() >= 0 and J.max() < m
            assert np.array_equal(U[J], np.eye(k))
            r00 = np.linalg.norm(b, axis=1).max()                # the first pivot: the longest row
            resid = np.linalg.norm(b - U @ b[J], axis=1).max()
            assert resid <= 2.0 * rel * r00, (m, k, resid / r00)
            # and as good as the oracle's decomposition of the same block
            resid_o = np.linalg.norm(b - Uo @ b[Jo], axis=1).max()
            assert resid <= max(3.0 * resid_o, rel * r00)
            assert np.abs(U).max() <= 10.0


def test_row_id_rank_cap_and_zero_block(L):
    rng = np.random.default_rng(5)
    blocks = [rng.standard_normal((80, 128)), np.zeros((32, 128)), rng.standard_normal((48, 128)) * 1e-12]
    res = _row_id(L, blocks, 128, 20, 1e-6, 1e-8)
    assert res[0][0] == 20                       # cap
    assert res[1][0] == 1 and np.all(np.isfinite(res[1][2]))   # a zero block keeps one row, U finite
    assert res[2][0] == 1                        # below the absolute threshold after the first pivot


@pytest.mark.parametrize("n,r,s,h", [(512, 8, 128, 1.5), (1000, 22, 256, 2.0), (777, 54, 512, 3.0), (300, 90, 100, 4.0),
                                     (2048, 3, 384, 0.7), (256, 1, 1, 0.5)])
def test_kernel_sample_matches_oracle(n, r, s, h):
    from gpu_helpers import dev
    from oracle import hss as ohss
    from paper_2108_04167_amd import binding
    rng = np.random.default_rng(n + s)
    F = rng.standard_normal((n, r))
    Om = rng.standard_normal((n, s))
    ctx = binding.Context()
    S = ctx.hss_kernel_sample(dev(F), h, dev(Om)).cpu().numpy()
    ref = ohss.sample(F, Om, h)
    assert np.abs(S - ref).max() <= 1e-12 * np.abs(ref).max()
    ctx.close()


def _philox4x32_10(ctr, key):
    """Philox4x32-10 from its published definition (Salmon et al., SC'11)."""
    M0, M1, W0, W1 = 0xD2511F53, 0xCD9E8D57, 0x9E3779B9, 0xBB67AE85
    c = list(ctr)
    k = list(key)
    for _ in range(10):
        p0, p1 = M0 * c[0], M1 * c[2]
        c = [((p1 >> 32) ^ c[1] ^ k[0]) & 0xFFFFFFFF, p1 & 0xFFFFFFFF, ((p0 >> 32) ^ c[3] ^ k[1]) & 0xFFFFFFFF, p0 & 0xFFFFFFFF]
        k = [(k[0] + W0) & 0xFFFFFFFF, (k[1] + W1) & 0xFFFFFFFF]
    return c


def test_omega_generator(L):
    import math
    import torch
    from gpu_helpers import ptr
    n, s, seed = 4096, 100, 12345
    Om = torch.zeros((n, s), dtype=torch.float64, device="cuda:0")
    L.hsx_omega.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_uint64]
    assert L.hsx_omega(None, ptr(Om), n, s, seed) == 0
    Om = Om.cpu().numpy()
    assert abs(Om.mean()) < 0.01 and abs(Om.std() - 1.0) < 0.01
    assert abs(np.mean(Om ** 4) - 3.0) < 0.1
    assert abs(np.corrcoef(Om[:, 0], Om[:, 1])[0, 1]) < 0.06
    # bits: element (row, col) comes from the Philox block with counter (row, 0, col//2, 0) and key (seed, 0)
    for (row, col) in [(0, 0), (0, 1), (7, 42), (4095, 99)]:
        o = _philox4x32_10([row, 0, col // 2, 0], [seed & 0xFFFFFFFF, seed >> 32])
        a = ((o[0] << 32) | o[1]) >> 11
        b = ((o[2] << 32) | o[3]) >> 11
        u1 = (a + 0.5) / 2.0 ** 53
        u2 = (b + 0.5) / 2.0 ** 53
        rad = math.sqrt(-2.0 * math.log(u1))
        val = rad * (math.cos(2 * math.pi * u2) if col % 2 == 0 else math.sin(2 * math.pi * u2))
        assert Om[row, col] == pytest.approx(val, rel=1e-12, abs=1e-13)
