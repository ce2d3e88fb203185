// Entry points used only by the GPU unit tests of the building blocks.  They are built into a library of
// their own (libhsssvm_hooks.so, linked against libhsssvm.so) so that the shipped library exports nothing
// but the C ABI of include/hss_svm.h; declarations in test_hooks.h.
#include "test_hooks.h"
#include "../csrc/common.h"
#include <algorithm>

namespace {
__global__ void probe_mfma_kernel(const double* a, const double* b, double* d) {
    int l = threadIdx.x;
    v4d acc = (v4d){0.0, 0.0, 0.0, 0.0};
    acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a[l], b[l], acc, 0, 0, 0);
    for (int v = 0; v < 4; ++v) d[l * 4 + v] = acc[v];
}
}  // namespace

extern "C" {

// d[l*4+v] = accumulator register v of lane l after one 16x16x4 f64 MFMA with per-lane operands a[l], b[l].
int hsx_probe_mfma(const double* a_dev, const double* b_dev, double* d_dev) {
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(1), dim3(64), 0, 0, a_dev, b_dev, d_dev);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipDeviceSynchronize());
    return HSS_OK;
}

// Batched GEMM on matrices living in one device buffer `base`: item i uses offsets offs[3i..3i+2]
// (in doubles) and dims[6i..6i+5] = M, N, K, lda, ldb, ldc.
int hsx_bgemm(void* stream, int nitems, const int32_t* dims_host, const int64_t* offs_host, double* base_dev, int transA,
              int transB, double alpha, double beta) {
    hipStream_t st = (hipStream_t)stream;
    std::vector<GemmItem> items(nitems);
    int maxM = 0, maxN = 0;
    for (int i = 0; i < nitems; ++i) {
        const int32_t* d = dims_host + 6 * i;
        items[i] = GemmItem{base_dev + offs_host[3 * i], base_dev + offs_host[3 * i + 1], base_dev + offs_host[3 * i + 2],
                            d[0], d[1], d[2], d[3], d[4], d[5]};
        if (d[0] > maxM) maxM = d[0];
        if (d[1] > maxN) maxN = d[1];
    }
    DevBuf tab;
    HSS_TRY(tab.reserve(sizeof(GemmItem) * (size_t)nitems));
    HIP_TRY(hipMemcpyAsync(tab.p, items.data(), sizeof(GemmItem) * (size_t)nitems, hipMemcpyHostToDevice, st));
    HSS_TRY(bgemm(st, tab.as<GemmItem>(), nitems, maxM, maxN, transA != 0, transB != 0, alpha, beta));
    HIP_TRY(hipStreamSynchronize(st));
    return HSS_OK;
}

}  // extern "C"

// ---- building blocks exercised by tests/test_gpu_blocks.py ----
#include "../csrc/dense.h"
#include "../csrc/levels.h"
#include "../csrc/rowid.h"

extern "C" {

// Inverse of nmat square matrices living in `base` (row-major, tight): offs[2i] = A_i (destroyed),
// offs[2i+1] = X_i (output).
int hsx_inverse(void* stream, int nmat, const int32_t* n_host, const int64_t* offs_host, double* base_dev,
                int32_t* flags_out_host) {
    hipStream_t st = (hipStream_t)stream;
    DescArena ar;
    HSS_TRY(ar.init(size_t(32) << 20));
    DevBuf piv, flags;
    int64_t tot = 0;
    for (int i = 0; i < nmat; ++i) tot += n_host[i];
    HSS_TRY(piv.reserve(sizeof(int) * std::max<int64_t>(tot, 1)));
    HSS_TRY(flags.reserve(sizeof(int) * 4));
    HIP_TRY(hipMemsetAsync(flags.p, 0, sizeof(int) * 4, st));
    std::vector<LUItem> lu(nmat);
    std::vector<double*> X(nmat);
    std::vector<int> ldx(nmat);
    int64_t po = 0;
    for (int i = 0; i < nmat; ++i) {
        lu[i] = LUItem{base_dev + offs_host[2 * i], piv.as<int>() + po, n_host[i], n_host[i]};
        X[i] = base_dev + offs_host[2 * i + 1];
        ldx[i] = n_host[i];
        po += n_host[i];
    }
    HSS_TRY(bgetrf(st, ar, lu, true, 1e-13, flags.as<int>()));
    HSS_TRY(bgetri(st, ar, lu, X, ldx));
    HIP_TRY(hipMemcpyAsync(flags_out_host, flags.p, sizeof(int), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    return HSS_OK;
}

// In-place Cholesky (lower factor, strict upper triangle zeroed) of nmat SPD matrices at offs[i].
int hsx_chol(void* stream, int nmat, const int32_t* n_host, const int64_t* offs_host, double* base_dev) {
    hipStream_t st = (hipStream_t)stream;
    DescArena ar;
    HSS_TRY(ar.init(size_t(32) << 20));
    DevBuf sc, flags;
    HSS_TRY(sc.reserve(sizeof(double) * (size_t)nmat * 1024));
    HSS_TRY(flags.reserve(sizeof(int) * 4));
    HIP_TRY(hipMemsetAsync(flags.p, 0, sizeof(int) * 4, st));
    std::vector<LUItem> lu(nmat);
    for (int i = 0; i < nmat; ++i) lu[i] = LUItem{base_dev + offs_host[i], nullptr, n_host[i], n_host[i]};
    HSS_TRY(bchol(st, ar, lu, sc.as<double>(), flags.as<int>()));
    HIP_TRY(hipStreamSynchronize(st));
    return HSS_OK;
}

// Row interpolative decompositions of `nnodes` row blocks of A (rows x ld, ld a multiple of 128, <= 512);
// block t = rows moff[t] .. moff[t+1].  gram = 0: row-pivoted Gram-Schmidt on the rows (one launch per pivot
// step); gram = 1: pivoted Cholesky of the blocks' Gram matrices A_t A_t^T (the form the compression uses for
// relative thresholds of 3e-6 and above).  Outputs: ranks (host), J (host, nnodes x kcap), U (device, tight
// msz_t x k_t blocks one after the other in node order; caller sizes it as rows x kcap).
int hsx_row_id(void* stream, const double* A_dev, int32_t ld, int32_t nnodes, const int64_t* moff_host, int32_t kcap,
               double rel, double abs_tol, int32_t gram, int32_t* ranks_host, int32_t* J_host, double* U_dev) {
    return hsx_row_id_blocks(stream, A_dev, ld, nnodes, moff_host, kcap, rel, abs_tol, gram, 32, ranks_host, J_host, U_dev);
}

// The same with the number of rows a workgroup of the row-wise kernels takes (the library uses 32): a different
// split of the same work over the grid must give the same bits.
int hsx_row_id_blocks(void* stream, const double* A_dev, int32_t ld, int32_t nnodes, const int64_t* moff_host, int32_t kcap,
                      double rel, double abs_tol, int32_t gram, int32_t rows_per_block, int32_t* ranks_host,
                      int32_t* J_host, double* U_dev) {
    if (rows_per_block < 4 || rows_per_block % 4) return HSS_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    const int64_t rows = moff_host[nnodes];
    int maxm = 0;
    for (int t = 0; t < nnodes; ++t) maxm = std::max<int>(maxm, (int)(moff_host[t + 1] - moff_host[t]));
    DevBuf W, moff, Lc, n0, n1, sel, jtmp, rk, done, r11, koffd, uoffd, Jd;
    HSS_TRY(W.reserve(sizeof(double) * rows * ld));
    HSS_TRY(moff.reserve(sizeof(int64_t) * (nnodes + 1)));
    HSS_TRY(Lc.reserve(sizeof(double) * rows * kcap));
    HSS_TRY(n0.reserve(sizeof(double) * rows));
    HSS_TRY(n1.reserve(sizeof(double) * rows));
    HSS_TRY(sel.reserve(sizeof(int) * rows));
    HSS_TRY(jtmp.reserve(sizeof(int) * (size_t)nnodes * kcap));
    HSS_TRY(rk.reserve(sizeof(int) * nnodes));
    HSS_TRY(done.reserve(sizeof(int) * nnodes));
    HSS_TRY(r11.reserve(sizeof(double) * nnodes));
    HIP_TRY(hipMemcpyAsync(W.p, A_dev, sizeof(double) * rows * ld, hipMemcpyDeviceToDevice, st));
    HIP_TRY(hipMemcpyAsync(moff.p, moff_host, sizeof(int64_t) * (nnodes + 1), hipMemcpyHostToDevice, st));
    IdLevelArgs ia;
    ia.W = W.as<double>(); ia.ld = ld; ia.moff = moff.as<int64_t>(); ia.kcap = kcap; ia.kc = kcap; ia.rows_per_block = rows_per_block;
    ia.rel = rel; ia.abs_tol = abs_tol; ia.done = done.as<int>(); ia.r11 = r11.as<double>(); ia.jtmp = jtmp.as<int>();
    ia.rk = rk.as<int>(); ia.Lc = Lc.as<double>(); ia.sel = sel.as<int>(); ia.active = nullptr;
    if (gram) {
        DescArena ar;
        HSS_TRY(ar.init(size_t(8) << 20));
        DevBuf Gm, goffd;
        std::vector<int64_t> goff(nnodes + 1, 0);
        std::vector<GemmItem> gg(nnodes);
        for (int t = 0; t < nnodes; ++t) {
            const int64_t m = moff_host[t + 1] - moff_host[t];
            goff[t + 1] = goff[t] + m * m;
        }
        HSS_TRY(Gm.reserve(sizeof(double) * std::max<int64_t>(goff[nnodes], 1)));
        HSS_TRY(goffd.reserve(sizeof(int64_t) * (nnodes + 1)));
        HIP_TRY(hipMemcpyAsync(goffd.p, goff.data(), sizeof(int64_t) * (nnodes + 1), hipMemcpyHostToDevice, st));
        for (int t = 0; t < nnodes; ++t) {
            const int m = (int)(moff_host[t + 1] - moff_host[t]);
            const double* At = W.as<double>() + (size_t)moff_host[t] * ld;
            gg[t] = GemmItem{At, At, Gm.as<double>() + goff[t], m, m, ld, ld, ld, m};
        }
        HSS_TRY(bgemm_host(st, ar, gg, false, true, 1.0, 0.0));
        HIP_TRY(hipMemsetAsync(Lc.p, 0, sizeof(double) * rows * kcap, st));
        HSS_TRY(id_chol(st, ia, nnodes, maxm, Gm.as<double>(), goffd.as<int64_t>()));
        HIP_TRY(hipStreamSynchronize(st));   // the arena and the Gram matrices go out of scope
    } else {
        HSS_TRY(id_init(st, ia, nnodes, maxm, n0.as<double>()));
        HSS_TRY(id_steps(st, ia, nnodes, maxm, n0.as<double>(), n1.as<double>()));
    }
    HIP_TRY(hipMemcpyAsync(ranks_host, rk.p, sizeof(int) * nnodes, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    std::vector<int64_t> koff(nnodes + 1, 0), uoff(nnodes + 1, 0);
    for (int t = 0; t < nnodes; ++t) {
        koff[t + 1] = koff[t] + ranks_host[t];
        uoff[t + 1] = uoff[t] + (int64_t)ranks_host[t] * (moff_host[t + 1] - moff_host[t]);
    }
    HSS_TRY(koffd.reserve(sizeof(int64_t) * (nnodes + 1)));
    HSS_TRY(uoffd.reserve(sizeof(int64_t) * (nnodes + 1)));
    HSS_TRY(Jd.reserve(sizeof(int) * std::max<int64_t>(koff[nnodes], 1)));
    HIP_TRY(hipMemcpyAsync(koffd.p, koff.data(), sizeof(int64_t) * (nnodes + 1), hipMemcpyHostToDevice, st));
    HIP_TRY(hipMemcpyAsync(uoffd.p, uoff.data(), sizeof(int64_t) * (nnodes + 1), hipMemcpyHostToDevice, st));
    HSS_TRY(id_finish(st, ia, nnodes, maxm, koffd.as<int64_t>(), uoffd.as<int64_t>(), U_dev, Jd.as<int>()));
    std::vector<int> Jt(std::max<int64_t>(koff[nnodes], 1));
    HIP_TRY(hipMemcpyAsync(Jt.data(), Jd.p, sizeof(int) * koff[nnodes], hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    for (int t = 0; t < nnodes; ++t)
        for (int j = 0; j < ranks_host[t]; ++j) J_host[(size_t)t * kcap + j] = Jt[koff[t] + j];
    return HSS_OK;
}

// Omega as hss_compress would draw it (n x s, row-major, tight).
int hsx_omega(void* stream, double* Om_dev, int64_t n, int32_t s, uint64_t seed) {
    hipStream_t st = (hipStream_t)stream;
    const int64_t n_pad = round_up(n, 256);
    const int s_pad = (int)round_up(s, 128);
    DevBuf tmp;
    HSS_TRY(tmp.reserve(sizeof(double) * n_pad * s_pad));
    HSS_TRY(omega_fill_launch(st, tmp.as<double>(), n, n_pad, s, s_pad, seed));
    HIP_TRY(hipMemcpy2DAsync(Om_dev, sizeof(double) * s, tmp.p, sizeof(double) * s_pad, sizeof(double) * s, n,
                             hipMemcpyDeviceToDevice, st));
    HIP_TRY(hipStreamSynchronize(st));
    return HSS_OK;
}

}  // extern "C"
