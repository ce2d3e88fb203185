// Kernel products for more features than the fused kernels hold in LDS (padded feature count above 112):
// S = K(rows, cols) * Omega through row stripes of the kernel matrix formed in HBM --
//   Gram stripe  G = F_rows F_cols^T                              batched GEMM on the matrix cores,
//   K stripe     exp(min(0, G/h^2 - nu_i/(2h^2) - nu_j/(2h^2)))   elementwise, in place,
//   S stripe     K stripe * Omega                                  batched GEMM.
// The stripe costs 16 bytes of HBM traffic per kernel entry on top of the matrix work, which the fused kernels avoid;
// it is the fallback for wide data (hundreds of features), where the Gram part dominates anyway.
#include "common.h"
#include <algorithm>

namespace {

// G[i][j] <- exp(min(0, G[i][j] / h^2 - nu_r[i] / (2h^2) - nu_c[j] / (2h^2))), G rows x cols with leading dimension cols
__global__ __launch_bounds__(256) void stripe_exp_kernel(double* __restrict__ G, int64_t rows, int64_t cols,
                                                         const double* __restrict__ nur, const double* __restrict__ nuc,
                                                         double inv2h2) {
    const int64_t total = rows * cols;
    for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
        const int64_t i = idx / cols, j = idx - i * cols;
        double x = 2.0 * inv2h2 * G[idx] - inv2h2 * (nur[i] + nuc[j]);
        x = x < 0.0 ? x : 0.0;
        G[idx] = exp(x);
    }
}

}  // namespace

// Same contract as sample_launch_window (sample.hip) for any r_pad: S (nr_pad x width, leading dimension ld) =
// K(rows, cols) Om, rows = the points (Fr, nur), cols = the points (Fp, nu), Om n_pad x width (leading dimension ld).
// Allocates its stripe (at most 8 GB) and returns after the stream has drained.
int sample_wide_launch(hipStream_t st, const double* Fr, const double* nur, int64_t nr_pad, const double* Fp,
                       const double* nu, int64_t n_pad, const double* Om, double* S, int r_pad, int width, int ld,
                       double h) {
    if (n_pad < 64 || nr_pad < 64 || n_pad % 64 || nr_pad % 64 || r_pad < 1 || width < 1 || ld < width ||
        n_pad >= (int64_t(1) << 31) || nr_pad >= (int64_t(1) << 31))
        return HSS_EUNSUPPORTED;
    const double inv2h2 = 1.0 / (2.0 * h * h);
    // stripe height: 2^30 doubles, whole 64-row tiles, and few enough tiles for one launch of the contraction
    int64_t rb = (int64_t(1) << 30) / n_pad / 64 * 64;
    rb = std::max<int64_t>(64, std::min(rb, nr_pad));
    const int64_t tilesW = (width + 63) / 64;
    while (rb > 64 && (rb / 64) * tilesW > 65535) rb -= 64;
    DevBuf G, items_dev;
    HSS_TRY(G.reserve(sizeof(double) * (size_t)rb * n_pad));
    // Gram stripe in column panels, so that one item has at most 65535 tiles
    const int64_t tilesM = rb / 64;
    const int64_t pc = std::max<int64_t>(64, 65535 / tilesM * 64);
    std::vector<GemmItem> items;
    HSS_TRY(items_dev.reserve(sizeof(GemmItem) * (size_t)((n_pad + pc - 1) / pc + 1)));
    for (int64_t r0 = 0; r0 < nr_pad; r0 += rb) {
        const int64_t rows = std::min(rb, nr_pad - r0);
        items.clear();
        for (int64_t c0 = 0; c0 < n_pad; c0 += pc)
            items.push_back(GemmItem{Fr + (size_t)r0 * r_pad, Fp + (size_t)c0 * r_pad, G.as<double>() + c0, (int32_t)rows,
                                     (int32_t)std::min(pc, n_pad - c0), r_pad, r_pad, r_pad, (int32_t)n_pad});
        HIP_TRY(hipMemcpyAsync(items_dev.p, items.data(), sizeof(GemmItem) * items.size(), hipMemcpyHostToDevice, st));
        HSS_TRY(bgemm(st, items_dev.as<GemmItem>(), (int)items.size(), (int)rows, (int)std::min(pc, n_pad), false, true, 1.0,
                      0.0));
        hipLaunchKernelGGL(stripe_exp_kernel, dim3(8192), dim3(256), 0, st, G.as<double>(), rows, n_pad, nur + r0, nu,
                           inv2h2);
        HIP_TRY(hipGetLastError());
        HIP_TRY(hipStreamSynchronize(st));        // the item table is rewritten for the contraction
        const GemmItem ci{G.as<double>(), Om, S + (size_t)r0 * ld, (int32_t)rows, width, (int32_t)n_pad, (int32_t)n_pad, ld, ld};
        HIP_TRY(hipMemcpyAsync(items_dev.p, &ci, sizeof(GemmItem), hipMemcpyHostToDevice, st));
        HSS_TRY(bgemm(st, items_dev.as<GemmItem>(), 1, (int)rows, width, false, false, 1.0, 0.0));
        HIP_TRY(hipStreamSynchronize(st));        // `ci` and the item table are reused by the next stripe
    }
    return HSS_OK;
}

// S = K(rows, cols) Om for a column window, by the fused kernel when the features fit it, else through stripes.
int kernel_product_launch(hipStream_t st, const double* Fr, const double* nur, int64_t nr_pad, const double* Fp,
                          const double* nu, int64_t n_pad, const double* Om, double* S, int r_pad, int width, int ld,
                          double h) {
    if (r_pad <= 112) return sample_launch_window(st, Fr, nur, nr_pad, Fp, nu, n_pad, Om, S, r_pad, width, ld, h);
    return sample_wide_launch(st, Fr, nur, nr_pad, Fp, nu, n_pad, Om, S, r_pad, width, ld, h);
}
