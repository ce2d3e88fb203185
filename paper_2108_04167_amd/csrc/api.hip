// C ABI of libhsssvm (see include/hss_svm.h for the contract of every call).
#include "ctx.h"
#include <algorithm>
#include <cmath>
#include <cstring>

extern "C" {

const char* hss_strerror(int code) {
    switch (code) {
        case HSS_OK: return "ok";
        case HSS_EINVAL: return "invalid argument";
        case HSS_ESTATE: return "call out of order";
        case HSS_ENOMEM: return "out of memory";
        case HSS_EHIP: return "HIP runtime error";
        case HSS_EUNSUPPORTED: return "size not supported by the kernels";
        default: break;
    }
    if (code > 0) return "completed with numerical warnings (bit mask of HSS_W*)";
    return "unknown error";
}

int hss_create(hss_ctx** out, void* hip_stream) {
    if (!out) return HSS_EINVAL;
    hss_ctx* c = new (std::nothrow) hss_ctx();
    if (!c) return HSS_ENOMEM;
    c->stream = (hipStream_t)hip_stream;
    // set-up of the allocation-free entry point: the scratch array's address on this device.  A failure here
    // is not one of hss_create (the entry point asks again and reports it).
    double* unused = nullptr;
    (void)noalloc_scratch_for_current_device(&unused);
    *out = c;
    return HSS_OK;
}

void hss_destroy(hss_ctx* ctx) {
    if (!ctx) return;
    (void)hipStreamSynchronize(ctx->stream);
    if (ctx->gstream) {
        (void)hipStreamSynchronize(ctx->gstream);
        (void)hipStreamDestroy(ctx->gstream);
    }
    if (ctx->gevent) (void)hipEventDestroy(ctx->gevent);
    delete ctx;
}

int hss_set_i64(hss_ctx* c, const char* key, int64_t v) {
    if (!c || !key) return HSS_EINVAL;
    if (!strcmp(key, "sample_width")) { if (v < 1) return HSS_EINVAL; c->opt_s = v; }
    else if (!strcmp(key, "oversample")) { if (v < 0) return HSS_EINVAL; c->opt_p = v; }
    else if (!strcmp(key, "max_rank")) { if (v < 0) return HSS_EINVAL; c->opt_max_rank = v; }
    else if (!strcmp(key, "seed")) c->opt_seed = v;
    else if (!strcmp(key, "psd_guard")) c->opt_guard = v ? 1 : 0;
    else if (!strcmp(key, "merge_top")) c->opt_merge_top = v ? 1 : 0;
    else if (!strcmp(key, "graph")) c->opt_graph = v ? 1 : 0;
    else if (!strcmp(key, "sampling")) { if (v != 0 && v != 1) return HSS_EINVAL; c->opt_sampling = v; }
    else if (!strcmp(key, "ann_neighbours")) { if (v < 1 || v > 64) return HSS_EINVAL; c->opt_ann_k = v; }
    else if (!strcmp(key, "ann_cell")) { if (v < 2 || v > (1 << 20)) return HSS_EINVAL; c->opt_ann_cell = v; }
    else if (!strcmp(key, "ann_trees")) { if (v < 1 || v > 64) return HSS_EINVAL; c->opt_ann_trees = v; }
    else if (!strcmp(key, "clustering")) { if (v != 0 && v != 1) return HSS_EINVAL; c->opt_cluster = v; }
    else if (!strcmp(key, "clustering_iterations")) { if (v < 0 || v > 64) return HSS_EINVAL; c->opt_cluster_iters = v; }
    else if (!strcmp(key, "cache_basis")) { c->opt_cache_basis = v ? 1 : 0; if (!v) c->basis_cached = false; }
    else if (!strcmp(key, "adaptive_start")) { if (v < 0) return HSS_EINVAL; c->opt_adapt_start = v; }
    else if (!strcmp(key, "adaptive_step")) { if (v < 1) return HSS_EINVAL; c->opt_adapt_step = v; }
    else if (!strcmp(key, "block_cache_mib")) { if (v < 0 || v > (int64_t(1) << 24)) return HSS_EINVAL; c->cache.set_cap((size_t)v << 20); }
    else return HSS_EINVAL;
    return HSS_OK;
}

int hss_set_f64(hss_ctx* c, const char* key, double v) {
    if (!c || !key) return HSS_EINVAL;
    if (!strcmp(key, "abs_tol")) { if (!(v >= 0.0)) return HSS_EINVAL; c->opt_abs_tol = v; }
    else return HSS_EINVAL;
    return HSS_OK;
}

int hss_kernel_sample(hss_ctx* ctx, const double* F_dev, int64_t n, int32_t r, double h, const double* Omega_dev,
                      int32_t s, double* S_out_dev) {
    if (!ctx || !F_dev || !Omega_dev || !S_out_dev || n < 1 || r < 1 || s < 1 || !(h > 0.0)) return HSS_EINVAL;
    if (r > MAX_FEATURES) return HSS_EUNSUPPORTED;
    CacheScope cache_scope(&ctx->cache);
    hipStream_t st = ctx->stream;
    const int64_t n_pad = round_up(n, 256);
    const int r_pad = feature_pad(r), s_pad = (int)round_up(s, 128);
    DevBuf Fp, nu, Om, S, mean;
    HSS_TRY(Fp.reserve(sizeof(double) * n_pad * r_pad));
    HSS_TRY(nu.reserve(sizeof(double) * n_pad));
    HSS_TRY(Om.reserve(sizeof(double) * n_pad * s_pad));
    HSS_TRY(S.reserve(sizeof(double) * n_pad * s_pad));
    HSS_TRY(gather_pad_rows_launch(st, F_dev, nullptr, Fp.as<double>(), n, n_pad, r, r_pad));
    HSS_TRY(gather_pad_rows_launch(st, Omega_dev, nullptr, Om.as<double>(), n, n_pad, s, s_pad));
    // the points minus their mean (see vec.h); S itself serves as the work space of the means
    HSS_TRY(mean.reserve(sizeof(double) * r));
    HSS_TRY(column_means_launch(st, Fp.as<double>(), n, r, r_pad, S.as<double>(), mean.as<double>()));
    HSS_TRY(centre_rows_launch(st, Fp.as<double>(), n, r, r_pad, mean.as<double>()));
    HSS_TRY(row_norms_launch(st, Fp.as<double>(), nu.as<double>(), n_pad, r_pad));
    HSS_TRY(kernel_product_launch(st, Fp.as<double>(), nu.as<double>(), n_pad, Fp.as<double>(), nu.as<double>(), n_pad,
                                  Om.as<double>(), S.as<double>(), r_pad, s_pad, s_pad, h));
    HIP_TRY(hipMemcpy2DAsync(S_out_dev, sizeof(double) * s, S.p, sizeof(double) * s_pad, sizeof(double) * s, n,
                             hipMemcpyDeviceToDevice, st));
    HIP_TRY(hipStreamSynchronize(st));   // the temporaries are freed on return
    return HSS_OK;
}

int hss_compress(hss_ctx* ctx, const double* F_dev, const double* y_dev, int64_t n, int32_t r, double h, int32_t leaf,
                 double tol) {
    if (!ctx) return HSS_EINVAL;
    CacheScope cache_scope(&ctx->cache);
    return hss_compress_impl(ctx, F_dev, y_dev, n, r, h, leaf, tol, nullptr, 0);
}

int hss_compress_with_samples(hss_ctx* ctx, const double* F_dev, const double* y_dev, int64_t n, int32_t r, double h,
                              int32_t leaf, double tol, const double* Omega_dev, int32_t s) {
    if (!Omega_dev || !ctx) return HSS_EINVAL;
    CacheScope cache_scope(&ctx->cache);
    return hss_compress_impl(ctx, F_dev, y_dev, n, r, h, leaf, tol, Omega_dev, s);
}

int hss_import(hss_ctx* ctx, const double* F_dev, const double* y_dev, int64_t n, int32_t r, double h, int32_t leaf,
               const int64_t* perm, const int32_t* sizes, const int32_t* ranks, const double* D, const double* U,
               const int32_t* J, const double* B, double delta) {
    if (!ctx) return HSS_EINVAL;
    CacheScope cache_scope(&ctx->cache);
    return hss_import_impl(ctx, F_dev, y_dev, n, r, h, leaf, perm, sizes, ranks, D, U, J, B, delta);
}

int hss_error_estimate(hss_ctx* c, int32_t nprobe, uint64_t seed, double* rel_err_out) {
    if (!c || !rel_err_out || nprobe < 1 || nprobe > 128) return HSS_EINVAL;
    if (!c->compressed) return HSS_ESTATE;
    CacheScope cache_scope(&c->cache);
    hipStream_t st = c->stream;
    const int64_t n = c->n, n_pad = c->n_pad;
    // K Z through the 16-column product when the probes fit, else through a 128-column block of the sampling kernel
    const int sp = nprobe <= 16 ? 16 : 128;
    DevBuf Z, KZ, t, r, work;
    HSS_TRY(Z.reserve(sizeof(double) * n_pad * sp));
    HSS_TRY(KZ.reserve(sizeof(double) * n_pad * sp));
    HSS_TRY(t.reserve(sizeof(double) * n));
    HSS_TRY(r.reserve(sizeof(double) * n));
    HSS_TRY(omega_fill_launch(st, Z.as<double>(), n, n_pad, nprobe, sp, seed));
    if (sp == 16)
        HSS_TRY(sample_narrow_launch(st, c->Fp.as<double>(), c->nu.as<double>(), n_pad, c->Fp.as<double>(), c->nu.as<double>(),
                                     n_pad, Z.as<double>(), KZ.as<double>(), c->r_pad, c->h, work));
    else
        HSS_TRY(kernel_product_launch(st, c->Fp.as<double>(), c->nu.as<double>(), n_pad, c->Fp.as<double>(),
                                      c->nu.as<double>(), n_pad, Z.as<double>(), KZ.as<double>(), c->r_pad, sp, sp, c->h));
    double* part = c->partial.as<double>();
    double* scal = c->scal.as<double>();
    double num = 0.0, den = 0.0;
    for (int j = 0; j < nprobe; ++j) {
        HSS_TRY(vec_column(st, c->mv_x.as<double>(), Z.as<double>(), n, sp, j));
        HSS_TRY(hss_matvec_perm(c));                                    // mv_y = (K~ + delta I) z
        HSS_TRY(vec_column(st, t.as<double>(), KZ.as<double>(), n, sp, j));      // t = K z
        HIP_TRY(hipMemcpyAsync(r.p, c->mv_y.p, sizeof(double) * n, hipMemcpyDeviceToDevice, st));
        if (c->delta != 0.0) HSS_TRY(vec_axpby(st, r.as<double>(), c->mv_x.as<double>(), -c->delta, 1.0, n));
        HSS_TRY(vec_axpby(st, r.as<double>(), t.as<double>(), -1.0, 1.0, n));    // r = K~ z - K z
        HSS_TRY(vec_dot(st, r.as<double>(), r.as<double>(), n, part, scal));
        HSS_TRY(vec_dot(st, t.as<double>(), t.as<double>(), n, part, scal + 1));
        double two[2];
        HIP_TRY(hipMemcpyAsync(two, scal, sizeof(two), hipMemcpyDeviceToHost, st));
        HIP_TRY(hipStreamSynchronize(st));
        num += two[0];
        den += two[1];
    }
    *rel_err_out = den > 0.0 ? std::sqrt(num / den) : 0.0;
    return HSS_OK;
}

int hss_ulv_factor(hss_ctx* ctx, double beta) {
    if (!ctx) return HSS_EINVAL;
    CacheScope cache_scope(&ctx->cache);
    return ulv_factor_impl(ctx, beta);
}

int hss_ulv_solve(hss_ctx* c, double* rhs, int32_t nrhs) {
    if (!c || !rhs || nrhs < 1) return HSS_EINVAL;
    if (!c->compressed || !c->factored) return HSS_ESTATE;
    CacheScope cache_scope(&c->cache);
    hipStream_t st = c->stream;
    const int64_t* perm = c->perm.as<int64_t>();
    // groups of up to MAX_NRHS columns share one pass over the factors
    for (int j0 = 0; j0 < nrhs;) {
        const int g = std::min(nrhs - j0, MAX_NRHS);
        const int nr = g == 1 ? 1 : (g == 2 ? 2 : 4);
        double* cols = rhs + (size_t)j0 * c->n;
        HSS_TRY(vec_gather_cols(st, solve_rhs(c), cols, perm, c->n, nr, g));
        HSS_TRY(ulv_solve_inplace(c, nr));
        HSS_TRY(vec_scatter_cols(st, cols, solve_sol(c, nr), perm, c->n, nr, g));
        j0 += g;
    }
    return HSS_OK;
}

int hss_matvec(hss_ctx* c, const double* x, double* y) {
    if (!c || !x || !y) return HSS_EINVAL;
    if (!c->compressed) return HSS_ESTATE;
    CacheScope cache_scope(&c->cache);
    hipStream_t st = c->stream;
    const int64_t* perm = c->perm.as<int64_t>();
    HSS_TRY(vec_gather(st, c->mv_x.as<double>(), x, perm, c->n));
    HSS_TRY(hss_matvec_perm(c));
    HSS_TRY(vec_scatter(st, y, c->mv_y.as<double>(), perm, c->n));
    return HSS_OK;
}

int admm_svm_train_multi(hss_ctx* c, const double* C_list, int32_t nC, double beta, int32_t maxit, double* x_out,
                         double* z_out, double* mu_out, double* bias_out, int64_t* n_margin_out) {
    if (!c || !C_list || nC < 1 || !(beta > 0.0) || maxit < 0) return HSS_EINVAL;
    for (int j = 0; j < nC; ++j)
        if (!(C_list[j] > 0.0)) return HSS_EINVAL;
    if (!c->compressed) return HSS_ESTATE;
    CacheScope cache_scope(&c->cache);
    int warn = 0;
    if (!c->factored || c->beta != beta) {
        int rc = ulv_factor_impl(c, beta);
        if (rc < 0) return rc;
        warn |= rc;
    }
    hipStream_t st = c->stream;
    const int64_t n = c->n;
    const size_t nb = sizeof(double) * n;
    const int width = nC == 1 ? 1 : (nC == 2 ? 2 : MAX_NRHS);
    HSS_TRY(c->v_x.reserve(nb * width));
    HSS_TRY(c->v_z.reserve(nb * width));
    HSS_TRY(c->v_mu.reserve(nb * width));
    HSS_TRY(c->v_w.reserve(nb));
    HSS_TRY(c->v_e.reserve(nb));
    HSS_TRY(c->v_t.reserve(nb));
    HSS_TRY(c->v_u.reserve(nb));
    HSS_TRY(c->partial.reserve(sizeof(double) * (4 + 2 * MAX_NRHS) * VEC_BLOCKS));
    double* part = c->partial.as<double>();
    double* scal = c->scal.as<double>();
    double* w1 = scal + 4;
    const int64_t* perm = c->perm.as<int64_t>();
    // w = Y K_beta^{-1} e,  w1 = e^T K_beta^{-1} e: the same for every C (Algorithm 3, the lines before the loop)
    HSS_TRY(fill_launch(st, solve_rhs(c), n, 1.0));
    HSS_TRY(ulv_solve_inplace(c, 1));
    HSS_TRY(vec_dot(st, solve_sol(c, 1), nullptr, n, part, w1));
    HSS_TRY(vec_mul(st, c->v_w.as<double>(), c->yp.as<double>(), solve_sol(c, 1), n));
    for (int j0 = 0; j0 < nC;) {
        const int g = std::min(nC - j0, MAX_NRHS);
        const int nr = g == 1 ? 1 : (g == 2 ? 2 : 4);     // three columns run as four, the last one twice
        CBox box;
        for (int j = 0; j < 4; ++j) box.c[j] = C_list[j0 + std::min(j, g - 1)];
        AdmmVecs v{c->v_x.as<double>(), c->v_z.as<double>(), c->v_mu.as<double>(), solve_rhs(c), solve_sol(c, nr),
                   c->yp.as<double>(), c->v_w.as<double>()};
        double* pa = part + 4 * VEC_BLOCKS;
        double* pb = pa + MAX_NRHS * VEC_BLOCKS;
        HSS_TRY(admm_start(st, v, n, nr, pa));
        int it = 0;
        if (c->opt_graph && maxit >= 16) {
            // Two iterations (the partial-sum buffers alternate) recorded once into a HIP graph and replayed: the
            // host then issues one launch per pair of iterations instead of one per tree level and sweep.  The
            // recording runs on a stream of the library's own (a caller's stream may be the null stream, which
            // cannot be captured), ordered after and before the caller's stream by events.
            if (!c->gstream) HIP_TRY(hipStreamCreateWithFlags(&c->gstream, hipStreamNonBlocking));
            if (!c->gevent) HIP_TRY(hipEventCreateWithFlags(&c->gevent, hipEventDisableTiming));
            HIP_TRY(hipEventRecord(c->gevent, st));
            HIP_TRY(hipStreamWaitEvent(c->gstream, c->gevent, 0));
            hipGraph_t graph = nullptr;
            hipGraphExec_t exec = nullptr;
            HIP_TRY(hipStreamBeginCapture(c->gstream, hipStreamCaptureModeRelaxed));
            c->stream = c->gstream;
            int rc = ulv_solve_inplace(c, nr);
            if (rc >= 0) rc = admm_step(c->gstream, v, n, nr, box, beta, w1, pa, pb);
            if (rc >= 0) rc = ulv_solve_inplace(c, nr);
            if (rc >= 0) rc = admm_step(c->gstream, v, n, nr, box, beta, w1, pb, pa);
            c->stream = st;
            hipError_t e = hipStreamEndCapture(c->gstream, &graph);
            if (rc >= 0 && e == hipSuccess) e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
            if (rc >= 0 && e == hipSuccess)
                for (; it + 2 <= maxit && e == hipSuccess; it += 2) e = hipGraphLaunch(exec, c->gstream);
            if (e == hipSuccess) e = hipEventRecord(c->gevent, c->gstream);
            if (e == hipSuccess) e = hipStreamWaitEvent(st, c->gevent, 0);
            // the executable graph is destroyed once its launches have drained
            if (exec) {
                (void)hipStreamSynchronize(c->gstream);
                (void)hipGraphExecDestroy(exec);
            }
            if (graph) (void)hipGraphDestroy(graph);
            if (rc < 0) return rc;
            if (e != hipSuccess) return HSS_EHIP;
        }
        for (; it < maxit; ++it) {
            HSS_TRY(ulv_solve_inplace(c, nr));
            HSS_TRY(admm_step(st, v, n, nr, box, beta, w1, pa, pb));
            std::swap(pa, pb);
        }
        // per column: bias over the margin set with one HSS mat-vec (eq. 7; sign from the margin condition)
        for (int j = 0; j < g; ++j) {
            double* zc = c->v_t.as<double>();
            double* tmp = c->v_u.as<double>();
            double* ebar = c->v_e.as<double>();
            const double C = C_list[j0 + j];
            HSS_TRY(vec_column(st, zc, v.z, n, nr, j));
            HSS_TRY(margin_indicator(st, zc, C, ebar, n));
            HIP_TRY(hipMemcpyAsync(c->mv_x.p, ebar, nb, hipMemcpyDeviceToDevice, st));
            HSS_TRY(hss_matvec_perm(c));
            HSS_TRY(bias_sums(st, zc, c->yp.as<double>(), c->mv_y.as<double>(), ebar, n, part, scal));
            double sums[3];
            HIP_TRY(hipMemcpyAsync(sums, scal, sizeof(sums), hipMemcpyDeviceToHost, st));
            const size_t off = (size_t)(j0 + j) * n;
            if (z_out) HSS_TRY(vec_scatter(st, z_out + off, zc, perm, n));
            if (x_out) {
                HSS_TRY(vec_column(st, tmp, v.x, n, nr, j));
                HSS_TRY(vec_scatter(st, x_out + off, tmp, perm, n));
            }
            if (mu_out) {
                HSS_TRY(vec_column(st, tmp, v.mu, n, nr, j));
                HSS_TRY(vec_scatter(st, mu_out + off, tmp, perm, n));
            }
            HIP_TRY(hipStreamSynchronize(st));
            const int64_t cnt = (int64_t)(sums[2] + 0.5);
            double b = 0.0;
            if (cnt > 0) b = (sums[0] - sums[1]) / (double)cnt;
            else warn |= HSS_WNOMARGIN;
            if (bias_out) bias_out[j0 + j] = b;
            if (n_margin_out) n_margin_out[j0 + j] = cnt;
        }
        j0 += g;
    }
    c->warnings |= warn;
    return warn;
}

int admm_svm_train(hss_ctx* c, double C, double beta, int32_t maxit, double* x_out, double* z_out, double* mu_out,
                   double* bias_out, int64_t* n_margin_out) {
    return admm_svm_train_multi(c, &C, 1, beta, maxit, x_out, z_out, mu_out, bias_out, n_margin_out);
}

int svm_decision(hss_ctx* c, const double* G, int64_t n_test, const double* z, double bias, double* dec) {
    if (!c || !G || !z || !dec || n_test < 0) return HSS_EINVAL;
    if (!c->compressed) return HSS_ESTATE;
    if (n_test == 0) return HSS_OK;
    CacheScope cache_scope(&c->cache);
    hipStream_t st = c->stream;
    // dec = K(G, F) (y .* z) + b is the sampling product with the test points as rows, the training points as
    // columns and one "random" column y .* z: the fused Gram + exp + contraction in its 16-column form, of which
    // the first column is used
    const int sp = 16;
    const int64_t nt_pad = round_up(n_test, 256);
    DevBuf Gp, nug, Om, S, work;
    HSS_TRY(Gp.reserve(sizeof(double) * nt_pad * c->r_pad));
    HSS_TRY(nug.reserve(sizeof(double) * nt_pad));
    HSS_TRY(Om.reserve(sizeof(double) * c->n_pad * sp));
    HSS_TRY(S.reserve(sizeof(double) * nt_pad * sp));
    HSS_TRY(gather_pad_rows_launch(st, G, nullptr, Gp.as<double>(), n_test, nt_pad, c->r, c->r_pad));
    HSS_TRY(centre_rows_launch(st, Gp.as<double>(), n_test, c->r, c->r_pad, c->centre.as<double>()));   // as the training points
    HSS_TRY(row_norms_launch(st, Gp.as<double>(), nug.as<double>(), nt_pad, c->r_pad));
    HSS_TRY(fill_launch(st, Om.as<double>(), c->n_pad * sp, 0.0));
    HSS_TRY(zy_column(st, Om.as<double>(), sp, z, c->yp.as<double>(), c->perm.as<int64_t>(), c->n));
    HSS_TRY(sample_narrow_launch(st, Gp.as<double>(), nug.as<double>(), nt_pad, c->Fp.as<double>(), c->nu.as<double>(),
                                 c->n_pad, Om.as<double>(), S.as<double>(), c->r_pad, c->h, work));
    HSS_TRY(decision_finish(st, dec, S.as<double>(), sp, bias, n_test));
    HIP_TRY(hipStreamSynchronize(st));   // the temporaries are freed on return
    return HSS_OK;
}

int hss_stream_copy(hss_ctx* c, const double* src, double* dst, int64_t n) {
    if (!c || !src || !dst || n < 2 || (n & 1)) return HSS_EINVAL;
    if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15) return HSS_EINVAL;
    return stream_copy_launch(c->stream, src, dst, n);
}

int hss_export_neighbours(hss_ctx* c, int32_t* k_out, int32_t* idx_out, double* dist_out) {
    if (!c || !k_out) return HSS_EINVAL;
    if (!c->compressed || c->ann_k <= 0 || !c->nbr_idx.p) return HSS_ESTATE;
    *k_out = c->ann_k;
    if (!idx_out && !dist_out) return HSS_OK;
    const size_t cnt = (size_t)c->n * c->ann_k;
    if (idx_out) HIP_TRY(hipMemcpyAsync(idx_out, c->nbr_idx.p, sizeof(int32_t) * cnt, hipMemcpyDeviceToHost, c->stream));
    if (dist_out) HIP_TRY(hipMemcpyAsync(dist_out, c->nbr_dist.p, sizeof(double) * cnt, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(hipStreamSynchronize(c->stream));
    return HSS_OK;
}

int hss_stats(hss_ctx* c, hss_stats_t* o) {
    if (!c || !o) return HSS_EINVAL;
    memset(o, 0, sizeof(*o));
    o->n = c->n; o->r = c->r; o->leaf = c->leaf; o->levels = c->L;
    o->sample_width = c->s; o->rank_cap = c->kcap;
    o->sample_width_used = c->width_used; o->nodes_redone = c->nodes_redone;
    if (c->compressed) {
        for (int l = 1; l <= c->L; ++l)
            for (int t = 0; t < c->lev[l].N; ++t) {
                const int k = c->lev[l].rk[t];
                o->rank_max = std::max<int64_t>(o->rank_max, k);
                o->rank_sum += k;
                if (k == c->kcap && k < c->lev[l].msz[t]) o->nodes_at_cap++;
            }
    }
    o->generator_bytes = c->generator_bytes;
    o->factor_bytes = c->factored ? c->factor_bytes : 0;
    o->factor_bytes_compact = c->factored ? c->factor_bytes_compact : 0;
    o->sample_flops = c->sample_flops;
    o->delta = c->delta;
    o->beta = c->factored ? c->beta : -1.0;
    o->t_tree = c->t_tree; o->t_sample = c->t_sample; o->t_levels = c->t_levels; o->t_guard = c->t_guard;
    o->t_factor = c->t_factor;
    o->t_sample_kernel = c->t_sample_kernel;
    o->warnings = c->warnings;
    return HSS_OK;
}

int hss_export_sizes(hss_ctx* c, int64_t* nnodes, int64_t* u_len, int64_t* j_len, int64_t* b_len) {
    if (!c || !nnodes || !u_len || !j_len || !b_len) return HSS_EINVAL;
    if (!c->compressed) return HSS_ESTATE;
    *nnodes = (int64_t(2) << c->L) - 1;
    *u_len = *j_len = *b_len = 0;
    for (int l = 0; l <= c->L; ++l) {
        Level& lv = c->lev[l];
        if (l >= 1) { *u_len += lv.uoff[lv.N]; *j_len += lv.koff[lv.N]; }
        if (l < c->L) *b_len += lv.boff[lv.N];
    }
    return HSS_OK;
}

int hss_export(hss_ctx* c, int64_t* perm, int32_t* sizes, int32_t* ranks, double* D, double* U, int32_t* J, double* B,
               double* delta_out) {
    if (!c || !perm || !sizes || !ranks || !D || !U || !J || !B || !delta_out) return HSS_EINVAL;
    if (!c->compressed) return HSS_ESTATE;
    hipStream_t st = c->stream;
    memcpy(perm, c->perm_host.data(), sizeof(int64_t) * c->n);
    HIP_TRY(hipMemcpyAsync(D, c->Dleaf.p, sizeof(double) * (size_t)c->doff[c->lev[c->L].N], hipMemcpyDeviceToHost, st));
    int64_t node = 0, uo = 0, jo = 0, bo = 0;
    for (int l = 0; l <= c->L; ++l) {      // heap order = level by level, left to right
        Level& lv = c->lev[l];
        for (int t = 0; t < lv.N; ++t, ++node) {
            sizes[node] = lv.msz[t];
            ranks[node] = lv.rk[t];
        }
        if (l >= 1 && lv.uoff[lv.N] > 0) {
            HIP_TRY(hipMemcpyAsync(U + uo, lv.U.p, sizeof(double) * lv.uoff[lv.N], hipMemcpyDeviceToHost, st));
            HIP_TRY(hipMemcpyAsync(J + jo, lv.J.p, sizeof(int32_t) * lv.koff[lv.N], hipMemcpyDeviceToHost, st));
            uo += lv.uoff[lv.N];
            jo += lv.koff[lv.N];
        }
        if (l < c->L && lv.boff[lv.N] > 0) {
            HIP_TRY(hipMemcpyAsync(B + bo, lv.B.p, sizeof(double) * lv.boff[lv.N], hipMemcpyDeviceToHost, st));
            bo += lv.boff[lv.N];
        }
    }
    HIP_TRY(hipStreamSynchronize(st));
    *delta_out = c->delta;
    return HSS_OK;
}

}  // extern "C"
