// HSS compression of the Gaussian kernel matrix (Algorithm 3, first line), level by level up the
// cluster tree, the HSS mat-vec, the definiteness guard and the export of the generators.
//
//   leaf t:    D_t = K(I_t, I_t);  S_t = S(I_t,:) - D_t Omega(I_t,:);  row ID  S_t ~= U_t S_t(J_t,:)
//   inner t:   B_ab = K(skel_a, skel_b);  S_t = [S~_a - B_ab Om~_b; S~_b - B_ab^T Om~_a];  row ID (not at the root)
//   S~_t = S_t(J_t,:),  Om~_t = U_t^T [Om~_a; Om~_b]
// Every step is a batched launch over all nodes of a level; only the ranks come back to the host (one
// small copy per level) to size the next level.
#include "ctx.h"
#include <algorithm>
#include <chrono>
#include <cmath>

namespace {

double wall() {
    return std::chrono::duration<double>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

template <class T>
int upload(hss_ctx* c, DevBuf& buf, const std::vector<T>& v) {
    HSS_TRY(buf.reserve(sizeof(T) * std::max<size_t>(v.size(), 1)));
    if (!v.empty()) HIP_TRY(hipMemcpyAsync(buf.p, v.data(), sizeof(T) * v.size(), hipMemcpyHostToDevice, c->stream));
    return HSS_OK;
}

// smallest eigenvalue of the symmetric tridiagonal matrix (a: diagonal, b: off-diagonal) by bisection on
// the Sturm count
double tridiag_min_eig(const std::vector<double>& a, const std::vector<double>& b) {
    const int m = (int)a.size();
    double lo = a[0], hi = a[0];
    for (int i = 0; i < m; ++i) {
        double rad = (i > 0 ? std::fabs(b[i - 1]) : 0.0) + (i + 1 < m ? std::fabs(b[i]) : 0.0);
        lo = std::min(lo, a[i] - rad);
        hi = std::max(hi, a[i] + rad);
    }
    auto count_below = [&](double x) {   // number of eigenvalues < x
        int cnt = 0;
        double d = 1.0;
        for (int i = 0; i < m; ++i) {
            double off = i > 0 ? b[i - 1] * b[i - 1] : 0.0;
            d = a[i] - x - (i > 0 ? off / d : 0.0);
            if (d == 0.0) d = 1e-300;
            if (d < 0.0) ++cnt;
        }
        return cnt;
    };
    for (int it = 0; it < 200 && hi - lo > 1e-14 * std::max(1.0, std::fabs(lo) + std::fabs(hi)); ++it) {
        double mid = 0.5 * (lo + hi);
        if (count_below(mid) >= 1) hi = mid;
        else lo = mid;
    }
    return 0.5 * (lo + hi);
}

// c->centre = feature means of the points in c->Fp, and Fp minus them (see vec.h)
int centre_features(hss_ctx* c) {
    DevBuf work;
    HSS_TRY(work.reserve(sizeof(double) * centre_work_doubles(c->n, c->r)));
    HSS_TRY(c->centre.reserve(sizeof(double) * c->r));
    HSS_TRY(column_means_launch(c->stream, c->Fp.as<double>(), c->n, c->r, c->r_pad, work.as<double>(), c->centre.as<double>()));
    HSS_TRY(centre_rows_launch(c->stream, c->Fp.as<double>(), c->n, c->r, c->r_pad, c->centre.as<double>()));
    HIP_TRY(hipStreamSynchronize(c->stream));     // the work buffer is released on return
    return HSS_OK;
}

int build_matvec_tables(hss_ctx* c) {
    hipStream_t st = c->stream;
    const int L = c->L;
    HSS_TRY(c->mv_x.reserve(sizeof(double) * c->n));
    HSS_TRY(c->mv_y.reserve(sizeof(double) * c->n));
    double* mvx = c->mv_x.as<double>();
    double* mvy = c->mv_y.as<double>();
    for (int l = 1; l <= L; ++l) {
        Level& lv = c->lev[l];
        HSS_TRY(lv.xt.reserve(sizeof(double) * std::max<int64_t>(lv.koff[lv.N], 1)));
        HSS_TRY(lv.g.reserve(sizeof(double) * std::max<int64_t>(lv.koff[lv.N], 1)));
    }
    // transposed copies of the generators, so that every product of the mat-vec streams matrix rows
    c->arena.reset();
    for (int l = 1; l <= L; ++l) {
        Level& lv = c->lev[l];
        Level& pl = c->lev[l - 1];
        HSS_TRY(lv.UT.reserve(sizeof(double) * std::max<int64_t>(lv.uoff[lv.N], 1)));
        HSS_TRY(pl.BT.reserve(sizeof(double) * std::max<int64_t>(pl.boff[pl.N], 1)));
        std::vector<CopyItem> ci;
        for (int t = 0; t < lv.N; ++t) {
            const int m = lv.msz[t], k = lv.rk[t];
            if (k < m)
                ci.push_back(CopyItem{lv.U.as<double>() + lv.uoff[t], lv.UT.as<double>() + lv.uoff[t], k, m, k, m, COPY_TRANS,
                                      0, 0.0});
        }
        for (int i = 0; i < pl.N; ++i) {
            const int ka = lv.rk[2 * i], kb = lv.rk[2 * i + 1];
            ci.push_back(CopyItem{pl.B.as<double>() + pl.boff[i], pl.BT.as<double>() + pl.boff[i], kb, ka, kb, ka, COPY_TRANS,
                                  0, 0.0});
        }
        HSS_TRY(bcopy(st, c->arena, ci));
    }
    for (int l = L; l >= 1; --l) {
        Level& lv = c->lev[l];
        const double* xin = (l == L) ? mvx : c->lev[l + 1].xt.as<double>();
        std::vector<GemvItem> up(lv.N), dn(lv.N);
        bool even = true;
        for (int t = 0; t < lv.N; ++t) {
            const double* U = lv.U.as<double>() + lv.uoff[t];
            const double* UT = lv.UT.as<double>() + lv.uoff[t];
            const int32_t* J = lv.J.as<int32_t>() + lv.koff[t];
            const int m = lv.msz[t], k = lv.rk[t];
            if ((m | k) & 1) even = false;
            double* xt = lv.xt.as<double>() + lv.koff[t];
            const double* g = lv.g.as<double>() + lv.koff[t];
            // down: (node's rows) = U_t g_t, written where the children's g live (leaf: added to y)
            double* dst = (l == L) ? mvy + lv.moff[t] : c->lev[l + 1].g.as<double>() + lv.moff[t];
            if (k == m) {   // the node kept all its rows: U_t is the permutation with U(J_j, j) = 1
                up[t] = GemvItem{nullptr, xin + lv.moff[t], xt, J, k, m, m, GEMV_GATHER};
                dn[t] = GemvItem{nullptr, g, dst, J, m, k, k, GEMV_SCATTER};
            } else {
                up[t] = GemvItem{UT, xin + lv.moff[t], xt, nullptr, k, m, m, GEMV_DENSE};
                dn[t] = GemvItem{U, g, dst, nullptr, m, k, k, GEMV_DENSE};
            }
        }
        lv.mv_vec = even;
        HSS_TRY(upload(c, lv.mv_up, up));
        HSS_TRY(upload(c, lv.mv_dn_u, dn));
        // coupling through the parent's B: g_a (+)= B xt_b, g_b (+)= B^T xt_a
        Level& pl = c->lev[l - 1];
        std::vector<GemvItem> b1(pl.N), b2(pl.N);
        for (int i = 0; i < pl.N; ++i) {
            const int a = 2 * i, b = 2 * i + 1;
            const double* B = pl.B.as<double>() + pl.boff[i];
            const double* BT = pl.BT.as<double>() + pl.boff[i];
            b1[i] = GemvItem{B, lv.xt.as<double>() + lv.koff[b], lv.g.as<double>() + lv.koff[a], nullptr, lv.rk[a], lv.rk[b],
                             lv.rk[b], GEMV_DENSE};
            b2[i] = GemvItem{BT, lv.xt.as<double>() + lv.koff[a], lv.g.as<double>() + lv.koff[b], nullptr, lv.rk[b], lv.rk[a],
                             lv.rk[a], GEMV_DENSE};
        }
        b1.insert(b1.end(), b2.begin(), b2.end());      // one table: the two products of a pair write different vectors
        HSS_TRY(upload(c, lv.mv_dn_b, b1));
        lv.n_dn_b = 2 * pl.N;
    }
    Level& leafl = c->lev[L];
    std::vector<GemvItem> dd(leafl.N);
    bool leaves_even = true;
    for (int t = 0; t < leafl.N; ++t) {
        const int m = leafl.msz[t];
        if (m & 1) leaves_even = false;
        dd[t] = GemvItem{c->Dleaf.as<double>() + c->doff[t], mvx + leafl.moff[t], mvy + leafl.moff[t], nullptr, m, m, m,
                         GEMV_DENSE};
    }
    c->leaves_even = leaves_even;
    HSS_TRY(upload(c, leafl.mv_leaf_d, dd));
    HIP_TRY(hipStreamSynchronize(st));   // the host vectors above go out of scope
    c->arena.reset();
    return HSS_OK;
}

}  // namespace

// mv_y = (K~ + delta I) mv_x, cluster-tree order (two-pass HSS product).
int hss_matvec_perm(hss_ctx* c) {
    hipStream_t st = c->stream;
    const int L = c->L;
    double* mvx = c->mv_x.as<double>();
    double* mvy = c->mv_y.as<double>();
    for (int l = L; l >= 1; --l) {
        Level& lv = c->lev[l];
        HSS_TRY(bgemv_launch(st, lv.mv_up.as<GemvItem>(), lv.N, lv.maxk, lv.maxm, lv.mv_vec, 1.0, 0.0));
    }
    for (int l = 1; l <= L; ++l) {
        Level& lv = c->lev[l];
        // contribution handed down by the parent level (written by the parent's U g), then the coupling
        const double beta = (l == 1) ? 0.0 : 1.0;
        HSS_TRY(bgemv_launch(st, lv.mv_dn_b.as<GemvItem>(), lv.n_dn_b, lv.maxk, lv.maxk, lv.mv_vec, 1.0, beta));
        if (l < L) HSS_TRY(bgemv_launch(st, lv.mv_dn_u.as<GemvItem>(), lv.N, lv.maxm, lv.maxk, lv.mv_vec, 1.0, 0.0));
    }
    Level& leafl = c->lev[L];
    HSS_TRY(bgemv_launch(st, leafl.mv_leaf_d.as<GemvItem>(), leafl.N, leafl.maxm, leafl.maxm, c->leaves_even, 1.0, 0.0));
    if (L >= 1) HSS_TRY(bgemv_launch(st, leafl.mv_dn_u.as<GemvItem>(), leafl.N, leafl.maxm, leafl.maxk, leafl.mv_vec, 1.0, 1.0));
    if (c->delta != 0.0) HSS_TRY(vec_axpby(st, mvy, mvx, c->delta, 1.0, c->n));
    return HSS_OK;
}

namespace {

// delta = 1.1 * max(0, -lambda_min(K~)) from a Lanczos run on the HSS mat-vec (no re-orthogonalisation:
// only the extreme Ritz value is used).  The run stops when the smallest Ritz value has moved by less than
// 1e-3 (relative) over the last four steps, or after 512 steps.  The number of steps grows with
// lambda_max / |lambda_min|, i.e. with n: 32-37 steps on the workloads up to n = 262144, 89 at n = 1048576,
// about 200 at n = 4194304 (where 64 steps still see a positive Ritz value).
int definiteness_guard(hss_ctx* c) {
    hipStream_t st = c->stream;
    const int64_t n = c->n;
    c->delta = 0.0;
    const int iters = (int)std::min<int64_t>(n, 512);
    // the mat-vec of the run reads FP32 copies of the generators (half the traffic; matvec32.hip); if they do not fit
    // into memory, the FP64 mat-vec.  The copies' pool stays with the context.
    const bool use32 = build_matvec32(c) == HSS_OK;
    if (!use32) release_matvec32(c);
    struct Release32 {      // the item tables live in the upload arena: drained and reset on every way out
        hss_ctx* c;
        ~Release32() {
            (void)hipStreamSynchronize(c->stream);
            c->arena.reset();
            release_matvec32(c);
        }
    } release32{c};
    DevBuf vprev, vcur;
    HSS_TRY(vprev.reserve(sizeof(double) * n));
    HSS_TRY(vcur.reserve(sizeof(double) * n));
    std::vector<double> v0(n);
    uint64_t sd = 0x9E3779B97F4A7C15ull ^ (uint64_t)c->opt_seed;
    double nrm = 0.0;
    for (int64_t i = 0; i < n; ++i) {   // splitmix64 -> uniform(-1, 1)
        sd += 0x9E3779B97F4A7C15ull;
        uint64_t z = sd;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        z ^= z >> 31;
        v0[i] = (double)(z >> 11) * (2.0 / 9007199254740992.0) - 1.0;
        nrm += v0[i] * v0[i];
    }
    nrm = std::sqrt(nrm);
    for (auto& x : v0) x /= nrm;
    HIP_TRY(hipMemcpyAsync(vcur.p, v0.data(), sizeof(double) * n, hipMemcpyHostToDevice, st));
    HIP_TRY(hipMemsetAsync(vprev.p, 0, sizeof(double) * n, st));
    double* part = c->partial.as<double>();
    double* scal = c->scal.as<double>();
    double* w = c->mv_y.as<double>();
    std::vector<double> alpha, beta, ritz;
    double bprev = 0.0;
    for (int j = 0; j < iters; ++j) {
        HIP_TRY(hipMemcpyAsync(c->mv_x.p, vcur.p, sizeof(double) * n, hipMemcpyDeviceToDevice, st));
        HSS_TRY(use32 ? hss_matvec_perm32(c) : hss_matvec_perm(c));
        // alpha = w . v stays on the device for the update; the host sees it together with |w|^2: one wait per step
        HSS_TRY(vec_dot(st, w, vcur.as<double>(), n, part, scal));
        HSS_TRY(vec_lanczos_update(st, w, vcur.as<double>(), vprev.as<double>(), scal, bprev, n));
        HSS_TRY(vec_dot(st, w, w, n, part, scal + 1));
        double ab[2];
        HIP_TRY(hipMemcpyAsync(ab, scal, sizeof(ab), hipMemcpyDeviceToHost, st));
        HIP_TRY(hipStreamSynchronize(st));
        const double a = ab[0], b2 = ab[1];
        alpha.push_back(a);
        const double b = std::sqrt(b2 > 0.0 ? b2 : 0.0);
        if (!(b > 1e-12 * std::max(1.0, std::fabs(a))) || j + 1 == iters) break;
        ritz.push_back(tridiag_min_eig(alpha, beta));
        if (j >= 11 && std::fabs(ritz[j] - ritz[j - 4]) <= 1e-3 * std::fabs(ritz[j])) break;
        beta.push_back(b);
        // vprev <- vcur (the buffers change roles), vcur <- w / b
        std::swap(vprev.p, vcur.p);
        std::swap(vprev.bytes, vcur.bytes);
        HSS_TRY(vec_axpby(st, vcur.as<double>(), w, 1.0 / b, 0.0, n));
        bprev = b;
    }
    beta.resize(alpha.size() > 0 ? alpha.size() - 1 : 0);
    const double lam = tridiag_min_eig(alpha, beta);
    if (lam < 0.0) {
        c->delta = 1.1 * (-lam);
        c->warnings |= HSS_WSHIFT;
    }
    return HSS_OK;
}

}  // namespace

int hss_compress_impl(hss_ctx* c, const double* F, const double* y, int64_t n, int r, double h, int leaf, double tol,
                      const double* Omega, int s_in) {
    if (!c || !F || !y) return HSS_EINVAL;
    if (n < 1 || r < 1 || !(h > 0.0) || !(tol > 0.0) || !(tol <= 10.0)) return HSS_EINVAL;
    if (leaf < 2) return HSS_EINVAL;
    if (r > MAX_FEATURES || leaf > 1024) return HSS_EUNSUPPORTED;
    const int L = tree_depth(n, leaf);                       // any n: leaves of ceil or floor of n / 2^L points
    if (L > 24) return HSS_EUNSUPPORTED;
    const int64_t nl = int64_t(1) << L;
    const std::vector<int64_t> loff = level_offsets(n, L);   // rows of leaf t: loff[t] .. loff[t+1]-1
    const int maxleaf = (int)((n + nl - 1) / nl);
    const int s = Omega ? s_in : (int)c->opt_s;
    if (s < 1) return HSS_EINVAL;
    const int s_pad = (int)round_up(s, 128);
    if (s_pad > 2048) return HSS_EUNSUPPORTED;
    // The Gram form of the interpolative decomposition resolves pivots down to about 1e-7 of the largest one;
    // it is used when the relative stop threshold stays well above that, the Gram-Schmidt form (rows of at most
    // 1024 columns) otherwise.
    const bool gram_id = tol / 10.0 >= 3e-6;
    if (!gram_id && s_pad > 1024) return HSS_EUNSUPPORTED;
    // Adaptive sample width (option "adaptive_start" > 0): the decompositions first see `width` columns; the rank
    // cap at width w is w - p(w), never above the final cap.
    const bool ann = c->opt_sampling == 1 && !Omega;       // neighbour-based sample instead of K Omega
    const bool adaptive = !ann && c->opt_adapt_start > 0 && c->opt_adapt_start < s;
    const int step = (int)c->opt_adapt_step;
    if (adaptive && (s % 128 || c->opt_adapt_start % 128 || step < 128 || step % 128)) return HSS_EINVAL;
    auto cap_at = [&](int64_t w) { return w - (c->opt_p >= 0 ? c->opt_p : w / 2); };
    int64_t kcap = c->opt_max_rank > 0 ? c->opt_max_rank : cap_at(s);
    if (kcap > s) kcap = s;
    if (adaptive && kcap > cap_at(s)) kcap = cap_at(s);      // the final cap is the full sample's at most
    if (kcap < 1) return HSS_EINVAL;
    if (kcap > 512) return HSS_EUNSUPPORTED;
    int width = adaptive ? (int)c->opt_adapt_start : s;
    if (adaptive && cap_at(width) < 1) return HSS_EINVAL;

    hipStream_t st = c->stream;
    c->compressed = c->factored = c->basis_cached = false;
    c->cache.next_epoch();      // the blocks of the previous compression (released just below) stay within reach
    c->lev.clear();
    c->lev.resize(L + 1);
    c->n = n; c->r = r; c->leaf = leaf; c->L = L; c->s = s; c->s_pad = s_pad; c->kcap = (int)kcap;
    c->h = h; c->tol = tol; c->delta = 0.0; c->beta = -1.0; c->warnings = 0;
    c->width_used = width; c->nodes_redone = 0;
    c->ann_k = 0;
    c->r_pad = feature_pad(r);
    c->n_pad = round_up(n, 256);
    const int r_pad = c->r_pad;
    const int64_t n_pad = c->n_pad;
    if (!c->arena.h) HSS_TRY(c->arena.init(size_t(96) << 20));
    c->arena.reset();
    HSS_TRY(c->flags.reserve(sizeof(int) * 4));
    HIP_TRY(hipMemsetAsync(c->flags.p, 0, sizeof(int) * 4, st));
    HSS_TRY(c->partial.reserve(sizeof(double) * (4 + 2 * MAX_NRHS) * VEC_BLOCKS));
    HSS_TRY(c->scal.reserve(sizeof(double) * 16));

    // ---- labels must be +-1 (checked on the host copy); cluster tree on the device ----
    double t0 = wall();
    std::vector<double> yh(n);
    HIP_TRY(hipMemcpyAsync(yh.data(), y, sizeof(double) * n, hipMemcpyDeviceToHost, st));
    HSS_TRY(c->perm.reserve(sizeof(int64_t) * n));
    if (c->opt_cluster == 1)
        HSS_TRY(build_cluster_tree_2means(st, F, n, r, leaf, (int)c->opt_cluster_iters, c->perm.as<int64_t>(),
                                          c->flags.as<int>() + 3));
    else
        HSS_TRY(build_cluster_tree(st, F, n, r, leaf, c->perm.as<int64_t>(), c->flags.as<int>() + 3));
    c->perm_host.resize(n);
    int bad_f = 0;
    HIP_TRY(hipMemcpyAsync(c->perm_host.data(), c->perm.p, sizeof(int64_t) * n, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipMemcpyAsync(&bad_f, c->flags.as<int>() + 3, sizeof(int), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    if (bad_f) return HSS_EINVAL;   // a non-finite feature value
    for (int64_t i = 0; i < n; ++i)
        if (yh[i] != 1.0 && yh[i] != -1.0) return HSS_EINVAL;
    const int64_t* perm = c->perm.as<int64_t>();
    HSS_TRY(c->Fp.reserve(sizeof(double) * n_pad * r_pad));
    HSS_TRY(c->nu.reserve(sizeof(double) * n_pad));
    HSS_TRY(c->yp.reserve(sizeof(double) * n));
    HSS_TRY(gather_pad_rows_launch(st, F, perm, c->Fp.as<double>(), n, n_pad, r, r_pad));
    HSS_TRY(centre_features(c));
    HSS_TRY(row_norms_launch(st, c->Fp.as<double>(), c->nu.as<double>(), n_pad, r_pad));
    HSS_TRY(vec_gather(st, c->yp.as<double>(), y, perm, n));
    HIP_TRY(hipStreamSynchronize(st));
    c->t_tree = wall() - t0;

    // ---- Omega (all s columns) and the first `width` columns of S = K Omega ----
    // Two pairs of n_pad x s_pad buffers: level l works in pair (L - l) & 1.  A column of the rows handed from
    // level to level depends on the same column of S and Omega only, so a column window [c0, c1) that is sampled
    // later travels up through the finished levels on its own, in the same buffers (the wider columns of the
    // pairs are not touched before that; those of pair 0 hold Omega as drawn).
    DevBuf Sb[2], Ob[2], Wk;
    const size_t nsbytes = sizeof(double) * (size_t)n_pad * s_pad;
    const int LD = s_pad;
    HSS_TRY(Sb[0].reserve(nsbytes));
    if (!ann) HSS_TRY(Ob[0].reserve(nsbytes));
    t0 = wall();
    if (ann) {
        HSS_TRY(ann_search(c, F, (int)c->opt_ann_k, (int)c->opt_ann_cell, (int)c->opt_ann_trees, (uint64_t)c->opt_seed));
    } else if (Omega) HSS_TRY(gather_pad_rows_launch(st, Omega, perm, Ob[0].as<double>(), n, n_pad, s, s_pad));
    else HSS_TRY(omega_fill_launch(st, Ob[0].as<double>(), n, n_pad, s, s_pad, (uint64_t)c->opt_seed));
    c->t_sample_kernel = 0.0;
    c->sample_flops = 0.0;
    struct EventPair {      // destroyed on every way out of the function
        hipEvent_t a = nullptr, b = nullptr;
        ~EventPair() {
            if (a) (void)hipEventDestroy(a);
            if (b) (void)hipEventDestroy(b);
        }
    } evp;
    HIP_TRY(hipEventCreate(&evp.a));
    HIP_TRY(hipEventCreate(&evp.b));
    const hipEvent_t ev0 = evp.a, ev1 = evp.b;
    // S[:, c0:c1) = K Omega[:, c0:c1) into pair 0 (the leaf level's), timed with events on the stream
    auto sample_columns = [&](int c0, int c1) -> int {
        const int w = (int)round_up(c1 - c0, 128);
        if (hipEventRecord(ev0, st) != hipSuccess) return HSS_EHIP;
        int src = kernel_product_launch(st, c->Fp.as<double>(), c->nu.as<double>(), n_pad, c->Fp.as<double>(),
                                        c->nu.as<double>(), n_pad, Ob[0].as<double>() + c0, Sb[0].as<double>() + c0, r_pad, w,
                                        LD, h);
        (void)hipEventRecord(ev1, st);
        hipError_t serr = hipStreamSynchronize(st);
        float ms = 0.f;
        if (src >= 0 && serr == hipSuccess) (void)hipEventElapsedTime(&ms, ev0, ev1);
        if (src < 0) return src;
        if (serr != hipSuccess) return HSS_EHIP;
        c->t_sample_kernel += ms * 1e-3;
        c->sample_flops += 2.0 * (double)n * (double)n * (double)((c1 - c0) + r);
        return HSS_OK;
    };
    if (!ann) HSS_TRY(sample_columns(0, width));
    c->t_sample = wall() - t0;

    // ---- leaf level: D_t and S_t = S - D Omega ----
    t0 = wall();
    c->doff.assign(nl + 1, 0);
    for (int64_t t = 0; t < nl; ++t) c->doff[t + 1] = c->doff[t] + (loff[t + 1] - loff[t]) * (loff[t + 1] - loff[t]);
    HSS_TRY(c->Dleaf.reserve(sizeof(double) * (size_t)c->doff[nl]));
    // columns [c0, c1) of the leaf sample rows:  S_t -= D_t Omega_t
    auto leaf_columns = [&](int c0, int c1) -> int {
        Level& lv = c->lev[L];
        std::vector<GemmItem> gm(lv.N);
        const int w = (int)round_up(c1 - c0, 128);
        for (int t = 0; t < lv.N; ++t)
            gm[t] = GemmItem{c->Dleaf.as<double>() + c->doff[t], Ob[0].as<double>() + (size_t)lv.moff[t] * LD + c0,
                             Sb[0].as<double>() + (size_t)lv.moff[t] * LD + c0, lv.msz[t], w, lv.msz[t], lv.msz[t], LD, LD};
        return bgemm_host(st, c->arena, gm, false, false, -1.0, 1.0);
    };
    {
        Level& lv = c->lev[L];
        lv.N = (int)nl;
        lv.msz.resize(lv.N);
        lv.moff = loff;
        for (int t = 0; t < lv.N; ++t) lv.msz[t] = (int)(loff[t + 1] - loff[t]);
        lv.maxm = maxleaf;
        std::vector<KBItem> kb(lv.N);
        for (int t = 0; t < lv.N; ++t)
            kb[t] = KBItem{nullptr, nullptr, loff[t], loff[t], c->Dleaf.as<double>() + c->doff[t], lv.msz[t], lv.msz[t],
                           lv.msz[t], 0};
        HSS_TRY(kernel_blocks(st, c->arena, kb, c->Fp.as<double>(), r_pad, h));
        if (L >= 1 && !ann) HSS_TRY(leaf_columns(0, width));
    }
    if (L >= 1) {
        if (!ann) {
            HSS_TRY(Sb[1].reserve(nsbytes));
            HSS_TRY(Ob[1].reserve(nsbytes));
        }
        if (!gram_id) HSS_TRY(Wk.reserve(nsbytes));
    }
    AnnWork ann_work;
    DevBuf ann_cols;                         // sample columns of the nodes of a level (N x s point indices)
    if (ann && L >= 1) HSS_TRY(ann_cols.reserve(sizeof(int64_t) * (size_t)nl * s));
    const int kc = (int)kcap;
    DevBuf Lc, norms0, norms1, sel, jtmp, rkd, done, r11, Gm, d_goff, d_active;
    if (L >= 1) {
        HSS_TRY(Lc.reserve(sizeof(double) * (size_t)n * kc));
        HSS_TRY(norms0.reserve(sizeof(double) * n));
        HSS_TRY(norms1.reserve(sizeof(double) * n));
        HSS_TRY(sel.reserve(sizeof(int) * n));
        HSS_TRY(jtmp.reserve(sizeof(int) * (size_t)nl * kc));
        HSS_TRY(rkd.reserve(sizeof(int) * nl));
        HSS_TRY(done.reserve(sizeof(int) * nl));
        HSS_TRY(r11.reserve(sizeof(double) * nl));
        HSS_TRY(d_active.reserve(sizeof(int) * nl));
    }
    // Columns [c0, c1) of the rows level l hands to its parent level (l >= 2), from the level's finished
    // decompositions:  S~ = S_t(J,:),  Om~ = U^T Om_t  laid out as the parent's rows, then
    // [S~_a - B Om~_b; S~_b - B^T Om~_a].
    auto push_columns = [&](int l, int c0, int c1) -> int {
        Level& lv = c->lev[l];
        Level& pl = c->lev[l - 1];
        const int N = lv.N;
        const int w = (int)round_up(c1 - c0, 128);
        const int pc = (L - l) & 1, pn = pc ^ 1;
        const double* Acur = Sb[pc].as<double>() + c0;
        const double* Ocur = Ob[pc].as<double>() + c0;
        double* Anext = Sb[pn].as<double>() + c0;
        double* Onext = Ob[pn].as<double>() + c0;
        const int64_t ktot = lv.koff[N];
        HSS_TRY(copy_rows_launch(st, Anext, LD, Acur, LD, lv.rowmap.as<int64_t>(), ktot, w));
        std::vector<GemmItem> g1(N);
        for (int t = 0; t < N; ++t)
            g1[t] = GemmItem{lv.U.as<double>() + lv.uoff[t], Ocur + (size_t)lv.moff[t] * LD, Onext + (size_t)lv.koff[t] * LD,
                             lv.rk[t], w, lv.msz[t], lv.rk[t], LD, LD};
        HSS_TRY(bgemm_host(st, c->arena, g1, true, false, 1.0, 0.0));
        std::vector<GemmItem> g2(pl.N), g3(pl.N);
        for (int i = 0; i < pl.N; ++i) {
            const int a = 2 * i, b = 2 * i + 1;
            const double* B = pl.B.as<double>() + pl.boff[i];
            g2[i] = GemmItem{B, Onext + (size_t)lv.koff[b] * LD, Anext + (size_t)lv.koff[a] * LD, lv.rk[a], w, lv.rk[b],
                             lv.rk[b], LD, LD};
            g3[i] = GemmItem{B, Onext + (size_t)lv.koff[a] * LD, Anext + (size_t)lv.koff[b] * LD, lv.rk[b], w, lv.rk[a],
                             lv.rk[b], LD, LD};
        }
        HSS_TRY(bgemm_host(st, c->arena, g2, false, false, -1.0, 1.0));
        HSS_TRY(bgemm_host(st, c->arena, g3, true, false, -1.0, 1.0));
        return HSS_OK;
    };
    int status = HSS_OK;
    for (int l = L; l >= 1 && status >= 0; --l) {
        Level& lv = c->lev[l];
        const int N = lv.N;
        const int64_t rows = lv.moff[N];
        const int pc = ann ? 0 : (L - l) & 1;
        double* Acur = Sb[pc].as<double>();
        HSS_TRY(upload(c, lv.d_moff, lv.moff));
        if (ann) {
            // the level's sample blocks S_t = K(rows of t, columns of the nearest outside neighbours of those rows)
            std::vector<int32_t> rownode((size_t)rows), ncols;
            for (int t = 0; t < N; ++t)
                for (int64_t q = lv.moff[t]; q < lv.moff[t + 1]; ++q) rownode[(size_t)q] = t;
            const int64_t* rowpoint = l == L ? nullptr : c->lev[l + 1].skel.as<int64_t>();
            HSS_TRY(ann_select_columns(c, ann_work, rowpoint, rownode, rows, N, l, s, ann_cols.as<int64_t>(), ncols));
            HSS_TRY(fill_launch(st, Acur, rows * (int64_t)LD, 0.0));
            std::vector<KBItem> kb(N);
            for (int t = 0; t < N; ++t)
                kb[t] = KBItem{rowpoint ? rowpoint + lv.moff[t] : nullptr, ann_cols.as<int64_t>() + (size_t)t * s, lv.moff[t], 0,
                               Acur + (size_t)lv.moff[t] * LD, lv.msz[t], ncols[t], LD, 0};
            HSS_TRY(kernel_blocks(st, c->arena, kb, c->Fp.as<double>(), r_pad, h));
        }
        // interpolative decompositions of the nodes of the level; with the adaptive width, again for the nodes
        // that the sample's rank cap cut, after widening the sample
        IdLevelArgs ia;
        ia.W = Wk.as<double>(); ia.moff = lv.d_moff.as<int64_t>(); ia.kc = kc;
        ia.rows_per_block = 32; ia.rel = tol / 10.0; ia.abs_tol = c->opt_abs_tol;
        ia.done = done.as<int>(); ia.r11 = r11.as<double>(); ia.jtmp = jtmp.as<int>(); ia.rk = rkd.as<int>();
        ia.Lc = Lc.as<double>(); ia.sel = sel.as<int>();
        ia.active = nullptr;
        std::vector<int> active(N, 1);
        std::vector<int64_t> goff;
        if (gram_id) {
            goff.assign(N + 1, 0);
            for (int t = 0; t < N; ++t) goff[t + 1] = goff[t] + (int64_t)lv.msz[t] * lv.msz[t];
            HSS_TRY(Gm.reserve(sizeof(double) * goff[N]));
            HSS_TRY(upload(c, d_goff, goff));
        }
        lv.rk.assign(N, 0);
        for (bool first = true;; first = false) {
            const int cap = (int)std::min<int64_t>(adaptive ? cap_at(width) : kcap, kcap);
            ia.kcap = cap;
            const int wpad = (int)round_up(width, 128);      // columns width .. wpad are zero
            ia.ld = gram_id ? LD : wpad;
            if (!first) {
                HSS_TRY(upload(c, d_active, active));
                ia.active = d_active.as<int>();
            }
            if (gram_id) {
                // pivoted Cholesky of the nodes' Gram matrices S_t S_t^T over the first `width` columns (one
                // workgroup per node, all steps in one launch)
                std::vector<GemmItem> gg;
                for (int t = 0; t < N; ++t) {
                    if (!active[t]) continue;
                    const double* St = Acur + (size_t)lv.moff[t] * LD;
                    gg.push_back(GemmItem{St, St, Gm.as<double>() + goff[t], lv.msz[t], lv.msz[t], wpad, LD, LD, lv.msz[t]});
                }
                HSS_TRY(bgemm_host(st, c->arena, gg, false, true, 1.0, 0.0));
                HSS_TRY(id_chol(st, ia, N, lv.maxm, Gm.as<double>(), d_goff.as<int64_t>()));
            } else {
                // row-pivoted Gram-Schmidt on a tight work copy of the first `width` columns, one launch per step
                HIP_TRY(hipMemcpy2DAsync(Wk.p, sizeof(double) * wpad, Acur, sizeof(double) * LD, sizeof(double) * wpad,
                                         (size_t)rows, hipMemcpyDeviceToDevice, st));
                HSS_TRY(id_init(st, ia, N, lv.maxm, norms0.as<double>()));
                HSS_TRY(id_steps(st, ia, N, lv.maxm, norms0.as<double>(), norms1.as<double>()));
            }
            HIP_TRY(hipMemcpyAsync(lv.rk.data(), rkd.p, sizeof(int) * N, hipMemcpyDeviceToHost, st));
            HIP_TRY(hipStreamSynchronize(st));
            c->arena.reset();
            int ncut = 0;
            for (int t = 0; t < N; ++t) {
                const int k = lv.rk[t];
                if (k < 1 || k > lv.msz[t]) return HSS_EHIP;   // the kernels guarantee 1 <= k <= size
                active[t] = active[t] && k == cap && k < lv.msz[t];
                ncut += active[t];
            }
            if (!adaptive || ncut == 0 || width >= s || cap >= kcap) break;
            // widen: sample the next columns, take them through the leaf level and the finished levels
            const int c0 = width, c1 = std::min(s, width + step);
            const double tw = wall();
            status = sample_columns(c0, c1);
            if (status < 0) break;
            const double tw1 = wall();
            c->t_sample += tw1 - tw;
            t0 += tw1 - tw;                                   // sampling time is not level time
            status = leaf_columns(c0, c1);
            for (int ll = L; ll > l && status >= 0; --ll) status = push_columns(ll, c0, c1);
            if (status < 0) break;
            width = c1;
            c->nodes_redone += ncut;
        }
        if (status < 0) break;
        lv.koff.assign(N + 1, 0);
        lv.uoff.assign(N + 1, 0);
        lv.maxk = 0;
        for (int t = 0; t < N; ++t) {
            const int k = lv.rk[t];
            lv.koff[t + 1] = lv.koff[t] + k;
            lv.uoff[t + 1] = lv.uoff[t] + (int64_t)k * lv.msz[t];
            lv.maxk = std::max(lv.maxk, k);
            if (active[t]) c->warnings |= HSS_WRANK;          // still cut by a cap
        }
        const int64_t ktot = lv.koff[N];
        HSS_TRY(upload(c, lv.d_koff, lv.koff));
        HSS_TRY(upload(c, lv.d_uoff, lv.uoff));
        HSS_TRY(lv.U.reserve(sizeof(double) * lv.uoff[N]));
        HSS_TRY(lv.J.reserve(sizeof(int) * ktot));
        HSS_TRY(lv.skel.reserve(sizeof(int64_t) * ktot));
        HSS_TRY(lv.rowmap.reserve(sizeof(int64_t) * ktot));
        ia.active = nullptr;
        HSS_TRY(id_finish(st, ia, N, lv.maxm, lv.d_koff.as<int64_t>(), lv.d_uoff.as<int64_t>(), lv.U.as<double>(),
                          lv.J.as<int>()));
        HSS_TRY(rowmap_launch(st, lv.d_moff.as<int64_t>(), lv.d_koff.as<int64_t>(), jtmp.as<int>(), kc, N,
                              lv.rowmap.as<int64_t>()));
        HSS_TRY(gather_index_launch(st, lv.skel.as<int64_t>(), l == L ? nullptr : c->lev[l + 1].skel.as<int64_t>(),
                                    lv.rowmap.as<int64_t>(), ktot));
        // parent level
        Level& pl = c->lev[l - 1];
        pl.N = N / 2;
        pl.msz.resize(pl.N);
        pl.moff.assign(pl.N + 1, 0);
        pl.boff.assign(pl.N + 1, 0);
        pl.maxm = 0;
        for (int i = 0; i < pl.N; ++i) {
            pl.msz[i] = lv.rk[2 * i] + lv.rk[2 * i + 1];
            pl.moff[i + 1] = pl.moff[i] + pl.msz[i];
            pl.boff[i + 1] = pl.boff[i] + (int64_t)lv.rk[2 * i] * lv.rk[2 * i + 1];
            pl.maxm = std::max(pl.maxm, pl.msz[i]);
        }
        HSS_TRY(pl.B.reserve(sizeof(double) * pl.boff[pl.N]));
        std::vector<KBItem> kb(pl.N);
        for (int i = 0; i < pl.N; ++i) {
            const int a = 2 * i, b = 2 * i + 1;
            kb[i] = KBItem{lv.skel.as<int64_t>() + lv.koff[a], lv.skel.as<int64_t>() + lv.koff[b], 0, 0,
                           pl.B.as<double>() + pl.boff[i], lv.rk[a], lv.rk[b], lv.rk[b], 0};
        }
        HSS_TRY(kernel_blocks(st, c->arena, kb, c->Fp.as<double>(), r_pad, h));
        if (l - 1 >= 1 && !ann) HSS_TRY(push_columns(l, 0, width));
    }
    if (status < 0) return status;
    c->width_used = width;
    // root bookkeeping
    {
        Level& rl = c->lev[0];
        if (L == 0) {
            rl.N = 1;
            rl.msz.assign(1, (int)n);
            rl.moff = {0, n};
            rl.maxm = (int)n;
        }
        rl.rk.assign(1, 0);
        rl.koff = {0, 0};
        rl.uoff = {0, 0};
        rl.maxk = 0;
    }
    HIP_TRY(hipStreamSynchronize(st));
    c->arena.reset();
    c->t_levels = wall() - t0;

    c->generator_bytes = (int64_t)sizeof(double) * c->doff[nl];
    for (int l = 0; l <= L; ++l) {
        Level& lv = c->lev[l];
        if (l >= 1) c->generator_bytes += (int64_t)sizeof(double) * lv.uoff[lv.N];
        if (l < L) c->generator_bytes += (int64_t)sizeof(double) * lv.boff[lv.N];
    }
    HSS_TRY(build_matvec_tables(c));
    c->compressed = true;
    t0 = wall();
    if (c->opt_guard && L >= 1) HSS_TRY(definiteness_guard(c));
    HIP_TRY(hipStreamSynchronize(st));
    c->t_guard = wall() - t0;
    return c->warnings;
}

// Rebuilds a compressed context from generators in host memory (the arrays hss_export writes, or those of
// any other construction of the same HSS form): no sampling, no interpolative decompositions, no guard --
// the caller's delta is taken as given.
int hss_import_impl(hss_ctx* c, const double* F, const double* y, int64_t n, int r, double h, int leaf,
                    const int64_t* perm_h, const int32_t* sizes, const int32_t* ranks, const double* D, const double* U,
                    const int32_t* J, const double* B, double delta) {
    if (!c || !F || !y || !perm_h || !sizes || !ranks || !D || !U || !J || !B) return HSS_EINVAL;
    if (n < 1 || r < 1 || !(h > 0.0) || !(delta >= 0.0) || !(delta <= 1.7976931348623157e308)) return HSS_EINVAL;
    if (leaf < 2) return HSS_EINVAL;
    if (r > MAX_FEATURES || leaf > 1024) return HSS_EUNSUPPORTED;
    const int L = tree_depth(n, leaf);
    if (L > 24) return HSS_EUNSUPPORTED;
    const int64_t nl = int64_t(1) << L;
    const std::vector<int64_t> loff = level_offsets(n, L);   // rows of leaf t: loff[t] .. loff[t+1]-1
    // ---- host-side validation of the tree arrays ----
    {
        std::vector<char> seen(n, 0);
        for (int64_t i = 0; i < n; ++i) {
            if (perm_h[i] < 0 || perm_h[i] >= n || seen[perm_h[i]]) return HSS_EINVAL;
            seen[perm_h[i]] = 1;
        }
    }
    int kmax = 0;
    {
        int64_t jo = 0, uo = 0;
        std::vector<char> mark;
        for (int l = 0; l <= L; ++l)
            for (int64_t t = 0; t < (int64_t(1) << l); ++t) {
                const int64_t node = (int64_t(1) << l) - 1 + t;
                const int m = sizes[node], k = ranks[node];
                if (l == L ? m != loff[t + 1] - loff[t] : m != ranks[2 * node + 1] + ranks[2 * node + 2]) return HSS_EINVAL;
                if (l == 0) {
                    if (k != 0) return HSS_EINVAL;
                    continue;
                }
                if (k < 1 || k > m) return HSS_EINVAL;
                if (k > 512 || m > 1024) return HSS_EUNSUPPORTED;
                kmax = std::max(kmax, k);
                mark.assign(m, 0);
                for (int j = 0; j < k; ++j) {      // skeleton rows: distinct, inside the node
                    const int v = J[jo + j];
                    if (v < 0 || v >= m || mark[v]) return HSS_EINVAL;
                    mark[v] = 1;
                    // interpolative basis: row J_j of U is the j-th unit vector (the factorization relies on it)
                    const double* urow = U + uo + (int64_t)v * k;
                    for (int q = 0; q < k; ++q)
                        if (urow[q] != (q == j ? 1.0 : 0.0)) return HSS_EINVAL;
                }
                jo += k;
                uo += (int64_t)m * k;
            }
    }
    hipStream_t st = c->stream;
    c->compressed = c->factored = c->basis_cached = false;
    c->cache.next_epoch();
    c->lev.clear();
    c->lev.resize(L + 1);
    c->n = n; c->r = r; c->leaf = leaf; c->L = L; c->s = 0; c->s_pad = 0; c->kcap = std::max(kmax, 1);
    c->h = h; c->tol = 0.0; c->delta = delta; c->beta = -1.0; c->warnings = delta > 0.0 ? HSS_WSHIFT : 0;
    c->r_pad = feature_pad(r);
    c->n_pad = round_up(n, 256);
    c->t_tree = c->t_sample = c->t_levels = c->t_guard = c->t_sample_kernel = 0.0;
    c->sample_flops = 0.0;
    if (!c->arena.h) HSS_TRY(c->arena.init(size_t(96) << 20));
    c->arena.reset();
    HSS_TRY(c->flags.reserve(sizeof(int) * 4));
    HIP_TRY(hipMemsetAsync(c->flags.p, 0, sizeof(int) * 4, st));
    HSS_TRY(c->partial.reserve(sizeof(double) * (4 + 2 * MAX_NRHS) * VEC_BLOCKS));
    HSS_TRY(c->scal.reserve(sizeof(double) * 16));
    std::vector<double> yh(n);
    HIP_TRY(hipMemcpyAsync(yh.data(), y, sizeof(double) * n, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    for (int64_t i = 0; i < n; ++i)
        if (yh[i] != 1.0 && yh[i] != -1.0) return HSS_EINVAL;
    c->perm_host.assign(perm_h, perm_h + n);
    HSS_TRY(c->perm.reserve(sizeof(int64_t) * n));
    HIP_TRY(hipMemcpyAsync(c->perm.p, perm_h, sizeof(int64_t) * n, hipMemcpyHostToDevice, st));
    const int64_t* perm = c->perm.as<int64_t>();
    HSS_TRY(c->Fp.reserve(sizeof(double) * c->n_pad * c->r_pad));
    HSS_TRY(c->nu.reserve(sizeof(double) * c->n_pad));
    HSS_TRY(c->yp.reserve(sizeof(double) * n));
    HSS_TRY(gather_pad_rows_launch(st, F, perm, c->Fp.as<double>(), n, c->n_pad, r, c->r_pad));
    HSS_TRY(centre_features(c));
    HSS_TRY(row_norms_launch(st, c->Fp.as<double>(), c->nu.as<double>(), c->n_pad, c->r_pad));
    HSS_TRY(vec_gather(st, c->yp.as<double>(), y, perm, n));
    c->doff.assign(nl + 1, 0);
    for (int64_t t = 0; t < nl; ++t) c->doff[t + 1] = c->doff[t] + (loff[t + 1] - loff[t]) * (loff[t + 1] - loff[t]);
    HSS_TRY(c->Dleaf.reserve(sizeof(double) * (size_t)c->doff[nl]));
    HIP_TRY(hipMemcpyAsync(c->Dleaf.p, D, sizeof(double) * (size_t)c->doff[nl], hipMemcpyHostToDevice, st));
    // ---- levels: sizes, offsets, generators; skeleton points rebuilt from the skeleton rows ----
    int64_t uo = 0, jo = 0, bo = 0;
    std::vector<std::vector<int64_t>> skel(L + 1);
    for (int l = 0; l <= L; ++l) {
        Level& lv = c->lev[l];
        lv.N = 1 << l;
        const int64_t first = (int64_t(1) << l) - 1;
        lv.msz.assign(sizes + first, sizes + first + lv.N);
        lv.rk.assign(ranks + first, ranks + first + lv.N);
        lv.moff.assign(lv.N + 1, 0);
        lv.koff.assign(lv.N + 1, 0);
        lv.uoff.assign(lv.N + 1, 0);
        lv.maxm = lv.maxk = 0;
        for (int t = 0; t < lv.N; ++t) {
            lv.moff[t + 1] = lv.moff[t] + lv.msz[t];
            lv.koff[t + 1] = lv.koff[t] + lv.rk[t];
            lv.uoff[t + 1] = lv.uoff[t] + (int64_t)lv.msz[t] * lv.rk[t];
            lv.maxm = std::max(lv.maxm, lv.msz[t]);
            lv.maxk = std::max(lv.maxk, lv.rk[t]);
        }
        if (l >= 1) {
            HSS_TRY(upload(c, lv.d_moff, lv.moff));
            HSS_TRY(upload(c, lv.d_koff, lv.koff));
            HSS_TRY(upload(c, lv.d_uoff, lv.uoff));
            HSS_TRY(lv.U.reserve(sizeof(double) * std::max<int64_t>(lv.uoff[lv.N], 1)));
            HSS_TRY(lv.J.reserve(sizeof(int) * std::max<int64_t>(lv.koff[lv.N], 1)));
            HIP_TRY(hipMemcpyAsync(lv.U.p, U + uo, sizeof(double) * lv.uoff[lv.N], hipMemcpyHostToDevice, st));
            HIP_TRY(hipMemcpyAsync(lv.J.p, J + jo, sizeof(int) * lv.koff[lv.N], hipMemcpyHostToDevice, st));
            uo += lv.uoff[lv.N];
            jo += lv.koff[lv.N];
        }
        if (l < L) {
            lv.boff.assign(lv.N + 1, 0);
            for (int t = 0; t < lv.N; ++t) {
                const int64_t node = first + t;
                lv.boff[t + 1] = lv.boff[t] + (int64_t)ranks[2 * node + 1] * ranks[2 * node + 2];
            }
            HSS_TRY(lv.B.reserve(sizeof(double) * std::max<int64_t>(lv.boff[lv.N], 1)));
            HIP_TRY(hipMemcpyAsync(lv.B.p, B + bo, sizeof(double) * lv.boff[lv.N], hipMemcpyHostToDevice, st));
            bo += lv.boff[lv.N];
        }
    }
    {
        int64_t jbase = 0;
        std::vector<int64_t> joff(L + 2, 0);   // start of each level's block in J (heap order = level order)
        for (int l = 1; l <= L; ++l) {
            joff[l] = jbase;
            jbase += c->lev[l].koff[c->lev[l].N];
        }
        for (int l = L; l >= 1; --l) {
            Level& lv = c->lev[l];
            skel[l].resize(lv.koff[lv.N]);
            for (int t = 0; t < lv.N; ++t)
                for (int j = 0; j < lv.rk[t]; ++j) {
                    const int row = J[joff[l] + lv.koff[t] + j];
                    // rows of an inner node = the children's skeleton points, left child first
                    skel[l][lv.koff[t] + j] = l == L ? lv.moff[t] + row : skel[l + 1][c->lev[l + 1].koff[2 * t] + row];
                }
            HSS_TRY(lv.skel.reserve(sizeof(int64_t) * std::max<int64_t>(lv.koff[lv.N], 1)));
            HIP_TRY(hipMemcpyAsync(lv.skel.p, skel[l].data(), sizeof(int64_t) * skel[l].size(), hipMemcpyHostToDevice, st));
        }
    }
    c->generator_bytes = (int64_t)sizeof(double) * c->doff[nl];
    for (int l = 0; l <= L; ++l) {
        Level& lv = c->lev[l];
        if (l >= 1) c->generator_bytes += (int64_t)sizeof(double) * lv.uoff[lv.N];
        if (l < L) c->generator_bytes += (int64_t)sizeof(double) * lv.boff[lv.N];
    }
    HIP_TRY(hipStreamSynchronize(st));     // host staging (skel, the caller's arrays) may go away after return
    HSS_TRY(build_matvec_tables(c));
    c->compressed = true;
    return c->warnings;
}
