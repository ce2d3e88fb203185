// ULV factorization of A = K~ + (delta + beta) I and the forward/backward solve (Algorithm 3:
// "ULVfactorization" and the application of (ULV)^{-1}; Sec. 3.1, last bullet).
//
// Per node t with diagonal block D (m x m) and basis Uf (m x k) = blkdiag(R_a, R_b) U_t:
//   Q = [Q1 Q2] orthogonal with Q1 spanning range(Uf):  Q1^T = L1^{-1} Uf^T,  L1 L1^T = Uf^T Uf,
//                       Q2^T = L2^{-1} P^T,  P = blkdiag(R_a, R_b)^{-T} U_t^perp,  L2 L2^T = P^T P,
//     where U_t^perp is the explicit complement of the interpolative basis U_t = Pi [I; T];
//   Dh = Q^T D Q = [[Drr, Dre], [Der, Dee]];  the last m-k rows couple to nothing outside the node and are
//   eliminated through a partially pivoted LU of Dee;  Dt = Drr - Dre Dee^{-1} Der and R = Q1^T Uf = L1^T
//   go to the parent, whose diagonal block is [[Dt_a, R_a B R_b^T], [sym, Dt_b]].
// The solve uses the explicit operators
//   Mup   = [[I, -Dre Dee^{-1}], [0, Dee^{-1}]] Q^T         (up-sweep:  [b_r'; c_e] = Mup b)
//   Mdown = Q [[I, 0], [-Dee^{-1} Der, I]]                 (down-sweep: x = Mdown [x_r; c_e])
// so that both sweeps are plain matrix-vector products streaming the factors from HBM.
// Nodes whose rank equals their size eliminate nothing: they hand D and Uf to the parent unchanged and
// store no operator.  All steps are batched over the nodes of a level (in chunks that bound the
// temporary memory).
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

CopyItem cp(const double* src, double* dst, int rows, int cols, int lds, int ldd, int mode, double diag = 0.0) {
    return CopyItem{src, dst, rows, cols, lds, ldd, mode, 0, diag};
}
GemmItem gi(const double* A, const double* B, double* C, int M, int N, int K, int lda, int ldb, int ldc) {
    return GemmItem{A, B, C, M, N, K, lda, ldb, ldc};
}

// In-place inverse of the (single) root block: LU with partial pivoting, then U^{-1} L^{-1} P.
int invert_root(hss_ctx* c, double* D, int m, double tiny) {
    hipStream_t st = c->stream;
    DevBuf piv;
    HSS_TRY(piv.reserve(sizeof(int) * m));
    HSS_TRY(c->rootinv.reserve(sizeof(double) * (size_t)m * m));
    std::vector<LUItem> lu{LUItem{D, piv.as<int>(), m, m}};
    HSS_TRY(bgetrf(st, c->arena, lu, true, tiny, c->flags.as<int>()));
    HSS_TRY(bgetri(st, c->arena, lu, {c->rootinv.as<double>()}, {m}));
    HIP_TRY(hipStreamSynchronize(st));
    c->arena.reset();
    c->root_m = m;
    return HSS_OK;
}

// four right-hand sides: 4 rows per wavefront measured best (188 us on the widest level of the n = 262144
// workload against 212 us with 2 rows and 275 us with 1)
constexpr int WIDE_ROWS_PER_WAVE = 4;

int build_solve_tables(hss_ctx* c) {
    const int L = c->L;
    // every level vector is a slice of one pool (even offsets, the leaf input first)
    {
        int64_t total = 0;
        auto take = [&](int64_t len) {
            const int64_t o = total;
            total += round_up(std::max<int64_t>(len, 2), 2);
            return o;
        };
        std::vector<int64_t> ob(L + 1), ox(L + 1), oc(L + 1);
        for (int l = L; l >= 0; --l) {
            Level& lv = c->lev[l];
            const int64_t rows = lv.moff[lv.N];
            ob[l] = take(rows);
            ox[l] = take(rows);
            oc[l] = take(rows - lv.koff[lv.N]);
        }
        HSS_TRY(c->vpool.reserve(sizeof(double) * (size_t)total * MAX_NRHS));
        double* pool = c->vpool.as<double>();
        for (int l = 0; l <= L; ++l) {
            c->lev[l].bvec = pool + ob[l];
            c->lev[l].xvec = pool + ox[l];
            c->lev[l].ce = pool + oc[l];
        }
    }
    // When no leaf eliminates anything (rank == leaf size everywhere) the leaves' vectors ARE the vectors of
    // the level above (same layout), so that level works on them in place and the leaf level launches nothing.
    bool leaves_pass = L >= 1;
    for (int t = 0; leaves_pass && t < c->lev[L].N; ++t) leaves_pass = c->lev[L].pass[t] != 0;
    for (int l = 0; l <= L; ++l) c->lev[l].skip = false;
    if (leaves_pass) c->lev[L].skip = true;
    for (int l = L; l >= 0; --l) {
        Level& lv = c->lev[l];
        std::vector<SolveItem> up(lv.N), dn(lv.N);
        double* my_bvec = (leaves_pass && l == L - 1) ? c->lev[L].bvec : lv.bvec;
        double* my_xvec = (leaves_pass && l == L - 1) ? c->lev[L].xvec : lv.xvec;
        std::vector<int2> work, work_wide;
        // launch shape: enough workgroups to fill the chip (4 x rows_per_wave rows each); 16-byte loads when
        // every size and offset of the level is even
        int64_t rows_total = 0;
        bool even = true;
        for (int t = 0; t < lv.N; ++t) {
            rows_total += lv.msz[t];
            if ((lv.msz[t] | lv.rk[t]) & 1) even = false;
        }
        // measured on the widest level of the n = 262144 workload (1.07 GB per sweep): 2 rows per wavefront
        // 157 us, 4 rows 163 us, 8 rows 177 us -- many short-lived workgroups beat few long ones here
        // rows of at most 128 columns are one 16-byte load per lane: 4 of them per wavefront keep more bytes in flight
        int rpw = lv.maxm <= 128 ? 4 : 2;
        while (rpw > 1 && rows_total / (4 * rpw) < 4096) rpw >>= 1;
        lv.rows_per_wave = rpw;
        lv.vec = even;
        const int rb = 4 * rpw;
        for (int t = 0; t < lv.N; ++t) {
            const int m = lv.msz[t], k = lv.rk[t];
            if (l == 0) {
                up[t] = SolveItem{c->rootinv.as<double>(), my_bvec, nullptr, my_xvec, nullptr, m, m, m, m};
                dn[t] = up[t];
            } else {
                Level& pl = c->lev[l - 1];
                const double* Mu = lv.pass[t] ? nullptr : lv.Mup.as<double>() + lv.foff[t];
                const double* Md = lv.pass[t] ? nullptr : lv.Mdown.as<double>() + lv.foff[t];
                double* ce = lv.ce + (lv.moff[t] - lv.koff[t]);
                up[t] = SolveItem{Mu, my_bvec + lv.moff[t], nullptr, pl.bvec + lv.koff[t], ce, m, m, m, k};
                dn[t] = SolveItem{Md, pl.xvec + lv.koff[t], ce, my_xvec + lv.moff[t], nullptr, m, m, k, m};
            }
            for (int r0 = 0; r0 < m; r0 += rb) work.push_back(make_int2(t, r0));
            for (int r0 = 0; r0 < m; r0 += 4 * WIDE_ROWS_PER_WAVE) work_wide.push_back(make_int2(t, r0));
        }
        if (l == c->top_l) {
            c->top_in = my_bvec;
            c->top_out = my_xvec;
        }
        lv.nwork = (int)work.size();
        lv.nwork_wide = (int)work_wide.size();
        HSS_TRY(upload(c, lv.work_wide, work_wide));
        HSS_TRY(upload(c, lv.up_items, up));
        HSS_TRY(upload(c, lv.down_items, dn));
        HSS_TRY(upload(c, lv.work, work));
        HIP_TRY(hipStreamSynchronize(c->stream));
    }
    return HSS_OK;
}

// The cut level of the merged top.  One solve launches a kernel per level and sweep, each a dependent step of a
// few microseconds however little it reads; near the root the levels are small, so the levels 0 .. tl are better
// served by ONE product with the inverse of the reduced matrix at level tl (M x M, M = rows of level tl) although
// that matrix may hold more entries than the factors it replaces.  Model: a launch costs 3.5 us plus its bytes at
// 6.5 TB/s; tl minimises the modelled time of a solve.  M must be even and at most 4096.
int choose_top_level(hss_ctx* c) {
    const int L = c->L;
    const double t_launch = 3.5e-6, bw = 6.5e12;
    bool leaves_pass = L >= 1;
    for (int t = 0; leaves_pass && t < c->lev[L].N; ++t) leaves_pass = c->lev[L].pass[t] != 0;
    std::vector<double> t_level(L + 1, 0.0);      // one sweep of level l (l >= 1)
    for (int l = 1; l <= L; ++l) {
        if (l == L && leaves_pass) continue;
        t_level[l] = t_launch + 8.0 * (double)c->lev[l].foff[c->lev[l].N] / bw;
    }
    int best = 0;
    double best_t = 1e300;
    for (int tl = 0; tl <= L; ++tl) {
        const int64_t M = c->lev[tl].moff[c->lev[tl].N];
        if (tl > 0 && (M > 4096 || (M & 1))) continue;
        double t = t_launch + 8.0 * (double)M * (double)M / bw;
        for (int l = tl + 1; l <= L; ++l) t += 2.0 * t_level[l];
        if (t < best_t) { best_t = t; best = tl; }
    }
    return best;
}

// topT = inverse of the reduced matrix at level tl: the sweeps of the levels tl .. 0 .. tl applied to the identity,
// level by level as batched matrix products with the operators of the factorization.
int build_top_operator(hss_ctx* c, int tl) {
    hipStream_t st = c->stream;
    c->top_l = tl;
    c->top_m = (int)c->lev[tl].moff[c->lev[tl].N];
    if (tl == 0) return HSS_OK;                    // the root inverse itself, applied as a level
    const int M = c->top_m;
    const size_t dsz = sizeof(double);
    std::vector<DevBuf> Bm(tl + 1), Xm(tl + 1), Ce(tl + 1);
    for (int l = 0; l <= tl; ++l) {
        Level& lv = c->lev[l];
        const int64_t rows = lv.moff[lv.N], ke = rows - lv.koff[lv.N];
        HSS_TRY(Bm[l].reserve(dsz * rows * M));
        if (l < tl) HSS_TRY(Xm[l].reserve(dsz * rows * M));
        HSS_TRY(Ce[l].reserve(dsz * std::max<int64_t>(ke, 1) * M));
    }
    HSS_TRY(c->topT.reserve(dsz * (size_t)M * M));
    c->arena.reset();
    HSS_TRY(bcopy(st, c->arena, {cp(nullptr, Bm[tl].as<double>(), M, M, M, M, COPY_IDENTITY)}));
    for (int l = tl; l >= 1; --l) {                // up-sweep: [b_r'; c_e] = Mup b per node
        Level& lv = c->lev[l];
        std::vector<GemmItem> g;
        std::vector<CopyItem> ci;
        for (int t = 0; t < lv.N; ++t) {
            const int m = lv.msz[t], k = lv.rk[t];
            const double* b = Bm[l].as<double>() + (size_t)lv.moff[t] * M;
            double* up = Bm[l - 1].as<double>() + (size_t)lv.koff[t] * M;
            if (lv.pass[t]) {
                ci.push_back(cp(b, up, m, M, M, M, COPY_PLAIN));
                continue;
            }
            const double* Mu = lv.Mup.as<double>() + lv.foff[t];
            g.push_back(gi(Mu, b, up, k, M, m, m, M, M));
            g.push_back(gi(Mu + (size_t)k * m, b, Ce[l].as<double>() + (size_t)(lv.moff[t] - lv.koff[t]) * M, m - k, M, m, m, M, M));
        }
        HSS_TRY(bcopy(st, c->arena, ci));
        HSS_TRY(bgemm_host(st, c->arena, g, false, false, 1.0, 0.0));
    }
    {
        const int m = c->root_m;
        double* x0 = tl == 0 ? c->topT.as<double>() : Xm[0].as<double>();
        HSS_TRY(bgemm_host(st, c->arena, {gi(c->rootinv.as<double>(), Bm[0].as<double>(), x0, m, M, m, m, M, M)}, false, false,
                           1.0, 0.0));
    }
    for (int l = 1; l <= tl; ++l) {                // down-sweep: x = Mdown [x_r; c_e] per node
        Level& lv = c->lev[l];
        double* xout = l == tl ? c->topT.as<double>() : Xm[l].as<double>();
        std::vector<GemmItem> g1, g2;
        std::vector<CopyItem> ci;
        for (int t = 0; t < lv.N; ++t) {
            const int m = lv.msz[t], k = lv.rk[t];
            const double* xr = Xm[l - 1].as<double>() + (size_t)lv.koff[t] * M;
            double* x = xout + (size_t)lv.moff[t] * M;
            if (lv.pass[t]) {
                ci.push_back(cp(xr, x, m, M, M, M, COPY_PLAIN));
                continue;
            }
            const double* Md = lv.Mdown.as<double>() + lv.foff[t];
            g1.push_back(gi(Md, xr, x, m, M, k, m, M, M));
            g2.push_back(gi(Md + k, Ce[l].as<double>() + (size_t)(lv.moff[t] - lv.koff[t]) * M, x, m, M, m - k, m, M, M));
        }
        HSS_TRY(bcopy(st, c->arena, ci));
        HSS_TRY(bgemm_host(st, c->arena, g1, false, false, 1.0, 0.0));
        HSS_TRY(bgemm_host(st, c->arena, g2, false, false, 1.0, 1.0));
    }
    HIP_TRY(hipStreamSynchronize(st));             // the temporaries go out of scope
    c->arena.reset();
    return HSS_OK;
}

}  // namespace

int ulv_factor_impl(hss_ctx* c, double beta) {
    if (!c) return HSS_EINVAL;
    if (!c->compressed) return HSS_ESTATE;
    if (!(beta > 0.0)) return HSS_EINVAL;
    hipStream_t st = c->stream;
    const int L = c->L;
    const double shift = c->delta + beta;
    const double tiny = 1e-12 * std::max(1.0, shift);
    c->factored = false;
    const double t_start = wall();
    HIP_TRY(hipMemsetAsync(c->flags.p, 0, sizeof(int) * 4, st));
    c->arena.reset();

    DevBuf Dbuf[2];
    int cur = 0;
    // leaf blocks D + shift I
    {
        Level& lv = c->lev[L];
        HSS_TRY(Dbuf[cur].reserve(sizeof(double) * (size_t)c->doff[lv.N]));
        std::vector<CopyItem> ci(lv.N);
        for (int t = 0; t < lv.N; ++t)
            ci[t] = cp(c->Dleaf.as<double>() + c->doff[t], Dbuf[cur].as<double>() + c->doff[t], lv.msz[t], lv.msz[t],
                       lv.msz[t], lv.msz[t], COPY_PLAIN_ADD_DIAG, shift);
        HSS_TRY(bcopy(st, c->arena, ci));
    }
    int64_t bytes_solve = 0, bytes_compact = 0;

    // temporaries of one chunk of nodes
    DevBuf UT, PT0, PT, G2, L2i, QT, Tmp, Dh, E, Einv, W, Wp, ipiv, cholsc, T1;
    // doubles of m*m per chunk (about a dozen temporaries of that size live at once): larger chunks mean fewer, fuller
    // launches -- the widest level of the n = 262144 workload goes in one chunk of 512 nodes instead of three of 170,
    // which matters for the kernels that run one workgroup per node -- so the chunk grows from 48 M to at most 192 M
    // doubles while the temporaries stay within a quarter of the free device memory
    int64_t budget = int64_t(48) << 20;
    {
        size_t free_b = 0, total_b = 0;
        if (hipMemGetInfo(&free_b, &total_b) == hipSuccess) {
            const int64_t fit = (int64_t)((free_b + c->cache.held) / 4 / (12 * sizeof(double)));
            budget = std::min<int64_t>(int64_t(192) << 20, std::max<int64_t>(budget, fit));
        } else {
            (void)hipGetLastError();
        }
    }

    for (int l = L; l >= 1; --l) {
        Level& lv = c->lev[l];
        Level& pl = c->lev[l - 1];
        const int N = lv.N;
        const bool leaves = (l == L);
        Level* cl = leaves ? nullptr : &c->lev[l + 1];
        // offsets of this level's and the parent's diagonal blocks
        std::vector<int64_t> mm(N + 1, 0), pmm(pl.N + 1, 0);
        for (int t = 0; t < N; ++t) mm[t + 1] = mm[t] + (int64_t)lv.msz[t] * lv.msz[t];
        for (int i = 0; i < pl.N; ++i) pmm[i + 1] = pmm[i] + (int64_t)pl.msz[i] * pl.msz[i];
        HSS_TRY(Dbuf[cur ^ 1].reserve(sizeof(double) * pmm[pl.N]));
        double* Dc = Dbuf[cur].as<double>();
        double* Dn = Dbuf[cur ^ 1].as<double>();
        lv.pass.assign(N, 0);
        lv.foff.assign(N + 1, 0);
        lv.kkoff.assign(N + 1, 0);
        for (int t = 0; t < N; ++t) {
            const int m = lv.msz[t], k = lv.rk[t];
            lv.pass[t] = (k == m);
            lv.foff[t + 1] = lv.foff[t] + (lv.pass[t] ? 0 : (int64_t)m * m);
            lv.kkoff[t + 1] = lv.kkoff[t] + (int64_t)k * k;
            if (!lv.pass[t]) {
                const int64_t e = m - k;
                bytes_compact += 2 * (int64_t)sizeof(double) * ((int64_t)m * k + e * e + (int64_t)k * e);
            }
        }
        HSS_TRY(lv.Mup.reserve(sizeof(double) * std::max<int64_t>(lv.foff[N], 1)));
        HSS_TRY(lv.Mdown.reserve(sizeof(double) * std::max<int64_t>(lv.foff[N], 1)));
        HSS_TRY(lv.RT.reserve(sizeof(double) * lv.kkoff[N]));
        HSS_TRY(lv.RTi.reserve(sizeof(double) * lv.kkoff[N]));
        // The orthogonal change of basis Q of every node, the reduced bases R and the parents' off-diagonal
        // blocks R_a B R_b^T depend on the generators U and B only, not on beta: they are kept from the first
        // factorization of a compression and reused by every later one (caching across the grid, Sec. 3.2).
        const bool cached = c->basis_cached;
        HSS_TRY(lv.QT.reserve(sizeof(double) * std::max<int64_t>(lv.foff[N], 1)));
        HSS_TRY(pl.OffD.reserve(sizeof(double) * std::max<int64_t>(pl.boff[pl.N], 1)));
        double* RT = lv.RT.as<double>();
        double* RTi = lv.RTi.as<double>();
        const double* Ug = lv.U.as<double>();

        for (int t0 = 0; t0 < N;) {
            int t1 = t0;
            int64_t acc = 0;
            while (t1 < N && (t1 == t0 || acc + (int64_t)lv.msz[t1] * lv.msz[t1] <= budget)) {
                acc += (int64_t)lv.msz[t1] * lv.msz[t1];
                ++t1;
            }
            const int nc = t1 - t0;
            // local offsets inside the chunk temporaries
            std::vector<int64_t> o_mm(nc + 1, 0), o_km(nc + 1, 0), o_em(nc + 1, 0), o_ee(nc + 1, 0), o_ke(nc + 1, 0),
                o_e(nc + 1, 0);
            for (int q = 0; q < nc; ++q) {
                const int64_t m = lv.msz[t0 + q], k = lv.rk[t0 + q], e = m - k;
                o_mm[q + 1] = o_mm[q] + m * m;
                o_km[q + 1] = o_km[q] + k * m;
                o_em[q + 1] = o_em[q] + e * m;
                o_ee[q + 1] = o_ee[q] + e * e;
                o_ke[q + 1] = o_ke[q] + k * e;
                o_e[q + 1] = o_e[q] + e;
            }
            const size_t dsz = sizeof(double);
            if (!cached) {
                HSS_TRY(UT.reserve(dsz * std::max<int64_t>(o_km[nc], 1)));
                HSS_TRY(PT0.reserve(dsz * std::max<int64_t>(o_em[nc], 1)));
                if (!leaves) HSS_TRY(PT.reserve(dsz * std::max<int64_t>(o_em[nc], 1)));
                HSS_TRY(G2.reserve(dsz * std::max<int64_t>(o_ee[nc], 1)));
                HSS_TRY(L2i.reserve(dsz * std::max<int64_t>(o_ee[nc], 1)));
                HSS_TRY(cholsc.reserve(dsz * (size_t)nc * 1024));
            }
            HSS_TRY(E.reserve(dsz * std::max<int64_t>(o_ee[nc], 1)));
            HSS_TRY(Einv.reserve(dsz * std::max<int64_t>(o_ee[nc], 1)));
            HSS_TRY(Tmp.reserve(dsz * o_mm[nc]));
            HSS_TRY(Dh.reserve(dsz * o_mm[nc]));
            HSS_TRY(W.reserve(dsz * std::max<int64_t>(o_ke[nc], 1)));
            HSS_TRY(Wp.reserve(dsz * std::max<int64_t>(o_ke[nc], 1)));
            HSS_TRY(ipiv.reserve(sizeof(int) * std::max<int64_t>(o_e[nc], 1)));

            // ---- 1. UT = Uf^T = U^T blkdiag(R_a, R_b)^T for every node of the chunk ----
            if (!cached) {
                std::vector<CopyItem> ci;
                std::vector<GemmItem> ga;
                for (int q = 0; q < nc; ++q) {
                    const int t = t0 + q, m = lv.msz[t], k = lv.rk[t];
                    const double* U = Ug + lv.uoff[t];
                    double* ut = UT.as<double>() + o_km[q];
                    if (leaves) {
                        ci.push_back(cp(U, ut, k, m, k, m, COPY_TRANS));
                    } else {
                        const int a = 2 * t, b = 2 * t + 1, ka = cl->rk[a], kb = cl->rk[b];
                        ga.push_back(gi(U, cl->RT.as<double>() + cl->kkoff[a], ut, k, ka, ka, k, ka, m));
                        ga.push_back(gi(U + (size_t)ka * k, cl->RT.as<double>() + cl->kkoff[b], ut + ka, k, kb, kb, k, kb, m));
                    }
                }
                HSS_TRY(bcopy(st, c->arena, ci));
                HSS_TRY(bgemm_host(st, c->arena, ga, true, false, 1.0, 0.0));
            }
            // ---- 2. nodes that eliminate nothing ----
            {
                std::vector<CopyItem> ci;
                std::vector<GemmItem> ga;
                for (int q = 0; q < nc; ++q) {
                    const int t = t0 + q, m = lv.msz[t], k = lv.rk[t];
                    if (!lv.pass[t]) continue;
                    const double* U = Ug + lv.uoff[t];
                    if (!cached) {
                        ci.push_back(cp(UT.as<double>() + o_km[q], RT + lv.kkoff[t], k, k, m, k, COPY_PLAIN));
                        if (leaves) {
                            ci.push_back(cp(U, RTi + lv.kkoff[t], k, k, k, k, COPY_PLAIN));
                        } else {
                            const int a = 2 * t, b = 2 * t + 1, ka = cl->rk[a], kb = cl->rk[b];
                            ga.push_back(gi(cl->RTi.as<double>() + cl->kkoff[a], U, RTi + lv.kkoff[t], ka, k, ka, ka, k, k));
                            ga.push_back(gi(cl->RTi.as<double>() + cl->kkoff[b], U + (size_t)ka * k,
                                            RTi + lv.kkoff[t] + (size_t)ka * k, kb, k, kb, kb, k, k));
                        }
                    }
                    const int i = t / 2, pm = pl.msz[i];
                    const int64_t offp = (t & 1) ? (int64_t)lv.rk[t - 1] * pm + lv.rk[t - 1] : 0;
                    ci.push_back(cp(Dc + mm[t], Dn + pmm[i] + offp, m, m, m, pm, COPY_PLAIN));
                }
                HSS_TRY(bcopy(st, c->arena, ci));
                HSS_TRY(bgemm_host(st, c->arena, ga, false, false, 1.0, 0.0));
            }
            // ---- 3. nodes that eliminate m - k rows ----
            std::vector<int> gen;
            for (int q = 0; q < nc; ++q)
                if (!lv.pass[t0 + q]) gen.push_back(q);
            if (!gen.empty()) {
                double* pt0 = cached ? nullptr : PT0.as<double>();
                double* pt = cached ? nullptr : (leaves ? pt0 : PT.as<double>());
                if (!cached) HIP_TRY(hipMemsetAsync(pt0, 0, dsz * o_em[nc], st));
                std::vector<CompItem> comp;
                std::vector<GemmItem> gpt, gG1, gG2, gQ1, gQ2, gTmp, gDh, gW, gWp, gSch, gMu1, gMu2, gMd;
                std::vector<CopyItem> cId1, cId2, cE, cDrr, cMu, cMd1, cMd2;
                std::vector<LUItem> ch1, ch2, luE;
                std::vector<TrsmItem> tr1, tr2;
                std::vector<double*> einvp;
                std::vector<int> einvld;
                for (int q : gen) {
                    const int t = t0 + q, m = lv.msz[t], k = lv.rk[t], e = m - k;
                    const double* U = Ug + lv.uoff[t];
                    const int* J = lv.J.as<int>() + lv.koff[t];
                    double* qt = lv.QT.as<double>() + lv.foff[t];
                    double* tmp = Tmp.as<double>() + o_mm[q];
                    double* dh = Dh.as<double>() + o_mm[q];
                    double* ee = E.as<double>() + o_ee[q];
                    double* ei = Einv.as<double>() + o_ee[q];
                    double* w = W.as<double>() + o_ke[q];
                    double* wp = Wp.as<double>() + o_ke[q];
                    double* rt = RT + lv.kkoff[t];
                    double* rti = RTi + lv.kkoff[t];
                    double* mu = lv.Mup.as<double>() + lv.foff[t];
                    double* md = lv.Mdown.as<double>() + lv.foff[t];
                    const double* D = Dc + mm[t];
                    if (!cached) {      // the items that build Q^T, R^T, R^-T (their work buffers exist only then)
                        double* ut = UT.as<double>() + o_km[q];
                        double* p0 = pt0 + o_em[q];
                        double* pp = pt + o_em[q];
                        double* g2 = G2.as<double>() + o_ee[q];
                        double* l2i = L2i.as<double>() + o_ee[q];
                        comp.push_back(CompItem{U, J, p0, m, k, m, 0});
                        if (!leaves) {
                            const int a = 2 * t, b = 2 * t + 1, ka = cl->rk[a], kb = cl->rk[b];
                            gpt.push_back(gi(p0, cl->RTi.as<double>() + cl->kkoff[a], pp, e, ka, ka, m, ka, m));
                            gpt.push_back(gi(p0 + ka, cl->RTi.as<double>() + cl->kkoff[b], pp + ka, e, kb, kb, m, kb, m));
                        }
                        gG1.push_back(gi(ut, ut, rt, k, k, m, m, m, k));
                        gG2.push_back(gi(pp, pp, g2, e, e, m, m, m, e));
                        ch1.push_back(LUItem{rt, nullptr, k, k});
                        ch2.push_back(LUItem{g2, nullptr, e, e});
                        cId1.push_back(cp(nullptr, rti, k, k, k, k, COPY_IDENTITY));
                        cId2.push_back(cp(nullptr, l2i, e, e, e, e, COPY_IDENTITY));
                        tr1.push_back(TrsmItem{rt, rti, k, k, k, k});
                        tr2.push_back(TrsmItem{g2, l2i, e, e, e, e});
                        gQ1.push_back(gi(rti, ut, qt, k, m, k, k, m, m));
                        gQ2.push_back(gi(l2i, pp, qt + (size_t)k * m, e, m, e, e, m, m));
                    }
                    gTmp.push_back(gi(qt, D, tmp, m, m, m, m, m, m));
                    gDh.push_back(gi(tmp, qt, dh, m, m, m, m, m, m));
                    cE.push_back(cp(dh + (size_t)k * m + k, ee, e, e, m, e, COPY_PLAIN));
                    luE.push_back(LUItem{ee, ipiv.as<int>() + o_e[q], e, e});
                    einvp.push_back(ei);
                    einvld.push_back(e);
                    gW.push_back(gi(dh + k, ei, w, k, e, e, m, e, e));
                    gWp.push_back(gi(ei, dh + (size_t)k * m, wp, e, k, e, e, m, k));
                    const int i = t / 2, pm = pl.msz[i];
                    const int64_t offp = (t & 1) ? (int64_t)lv.rk[t - 1] * pm + lv.rk[t - 1] : 0;
                    double* dpar = Dn + pmm[i] + offp;
                    cDrr.push_back(cp(dh, dpar, k, k, m, pm, COPY_PLAIN));
                    gSch.push_back(gi(w, dh + (size_t)k * m, dpar, k, k, e, e, m, pm));
                    cMu.push_back(cp(qt, mu, k, m, m, m, COPY_PLAIN));
                    gMu1.push_back(gi(w, qt + (size_t)k * m, mu, k, m, e, e, m, m));
                    gMu2.push_back(gi(ei, qt + (size_t)k * m, mu + (size_t)k * m, e, m, e, e, m, m));
                    cMd1.push_back(cp(qt, md, m, k, m, m, COPY_TRANS));
                    cMd2.push_back(cp(qt + (size_t)k * m, md + k, m, e, m, m, COPY_TRANS));
                    gMd.push_back(gi(qt + (size_t)k * m, wp, md, m, k, e, m, k, m));
                }
                if (!cached) {      // Q^T = [L1^{-1} Uf^T; L2^{-1} P^T] and R^T = L1, R^{-T}: functions of U alone
                    HSS_TRY(complement_launch(st, c->arena, comp));
                    HSS_TRY(bgemm_host(st, c->arena, gpt, false, true, 1.0, 0.0));
                    HSS_TRY(bgemm_host(st, c->arena, gG1, false, true, 1.0, 0.0));
                    HSS_TRY(bgemm_host(st, c->arena, gG2, false, true, 1.0, 0.0));
                    HSS_TRY(bchol(st, c->arena, ch1, cholsc.as<double>(), c->flags.as<int>() + 1));
                    HSS_TRY(bchol(st, c->arena, ch2, cholsc.as<double>(), c->flags.as<int>() + 1));
                    HSS_TRY(bcopy(st, c->arena, cId1));
                    HSS_TRY(bcopy(st, c->arena, cId2));
                    HSS_TRY(btrsm(st, c->arena, tr1, true, false));
                    HSS_TRY(btrsm(st, c->arena, tr2, true, false));
                    HSS_TRY(bgemm_host(st, c->arena, gQ1, false, false, 1.0, 0.0));
                    HSS_TRY(bgemm_host(st, c->arena, gQ2, false, false, 1.0, 0.0));
                }
                HSS_TRY(bgemm_host(st, c->arena, gTmp, false, false, 1.0, 0.0));
                HSS_TRY(bgemm_host(st, c->arena, gDh, false, true, 1.0, 0.0));
                HSS_TRY(bcopy(st, c->arena, cE));
                HSS_TRY(bgetrf(st, c->arena, luE, true, tiny, c->flags.as<int>()));
                HSS_TRY(bgetri(st, c->arena, luE, einvp, einvld));
                HSS_TRY(bgemm_host(st, c->arena, gW, false, false, 1.0, 0.0));
                HSS_TRY(bgemm_host(st, c->arena, gWp, false, false, 1.0, 0.0));
                HSS_TRY(bcopy(st, c->arena, cDrr));
                HSS_TRY(bgemm_host(st, c->arena, gSch, false, false, -1.0, 1.0));
                HSS_TRY(bcopy(st, c->arena, cMu));
                HSS_TRY(bgemm_host(st, c->arena, gMu1, false, false, -1.0, 1.0));
                HSS_TRY(bgemm_host(st, c->arena, gMu2, false, false, 1.0, 0.0));
                HSS_TRY(bcopy(st, c->arena, cMd1));
                HSS_TRY(bcopy(st, c->arena, cMd2));
                HSS_TRY(bgemm_host(st, c->arena, gMd, true, false, -1.0, 1.0));
            }
            HIP_TRY(hipStreamSynchronize(st));
            c->arena.reset();
            t0 = t1;
        }
        // ---- 4. off-diagonal blocks of the parents: R_a B R_b^T and its transpose ----
        {
            std::vector<int64_t> o_t(pl.N + 1, 0);
            for (int i = 0; i < pl.N; ++i) o_t[i + 1] = o_t[i] + (int64_t)lv.rk[2 * i] * lv.rk[2 * i + 1];
            HSS_TRY(T1.reserve(sizeof(double) * std::max<int64_t>(o_t[pl.N], 1)));
            std::vector<GemmItem> g1(pl.N), g2(pl.N);
            std::vector<CopyItem> cu(pl.N), ct(pl.N);
            for (int i = 0; i < pl.N; ++i) {
                const int a = 2 * i, b = 2 * i + 1, ka = lv.rk[a], kb = lv.rk[b], pm = pl.msz[i];
                double* t1 = T1.as<double>() + o_t[i];
                double* off = pl.OffD.as<double>() + pl.boff[i];       // R_a B R_b^T (ka x kb), kept across betas
                double* dp = Dn + pmm[i];
                g1[i] = gi(RT + lv.kkoff[a], pl.B.as<double>() + pl.boff[i], t1, ka, kb, ka, ka, kb, kb);
                g2[i] = gi(t1, RT + lv.kkoff[b], off, ka, kb, kb, kb, kb, kb);
                cu[i] = cp(off, dp + ka, ka, kb, kb, pm, COPY_PLAIN);
                ct[i] = cp(off, dp + (size_t)ka * pm, kb, ka, kb, pm, COPY_TRANS);
            }
            if (!cached) {
                HSS_TRY(bgemm_host(st, c->arena, g1, true, false, 1.0, 0.0));
                HSS_TRY(bgemm_host(st, c->arena, g2, false, false, 1.0, 0.0));
            }
            HSS_TRY(bcopy(st, c->arena, cu));
            HSS_TRY(bcopy(st, c->arena, ct));
            HIP_TRY(hipStreamSynchronize(st));
            c->arena.reset();
        }
        cur ^= 1;
    }
    // ---- root ----
    {
        Level& rl = c->lev[0];
        rl.pass.assign(1, 0);
        rl.foff = {0, 0};
        const int m = rl.msz[0];
        HSS_TRY(invert_root(c, Dbuf[cur].as<double>(), m, tiny));
        bytes_compact += (int64_t)sizeof(double) * m * m;
    }
    // merged top: what a solve reads is the cut level's operator plus the operators of the levels below the cut
    HSS_TRY(build_top_operator(c, c->opt_merge_top ? choose_top_level(c) : 0));
    bytes_solve = (int64_t)sizeof(double) * c->top_m * c->top_m;
    for (int l = c->top_l + 1; l <= L; ++l) bytes_solve += 2 * (int64_t)sizeof(double) * c->lev[l].foff[c->lev[l].N];
    HSS_TRY(build_solve_tables(c));
    int fl[4] = {0, 0, 0, 0};
    HIP_TRY(hipMemcpyAsync(fl, c->flags.p, sizeof(fl), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    int warn = 0;
    if (fl[0] || fl[1]) warn |= HSS_WPIVOT;
    c->warnings |= warn;
    c->beta = beta;
    c->basis_cached = c->opt_cache_basis != 0;
    c->factor_bytes = bytes_solve;
    c->factor_bytes_compact = bytes_compact;
    c->factored = true;
    c->t_factor = wall() - t_start;
    return warn;
}

// The sweeps of one solve for nrhs interleaved right-hand sides sitting in the leaf-level input vector.
int ulv_solve_inplace(hss_ctx* c, int nrhs) {
    hipStream_t st = c->stream;
    const int L = c->L;
    double* pool = c->vpool.as<double>();
    // four right-hand sides on a wide level: the 16-row work list
    auto sweep = [&](Level& lv, const SolveItem* items) {
        const bool wide = nrhs == 4 && lv.rows_per_wave > 1;
        return solve_level_launch(st, items, wide ? lv.work_wide.as<int2>() : lv.work.as<int2>(),
                                  wide ? lv.nwork_wide : lv.nwork, wide ? WIDE_ROWS_PER_WAVE : lv.rows_per_wave, lv.vec, nrhs,
                                  pool, lv.maxm);
    };
    const int tl = c->top_l;
    for (int l = L; l > tl; --l) {
        Level& lv = c->lev[l];
        if (lv.skip) continue;
        HSS_TRY(sweep(lv, lv.up_items.as<SolveItem>()));
    }
    if (tl == 0) {
        HSS_TRY(sweep(c->lev[0], c->lev[0].up_items.as<SolveItem>()));
    } else {
        HSS_TRY(top_gemv_launch(st, c->topT.as<double>(), c->top_m, pool + (c->top_in - pool) * nrhs,
                                pool + (c->top_out - pool) * nrhs, nrhs));
    }
    for (int l = tl + 1; l <= L; ++l) {
        Level& lv = c->lev[l];
        if (lv.skip) continue;
        HSS_TRY(sweep(lv, lv.down_items.as<SolveItem>()));
    }
    return HSS_OK;
}

// x = (K~ + (delta + beta) I)^{-1} b in cluster-tree order.
int ulv_solve_perm(hss_ctx* c, const double* b_perm, double* x_perm) {
    hipStream_t st = c->stream;
    Level& ll = c->lev[c->L];
    if (b_perm != ll.bvec)
        HIP_TRY(hipMemcpyAsync(ll.bvec, b_perm, sizeof(double) * c->n, hipMemcpyDeviceToDevice, st));
    HSS_TRY(ulv_solve_inplace(c, 1));
    if (x_perm != ll.xvec)
        HIP_TRY(hipMemcpyAsync(x_perm, ll.xvec, sizeof(double) * c->n, hipMemcpyDeviceToDevice, st));
    return HSS_OK;
}
