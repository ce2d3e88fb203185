// HSS mat-vec with the generators held in FP32 copies (vectors and sums stay FP64): the definiteness guard runs
// Lanczos on it.  The guard wants lambda_min(K~) to a few per cent (its safety factor is 1.1), the mat-vec is bound
// by the bytes of the generators, and rounding them to FP32 perturbs K~ by about 6e-8 of its norm -- far below the
// negative eigenvalues the guard is after -- so the estimate costs half the traffic.  Same launch structure and
// item layout as the FP64 mat-vec (bgemv_rows_kernel); bias, error estimate and hss_matvec keep the FP64 one.
#include "ctx.h"
#include <algorithm>

namespace {

__device__ __forceinline__ double wave_sum64(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

__global__ __launch_bounds__(256) void to_float_kernel(const double* __restrict__ src, float* __restrict__ dst, int64_t count) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)gridDim.x * 256) dst[i] = (float)src[i];
}

// y = alpha * A x + beta * y per item (A in FP32, row-major), one wavefront per four consecutive rows.
// VEC4: 16-byte loads of four columns per lane (needs M, N, lda multiples of 4 and 16-byte aligned rows, 32-byte
// aligned x); NCH chunks of 256 columns cover the widest item.
template <bool VEC4, int NCH>
__global__ __launch_bounds__(256) void bgemv32_rows_kernel(const GemvItem32* __restrict__ items, double alpha, double beta) {
    const GemvItem32 it = items[blockIdx.x];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (it.mode != GEMV_DENSE) {
        for (int j = blockIdx.y * 256 + tid; j < it.M; j += gridDim.y * 256) {
            const double v = alpha * (it.mode == GEMV_GATHER ? it.x[it.perm[j]] : it.x[j]);
            double* dst = it.mode == GEMV_GATHER ? it.y + j : it.y + it.perm[j];
            *dst = beta != 0.0 ? v + beta * (*dst) : v;
        }
        return;
    }
    constexpr int R = 4;
    const int N = it.N;
    for (int row0 = (blockIdx.y * 4 + wave) * R; row0 < it.M; row0 += gridDim.y * 4 * R) {
        double s[R] = {0.0, 0.0, 0.0, 0.0};
        const float* rowp[R];
#pragma unroll
        for (int rr = 0; rr < R; ++rr) rowp[rr] = it.A + (size_t)(row0 + rr < it.M ? row0 + rr : it.M - 1) * it.lda;
        if (VEC4) {
            double xv[NCH][4];
#pragma unroll
            for (int k = 0; k < NCH; ++k) {
                const int c = 4 * lane + 256 * k;
#pragma unroll
                for (int u = 0; u < 4; ++u) xv[k][u] = 0.0;
                if (c < N) {
                    const double2 a = *reinterpret_cast<const double2*>(it.x + c);
                    const double2 b = *reinterpret_cast<const double2*>(it.x + c + 2);
                    xv[k][0] = a.x; xv[k][1] = a.y; xv[k][2] = b.x; xv[k][3] = b.y;
                }
            }
#pragma unroll
            for (int rr = 0; rr < R; ++rr) {
#pragma unroll
                for (int k = 0; k < NCH; ++k) {
                    const int c = 4 * lane + 256 * k;
                    const float4 a = *reinterpret_cast<const float4*>(rowp[rr] + (c < N ? c : 0));
                    s[rr] += (double)a.x * xv[k][0] + (double)a.y * xv[k][1] + (double)a.z * xv[k][2] + (double)a.w * xv[k][3];
                }
            }
        } else {
            for (int c0 = 0; c0 < N; c0 += 64) {        // uniform
                const int c = c0 + lane;
                const double xv = c < N ? it.x[c] : 0.0;
                const int cc = c < N ? c : 0;
#pragma unroll
                for (int rr = 0; rr < R; ++rr) s[rr] += (double)rowp[rr][cc] * xv;
            }
        }
#pragma unroll
        for (int rr = 0; rr < R; ++rr) s[rr] = wave_sum64(s[rr]);
        if (lane < R && row0 + lane < it.M) {
            const double v = alpha * (lane == 0 ? s[0] : lane == 1 ? s[1] : lane == 2 ? s[2] : s[3]);
            double* y = it.y + row0 + lane;
            *y = beta != 0.0 ? v + beta * (*y) : v;
        }
    }
}

int bgemv32_launch(hipStream_t st, const GemvItem32* items_dev, int nitems, int maxM, int maxN, bool vec4, double alpha,
                   double beta) {
    if (nitems <= 0 || maxM <= 0) return HSS_OK;
    if (maxN > 1024) return HSS_EUNSUPPORTED;
    int yc = (maxM + 15) / 16;
    while (yc > 1 && (int64_t)nitems * yc > 16384) yc = (yc + 1) / 2;
    const dim3 g((unsigned)nitems, (unsigned)yc), b(256);
    if (!vec4) hipLaunchKernelGGL((bgemv32_rows_kernel<false, 1>), g, b, 0, st, items_dev, alpha, beta);
    else if (maxN <= 256) hipLaunchKernelGGL((bgemv32_rows_kernel<true, 1>), g, b, 0, st, items_dev, alpha, beta);
    else if (maxN <= 512) hipLaunchKernelGGL((bgemv32_rows_kernel<true, 2>), g, b, 0, st, items_dev, alpha, beta);
    else hipLaunchKernelGGL((bgemv32_rows_kernel<true, 4>), g, b, 0, st, items_dev, alpha, beta);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}

int to_float(hipStream_t st, const double* src, float* dst, int64_t count) {
    if (count <= 0) return HSS_OK;
    const int64_t blocks = std::min<int64_t>((count + 255) / 256, 65536);
    hipLaunchKernelGGL(to_float_kernel, dim3((unsigned)blocks), dim3(256), 0, st, src, dst, count);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}

// item table into the context's upload arena (valid until the arena is reset)
int push_items(hss_ctx* c, const std::vector<GemvItem32>& v, const GemvItem32** out) {
    *out = nullptr;
    if (v.empty()) return HSS_OK;
    *out = (const GemvItem32*)c->arena.push(v.data(), sizeof(GemvItem32) * v.size(), c->stream);
    return *out ? HSS_OK : HSS_ENOMEM;
}

}  // namespace

// FP32 copies of the generators the mat-vec streams (leaf blocks, U, U^T, B, B^T) and its item tables (in the
// context's upload arena, which must not be reset while they are in use).  Needs the FP64 tables
// (build_matvec_tables) in place: same vectors, same item order.
int build_matvec32(hss_ctx* c) {
    hipStream_t st = c->stream;
    const int L = c->L;
    Matvec32& m = c->mv32;
    m.lev.clear();
    m.lev.resize(L + 1);
    double* mvx = c->mv_x.as<double>();
    double* mvy = c->mv_y.as<double>();
    Level& leafl = c->lev[L];
    // one allocation for all copies, every copy at a multiple of 64 floats
    auto pad = [](int64_t cnt) { return (cnt + 63) / 64 * 64; };
    int64_t total = pad(c->doff[leafl.N]);
    for (int l = 1; l <= L; ++l) total += 2 * pad(c->lev[l].uoff[c->lev[l].N]) + 2 * pad(c->lev[l - 1].boff[c->lev[l - 1].N]);
    HSS_TRY(m.pool.reserve(sizeof(float) * (size_t)std::max<int64_t>(total, 64)));
    float* next = m.pool.as<float>();
    auto take = [&](int64_t cnt) {
        float* p = next;
        next += pad(cnt);
        return p;
    };
    m.D = take(c->doff[leafl.N]);
    HSS_TRY(to_float(st, c->Dleaf.as<double>(), m.D, c->doff[leafl.N]));
    for (int l = 1; l <= L; ++l) {
        Level& lv = c->lev[l];
        Level& pl = c->lev[l - 1];
        Matvec32::Lev& ml = m.lev[l];
        const int64_t un = lv.uoff[lv.N], bn = pl.boff[pl.N];
        ml.U = take(un);
        ml.UT = take(un);
        ml.B = take(bn);
        ml.BT = take(bn);
        HSS_TRY(to_float(st, lv.U.as<double>(), ml.U, un));
        HSS_TRY(to_float(st, lv.UT.as<double>(), ml.UT, un));   // entries of nodes that kept all rows are never read
        HSS_TRY(to_float(st, pl.B.as<double>(), ml.B, bn));
        HSS_TRY(to_float(st, pl.BT.as<double>(), ml.BT, bn));
    }
    for (int l = L; l >= 1; --l) {
        Level& lv = c->lev[l];
        Level& pl = c->lev[l - 1];
        Matvec32::Lev& ml = m.lev[l];
        const double* xin = (l == L) ? mvx : c->lev[l + 1].xt.as<double>();
        std::vector<GemvItem32> up(lv.N), dn(lv.N);
        bool v4 = true;
        for (int t = 0; t < lv.N; ++t) {
            const float* U = ml.U + lv.uoff[t];
            const float* UT = ml.UT + lv.uoff[t];
            const int32_t* J = lv.J.as<int32_t>() + lv.koff[t];
            const int mm = lv.msz[t], k = lv.rk[t];
            if ((mm | k) & 3) v4 = false;
            double* xt = lv.xt.as<double>() + lv.koff[t];
            const double* g = lv.g.as<double>() + lv.koff[t];
            double* dst = (l == L) ? mvy + lv.moff[t] : c->lev[l + 1].g.as<double>() + lv.moff[t];
            if (k == mm) {
                up[t] = GemvItem32{nullptr, xin + lv.moff[t], xt, J, k, mm, mm, GEMV_GATHER};
                dn[t] = GemvItem32{nullptr, g, dst, J, mm, k, k, GEMV_SCATTER};
            } else {
                up[t] = GemvItem32{UT, xin + lv.moff[t], xt, nullptr, k, mm, mm, GEMV_DENSE};
                dn[t] = GemvItem32{U, g, dst, nullptr, mm, k, k, GEMV_DENSE};
            }
        }
        ml.vec4 = v4;
        HSS_TRY(push_items(c, up, &ml.up));
        HSS_TRY(push_items(c, dn, &ml.dn_u));
        std::vector<GemvItem32> b12(2 * (size_t)pl.N);
        for (int i = 0; i < pl.N; ++i) {
            const int a = 2 * i, b = 2 * i + 1;
            const float* B = ml.B + pl.boff[i];
            const float* BT = ml.BT + pl.boff[i];
            b12[i] = GemvItem32{B, lv.xt.as<double>() + lv.koff[b], lv.g.as<double>() + lv.koff[a], nullptr, lv.rk[a], lv.rk[b],
                                lv.rk[b], GEMV_DENSE};
            b12[pl.N + i] = GemvItem32{BT, lv.xt.as<double>() + lv.koff[a], lv.g.as<double>() + lv.koff[b], nullptr, lv.rk[b],
                                       lv.rk[a], lv.rk[a], GEMV_DENSE};
        }
        HSS_TRY(push_items(c, b12, &ml.dn_b));
        ml.n_dn_b = 2 * pl.N;
    }
    std::vector<GemvItem32> dd(leafl.N);
    bool leaves4 = true;
    for (int t = 0; t < leafl.N; ++t) {
        const int mm = leafl.msz[t];
        if (mm & 3) leaves4 = false;
        dd[t] = GemvItem32{m.D + c->doff[t], mvx + leafl.moff[t], mvy + leafl.moff[t], nullptr, mm, mm, mm, GEMV_DENSE};
    }
    m.leaves4 = leaves4;
    HSS_TRY(push_items(c, dd, &m.leaf_d));   // (the arena has copied the host vectors into its pinned staging area)
    m.ready = true;
    return HSS_OK;
}

// Drops the tables; the pool of copies stays allocated for the next compression of the context (it only grows).
void release_matvec32(hss_ctx* c) {
    DevBuf keep = std::move(c->mv32.pool);
    c->mv32 = Matvec32();
    c->mv32.pool = std::move(keep);
}

// mv_y = (K~ + delta I) mv_x with the FP32 generator copies (cluster-tree order)
int hss_matvec_perm32(hss_ctx* c) {
    hipStream_t st = c->stream;
    const int L = c->L;
    Matvec32& m = c->mv32;
    if (!m.ready) return HSS_ESTATE;
    for (int l = L; l >= 1; --l) {
        Level& lv = c->lev[l];
        HSS_TRY(bgemv32_launch(st, m.lev[l].up, lv.N, lv.maxk, lv.maxm, m.lev[l].vec4, 1.0, 0.0));
    }
    for (int l = 1; l <= L; ++l) {
        Level& lv = c->lev[l];
        const double beta = (l == 1) ? 0.0 : 1.0;
        HSS_TRY(bgemv32_launch(st, m.lev[l].dn_b, m.lev[l].n_dn_b, lv.maxk, lv.maxk, m.lev[l].vec4, 1.0, beta));
        if (l < L) HSS_TRY(bgemv32_launch(st, m.lev[l].dn_u, lv.N, lv.maxm, lv.maxk, m.lev[l].vec4, 1.0, 0.0));
    }
    Level& leafl = c->lev[L];
    HSS_TRY(bgemv32_launch(st, m.leaf_d, leafl.N, leafl.maxm, leafl.maxm, m.leaves4, 1.0, 0.0));
    if (L >= 1) HSS_TRY(bgemv32_launch(st, m.lev[L].dn_u, leafl.N, leafl.maxm, leafl.maxk, m.lev[L].vec4, 1.0, 1.0));
    if (c->delta != 0.0) HSS_TRY(vec_axpby(st, c->mv_y.as<double>(), c->mv_x.as<double>(), c->delta, 1.0, c->n));
    return HSS_OK;
}
