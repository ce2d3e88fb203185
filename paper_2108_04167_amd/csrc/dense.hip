// Batched small dense factorizations used by the level-by-level HSS algorithms:
// blocked LU (with or without partial pivoting), blocked triangular solves with many right-hand
// sides, and a few element-wise helpers.  All matrices are row-major.
//
// The blocked algorithms are driven from the host (dense_host.cpp style drivers below): per block
// column one "panel" kernel (one workgroup per matrix, one thread per matrix row, the row's panel
// entries in registers), one kernel that applies the row interchanges and solves for the U12
// block, and one batched MFMA GEMM for the trailing update.
#include "common.h"
#include "dense.h"
#include <algorithm>

namespace {

constexpr int NB = LU_NB;   // panel width

// --------------------------------------------------------------------------------------------
// Panel factorization of columns [j0, j0+nbw) on rows [j0, n).  One workgroup per matrix, thread t
// owns row j0+t.  Requires n - j0 <= 1024.
template <bool PIVOT>
__global__ __launch_bounds__(1024) void getrf_panel_kernel(const LUItem* __restrict__ items, int j0, double tiny,
                                                           int* __restrict__ flags) {
    const LUItem it = items[blockIdx.x];
    const int n = it.n;
    if (j0 >= n) return;
    const int rows = n - j0;
    const int nbw = (n - j0 < NB) ? (n - j0) : NB;
    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    const bool live = t < rows;

    __shared__ double prow[NB];
    __shared__ double crow[NB];
    __shared__ double red_v[16];
    __shared__ int red_i[16];
    __shared__ int piv_s;

    double row[NB];
    double* arow = it.A + (size_t)(j0 + t) * it.ld + j0;
#pragma unroll
    for (int c = 0; c < NB; ++c) row[c] = (live && c < nbw) ? arow[c] : 0.0;

#pragma clang loop unroll(full)
    for (int c = 0; c < NB; ++c) {
        if (c < nbw) {   // uniform across the workgroup
            int p = c;
            if (PIVOT) {
                double v = (live && t >= c) ? fabs(row[c]) : -1.0;
                int vi = t;
#pragma unroll
                for (int off = 32; off > 0; off >>= 1) {
                    double ov = __shfl_xor(v, off, 64);
                    int oi = __shfl_xor(vi, off, 64);
                    if (ov > v || (ov == v && oi < vi)) { v = ov; vi = oi; }
                }
                if (lane == 0) { red_v[wave] = v; red_i[wave] = vi; }
                __syncthreads();
                if (t == 0) {
                    double bv = red_v[0];
                    int bi = red_i[0];
                    const int nw = (int)(blockDim.x >> 6);
                    for (int w = 1; w < nw; ++w)
                        if (red_v[w] > bv || (red_v[w] == bv && red_i[w] < bi)) { bv = red_v[w]; bi = red_i[w]; }
                    piv_s = bi;
                    it.ipiv[j0 + c] = j0 + bi;
                }
                __syncthreads();
                p = piv_s;
            }
            // exchange rows c and p (inside the panel; the rest of the matrix is swapped later)
            if (t == p) {
#pragma unroll
                for (int u = 0; u < NB; ++u) prow[u] = row[u];
            }
            if (t == c && p != c) {
#pragma unroll
                for (int u = 0; u < NB; ++u) crow[u] = row[u];
            }
            __syncthreads();
            if (p != c) {
                if (t == p) {
#pragma unroll
                    for (int u = 0; u < NB; ++u) row[u] = crow[u];
                } else if (t == c) {
#pragma unroll
                    for (int u = 0; u < NB; ++u) row[u] = prow[u];
                }
            }
            const double pv = prow[c];
            if (t == 0 && !(fabs(pv) > tiny)) atomicOr(flags, 1);
            if (live && t > c) {
                const double l = (pv != 0.0) ? row[c] / pv : 0.0;
                row[c] = l;
#pragma unroll
                for (int u = 0; u < NB; ++u)
                    if (u > c) row[u] -= l * prow[u];
            }
            __syncthreads();
        }
    }
    if (live) {
#pragma unroll
        for (int c = 0; c < NB; ++c)
            if (c < nbw) arow[c] = row[c];
    }
}

// After the panel [j0, j0+nbw): apply its row interchanges to the columns outside the panel and
// turn the block row right of the panel into U12 = L11^{-1} A12.  One thread per column.
template <bool PIVOT>
__global__ __launch_bounds__(256) void getrf_rowops_kernel(const LUItem* __restrict__ items, int j0) {
    const LUItem it = items[blockIdx.x];
    const int n = it.n;
    if (j0 >= n) return;
    const int nbw = (n - j0 < NB) ? (n - j0) : NB;
    __shared__ double L11[NB * NB];
    __shared__ int piv[NB];
    for (int idx = threadIdx.x; idx < nbw * nbw; idx += blockDim.x) {
        int r = idx / nbw, c = idx - r * nbw;
        L11[r * NB + c] = it.A[(size_t)(j0 + r) * it.ld + j0 + c];
    }
    if (PIVOT && threadIdx.x < nbw) piv[threadIdx.x] = it.ipiv[j0 + threadIdx.x];
    __syncthreads();
    // columns outside the panel: [0, j0) and [j0+nbw, n)
    const int ncols = n - nbw;
    for (int q = blockIdx.y * blockDim.x + threadIdx.x; q < ncols; q += gridDim.y * blockDim.x) {
        const int col = q < j0 ? q : q + nbw;
        double* a = it.A + col;
        if (PIVOT) {
            for (int c = 0; c < nbw; ++c) {
                int p = piv[c];
                if (p != j0 + c) {
                    double x = a[(size_t)(j0 + c) * it.ld], y = a[(size_t)p * it.ld];
                    a[(size_t)(j0 + c) * it.ld] = y;
                    a[(size_t)p * it.ld] = x;
                }
            }
        }
        if (col >= j0 + nbw) {
            double u[NB];
#pragma unroll
            for (int c = 0; c < NB; ++c) u[c] = c < nbw ? a[(size_t)(j0 + c) * it.ld] : 0.0;
#pragma unroll
            for (int c = 1; c < NB; ++c) {
                if (c < nbw) {
                    double acc = u[c];
#pragma unroll
                    for (int d = 0; d < NB; ++d)
                        if (d < c) acc -= L11[c * NB + d] * u[d];
                    u[c] = acc;
                }
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int c = 0; c < NB; ++c)
                if (c < nbw) a[(size_t)(j0 + c) * it.ld] = u[c];
        }
    }
}

// Cholesky factor from an unpivoted LU of a symmetric positive definite matrix: A = L U with
// U = D L^T, so the Cholesky factor is L sqrt(D).  Two phases to keep reads of the diagonal apart
// from the writes: phase 0 copies sqrt(diag) into a scratch vector, phase 1 scales the lower
// triangle and zeroes the strict upper triangle.
__global__ void chol_diag_kernel(const LUItem* __restrict__ items, double* __restrict__ sq, int sq_stride,
                                 int* __restrict__ flags) {
    const LUItem it = items[blockIdx.x];
    for (int c = threadIdx.x; c < it.n; c += blockDim.x) {
        double d = it.A[(size_t)c * it.ld + c];
        if (!(d > 0.0)) { atomicOr(flags, 1); d = fabs(d) > 0.0 ? fabs(d) : 1.0; }
        sq[(size_t)blockIdx.x * sq_stride + c] = sqrt(d);
    }
}
__global__ void chol_scale_kernel(const LUItem* __restrict__ items, const double* __restrict__ sq, int sq_stride) {
    const LUItem it = items[blockIdx.x];
    const int n = it.n;
    const double* s = sq + (size_t)blockIdx.x * sq_stride;
    for (int idx = blockIdx.y * blockDim.x + threadIdx.x; idx < n * n; idx += gridDim.y * blockDim.x) {
        int r = idx / n, c = idx - r * n;
        double* a = it.A + (size_t)r * it.ld + c;
        if (c > r) *a = 0.0;
        else if (c == r) *a = s[c];
        else *a = (*a) * s[c];
    }
}

// --------------------------------------------------------------------------------------------
// Diagonal-block solve of a blocked triangular solve: X_i = T_ii^{-1} B_i for the nbw rows starting
// at i0; one thread per right-hand-side column.
template <bool LOWER, bool UNIT>
__global__ __launch_bounds__(256) void trsm_diag_kernel(const TrsmItem* __restrict__ items, int i0) {
    const TrsmItem it = items[blockIdx.x];
    const int n = it.n;
    if (i0 >= n) return;
    const int nbw = (n - i0 < NB) ? (n - i0) : NB;
    __shared__ double T[NB * NB];
    for (int idx = threadIdx.x; idx < nbw * nbw; idx += blockDim.x) {
        int r = idx / nbw, c = idx - r * nbw;
        T[r * NB + c] = it.T[(size_t)(i0 + r) * it.ldt + i0 + c];
    }
    __syncthreads();
    for (int col = blockIdx.y * blockDim.x + threadIdx.x; col < it.nrhs; col += gridDim.y * blockDim.x) {
        double* b = it.B + (size_t)i0 * it.ldb + col;
        double x[NB];
#pragma unroll
        for (int c = 0; c < NB; ++c) x[c] = c < nbw ? b[(size_t)c * it.ldb] : 0.0;
        if (LOWER) {
#pragma unroll
            for (int c = 0; c < NB; ++c) {
                if (c < nbw) {
                    double acc = x[c];
#pragma unroll
                    for (int d = 0; d < NB; ++d)
                        if (d < c) acc -= T[c * NB + d] * x[d];
                    x[c] = UNIT ? acc : acc / T[c * NB + c];
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
#pragma unroll
            for (int cc = 0; cc < NB; ++cc) {
                const int c = NB - 1 - cc;
                if (c < nbw) {
                    double acc = x[c];
#pragma unroll
                    for (int d = 0; d < NB; ++d)
                        if (d > c && d < nbw) acc -= T[c * NB + d] * x[d];
                    x[c] = UNIT ? acc : acc / T[c * NB + c];
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
#pragma unroll
        for (int c = 0; c < NB; ++c)
            if (c < nbw) b[(size_t)c * it.ldb] = x[c];
    }
}

// B (n x n) <- P * I for the row interchanges of a pivoted LU (ipiv[i] = row exchanged with row i at
// step i).  One workgroup per matrix.
__global__ __launch_bounds__(256) void perm_identity_kernel(const TrsmItem* __restrict__ items,
                                                            int* const* __restrict__ ipivs) {
    const TrsmItem it = items[blockIdx.x];
    const int n = it.n;
    __shared__ int p[1024];
    for (int i = threadIdx.x; i < n; i += blockDim.x) p[i] = i;
    __syncthreads();
    if (threadIdx.x == 0) {
        const int* ip = ipivs[blockIdx.x];
        for (int i = 0; i < n; ++i) {
            int q = ip[i];
            if (q != i) { int tmp = p[i]; p[i] = p[q]; p[q] = tmp; }
        }
    }
    __syncthreads();
    // row i of P*I is e_{p[i]}
    for (int idx = threadIdx.x; idx < n * n; idx += blockDim.x) {
        int r = idx / n, c = idx - r * n;
        it.B[(size_t)r * it.ldb + c] = (p[r] == c) ? 1.0 : 0.0;
    }
}

__global__ void bcopy_kernel(const CopyItem* __restrict__ items) {
    const CopyItem it = items[blockIdx.x];
    const int total = it.rows * it.cols;     // dst is rows x cols
    for (int idx = blockIdx.y * blockDim.x + threadIdx.x; idx < total; idx += gridDim.y * blockDim.x) {
        int r = idx / it.cols, c = idx - r * it.cols;
        double v;
        if (it.mode == COPY_IDENTITY) v = (r == c) ? 1.0 : 0.0;
        else if (it.mode == COPY_ZERO) v = 0.0;
        else if (it.mode == COPY_TRANS) v = it.src[(size_t)c * it.lds + r];
        else v = it.src[(size_t)r * it.lds + c];
        if (it.mode == COPY_PLAIN_ADD_DIAG && r == c) v += it.diag;
        it.dst[(size_t)r * it.ldd + c] = v;
    }
}

// Transposing items (dst[r][c] = src[c][r]) through 32 x 32 tiles in LDS, so that both the reads (along r, the
// contiguous index of src) and the writes (along c) are coalesced; a workgroup walks over the tiles of its item.
__global__ __launch_bounds__(256) void btrans_kernel(const CopyItem* __restrict__ items) {
    __shared__ double tile[32][33];
    const CopyItem it = items[blockIdx.x];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;       // 32 x 8
    const int tr = (it.rows + 31) / 32, tc = (it.cols + 31) / 32;
    for (int t = blockIdx.y; t < tr * tc; t += gridDim.y) {
        const int r0 = (t / tc) * 32, c0 = (t % tc) * 32;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int c = c0 + ty + 8 * u, r = r0 + tx;
            if (c < it.cols && r < it.rows) tile[ty + 8 * u][tx] = it.src[(size_t)c * it.lds + r];
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int r = r0 + ty + 8 * u, c = c0 + tx;
            if (r < it.rows && c < it.cols) it.dst[(size_t)r * it.ldd + c] = tile[tx][ty + 8 * u];
        }
        __syncthreads();
    }
}

}  // namespace

// ------------------------------------------------------------------------------------------------
// Host drivers
// ------------------------------------------------------------------------------------------------

static unsigned ychunks(int64_t work, int per_block) {
    int64_t c = (work + per_block - 1) / per_block;
    if (c < 1) c = 1;
    if (c > 64) c = 64;
    return (unsigned)c;
}

int bcopy(hipStream_t st, DescArena& ar, const std::vector<CopyItem>& items) {
    if (items.empty()) return HSS_OK;
    int64_t mx = 0;
    for (auto& it : items) mx = std::max<int64_t>(mx, (int64_t)it.rows * it.cols);
    if (mx == 0) return HSS_OK;
    // transposes go through the tiled kernel, everything else through the element-wise one
    std::vector<CopyItem> tr, pl;
    for (auto& it : items) (it.mode == COPY_TRANS ? tr : pl).push_back(it);
    if (!pl.empty()) {
        const CopyItem* d = (const CopyItem*)ar.push(pl.data(), sizeof(CopyItem) * pl.size(), st);
        if (!d) return HSS_ENOMEM;
        hipLaunchKernelGGL(bcopy_kernel, dim3((unsigned)pl.size(), ychunks(mx, 256 * 8)), dim3(256), 0, st, d);
        HIP_TRY(hipGetLastError());
    }
    if (!tr.empty()) {
        int64_t mt = 0;
        for (auto& it : tr) mt = std::max<int64_t>(mt, (int64_t)((it.rows + 31) / 32) * ((it.cols + 31) / 32));
        if (mt > 0) {
            const CopyItem* d = (const CopyItem*)ar.push(tr.data(), sizeof(CopyItem) * tr.size(), st);
            if (!d) return HSS_ENOMEM;
            hipLaunchKernelGGL(btrans_kernel, dim3((unsigned)tr.size(), ychunks(mt, 4)), dim3(256), 0, st, d);
            HIP_TRY(hipGetLastError());
        }
    }
    return HSS_OK;
}

int bgemm_host(hipStream_t st, DescArena& ar, const std::vector<GemmItem>& items, bool ta, bool tb, double alpha,
               double beta) {
    if (items.empty()) return HSS_OK;
    int maxM = 0, maxN = 0;
    for (auto& it : items) {
        maxM = std::max(maxM, it.M);
        maxN = std::max(maxN, it.N);
    }
    if (maxM == 0 || maxN == 0) return HSS_OK;
    const GemmItem* d = (const GemmItem*)ar.push(items.data(), sizeof(GemmItem) * items.size(), st);
    if (!d) return HSS_ENOMEM;
    return bgemm(st, d, (int)items.size(), maxM, maxN, ta, tb, alpha, beta);
}

// In-place blocked LU of every matrix in `mats`.  pivot: partial pivoting with interchanges recorded
// in ipiv (LAPACK convention, 0-based); otherwise no interchanges.  *flags_dev gets bit 0 set when a
// pivot with magnitude <= tiny is met.
int bgetrf(hipStream_t st, DescArena& ar, const std::vector<LUItem>& mats, bool pivot, double tiny, int* flags_dev) {
    if (mats.empty()) return HSS_OK;
    int maxn = 0;
    for (auto& m : mats) maxn = std::max(maxn, m.n);
    if (maxn == 0) return HSS_OK;
    if (maxn > 1024) return HSS_EUNSUPPORTED;
    const LUItem* d = (const LUItem*)ar.push(mats.data(), sizeof(LUItem) * mats.size(), st);
    if (!d) return HSS_ENOMEM;
    const unsigned nm = (unsigned)mats.size();
    std::vector<GemmItem> upd(mats.size());
    for (int j0 = 0; j0 < maxn; j0 += NB) {
        const int rows = maxn - j0;
        const unsigned threads = (unsigned)std::min<int64_t>(1024, round_up(rows, 64));
        if (pivot)
            hipLaunchKernelGGL(getrf_panel_kernel<true>, dim3(nm), dim3(threads), 0, st, d, j0, tiny, flags_dev);
        else
            hipLaunchKernelGGL(getrf_panel_kernel<false>, dim3(nm), dim3(threads), 0, st, d, j0, tiny, flags_dev);
        HIP_TRY(hipGetLastError());
        const bool last = j0 + NB >= maxn;
        if (pivot || !last) {
            unsigned yc = ychunks(maxn, 256);
            if (pivot)
                hipLaunchKernelGGL(getrf_rowops_kernel<true>, dim3(nm, yc), dim3(256), 0, st, d, j0);
            else
                hipLaunchKernelGGL(getrf_rowops_kernel<false>, dim3(nm, yc), dim3(256), 0, st, d, j0);
            HIP_TRY(hipGetLastError());
        }
        if (last) break;
        for (size_t i = 0; i < mats.size(); ++i) {
            const LUItem& m = mats[i];
            int rem = m.n - j0 - NB;
            if (rem < 0) rem = 0;
            double* a = m.A;
            upd[i] = GemmItem{a + (size_t)(j0 + NB) * m.ld + j0, a + (size_t)j0 * m.ld + j0 + NB,
                              a + (size_t)(j0 + NB) * m.ld + j0 + NB, rem, rem, rem > 0 ? NB : 0, m.ld, m.ld, m.ld};
        }
        HSS_TRY(bgemm_host(st, ar, upd, false, false, -1.0, 1.0));
    }
    return HSS_OK;
}

// Cholesky of symmetric positive definite matrices via unpivoted LU; the lower factor replaces the
// matrix, the strict upper triangle is zeroed.  scratch: at least mats.size() * maxn doubles.
int bchol(hipStream_t st, DescArena& ar, const std::vector<LUItem>& mats, double* scratch_dev, int* flags_dev) {
    if (mats.empty()) return HSS_OK;
    int maxn = 0;
    for (auto& m : mats) maxn = std::max(maxn, m.n);
    if (maxn == 0) return HSS_OK;
    HSS_TRY(bgetrf(st, ar, mats, false, 0.0, flags_dev));
    const LUItem* d = (const LUItem*)ar.push(mats.data(), sizeof(LUItem) * mats.size(), st);
    if (!d) return HSS_ENOMEM;
    hipLaunchKernelGGL(chol_diag_kernel, dim3((unsigned)mats.size()), dim3(256), 0, st, d, scratch_dev, maxn, flags_dev);
    HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(chol_scale_kernel, dim3((unsigned)mats.size(), ychunks((int64_t)maxn * maxn, 256 * 8)), dim3(256),
                       0, st, d, scratch_dev, maxn);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}

// B <- T^{-1} B for every item (T triangular n x n, B n x nrhs), blocked by NB rows.
int btrsm(hipStream_t st, DescArena& ar, const std::vector<TrsmItem>& items, bool lower, bool unit) {
    if (items.empty()) return HSS_OK;
    int maxn = 0, maxr = 0;
    for (auto& t : items) {
        maxn = std::max(maxn, t.n);
        maxr = std::max(maxr, t.nrhs);
    }
    if (maxn == 0 || maxr == 0) return HSS_OK;
    const unsigned nm = (unsigned)items.size();
    const unsigned yc = ychunks(maxr, 256);
    std::vector<GemmItem> upd(items.size());
    const int nblk = (maxn + NB - 1) / NB;
    for (int b = 0; b < nblk; ++b) {
        // forward: blocks in ascending order; backward: every matrix walks its own blocks from its
        // last one, so block index is counted from the end of each matrix.
        bool any = false;
        for (size_t i = 0; i < items.size(); ++i) {
            const TrsmItem& t = items[i];
            const int nb_i = (t.n + NB - 1) / NB;
            GemmItem g{nullptr, nullptr, nullptr, 0, 0, 0, t.ldt, t.ldb, t.ldb};
            if (b < nb_i && b > 0 && t.nrhs > 0) {
                if (lower) {
                    const int i0 = b * NB;
                    const int h = std::min(NB, t.n - i0);
                    g = GemmItem{t.T + (size_t)i0 * t.ldt, t.B, t.B + (size_t)i0 * t.ldb, h, t.nrhs, i0, t.ldt, t.ldb, t.ldb};
                } else {
                    const int i0 = (nb_i - 1 - b) * NB;
                    const int h = std::min(NB, t.n - i0);
                    const int k0 = i0 + h;
                    g = GemmItem{t.T + (size_t)i0 * t.ldt + k0, t.B + (size_t)k0 * t.ldb, t.B + (size_t)i0 * t.ldb,
                                 h, t.nrhs, t.n - k0, t.ldt, t.ldb, t.ldb};
                }
                any = true;
            }
            upd[i] = g;
        }
        if (any) HSS_TRY(bgemm_host(st, ar, upd, false, false, -1.0, 1.0));
        // diagonal blocks: for the backward sweep each matrix has its own i0, passed through a per-step
        // item table with the block offset folded into the pointers
        std::vector<TrsmItem> diag(items.size());
        for (size_t i = 0; i < items.size(); ++i) {
            const TrsmItem& t = items[i];
            const int nb_i = (t.n + NB - 1) / NB;
            TrsmItem q = t;
            if (b >= nb_i) { q.n = 0; diag[i] = q; continue; }
            const int i0 = lower ? b * NB : (nb_i - 1 - b) * NB;
            const int h = std::min(NB, t.n - i0);
            q.T = t.T + (size_t)i0 * t.ldt + i0;
            q.B = t.B + (size_t)i0 * t.ldb;
            q.n = h;
            diag[i] = q;
        }
        const TrsmItem* dd = (const TrsmItem*)ar.push(diag.data(), sizeof(TrsmItem) * diag.size(), st);
        if (!dd) return HSS_ENOMEM;
        if (lower && unit) hipLaunchKernelGGL((trsm_diag_kernel<true, true>), dim3(nm, yc), dim3(256), 0, st, dd, 0);
        else if (lower) hipLaunchKernelGGL((trsm_diag_kernel<true, false>), dim3(nm, yc), dim3(256), 0, st, dd, 0);
        else if (unit) hipLaunchKernelGGL((trsm_diag_kernel<false, true>), dim3(nm, yc), dim3(256), 0, st, dd, 0);
        else hipLaunchKernelGGL((trsm_diag_kernel<false, false>), dim3(nm, yc), dim3(256), 0, st, dd, 0);
        HIP_TRY(hipGetLastError());
    }
    return HSS_OK;
}

// X <- A^{-1} from a pivoted LU held in `lus` (A = P^T L U): X = U^{-1} L^{-1} P.  X must not alias A.
int bgetri(hipStream_t st, DescArena& ar, const std::vector<LUItem>& lus, const std::vector<double*>& X,
           const std::vector<int>& ldx) {
    if (lus.empty()) return HSS_OK;
    std::vector<TrsmItem> items(lus.size());
    std::vector<int*> ip(lus.size());
    int maxn = 0;
    for (size_t i = 0; i < lus.size(); ++i) {
        items[i] = TrsmItem{lus[i].A, X[i], lus[i].n, lus[i].n, lus[i].ld, ldx[i]};
        ip[i] = lus[i].ipiv;
        maxn = std::max(maxn, lus[i].n);
    }
    if (maxn == 0) return HSS_OK;
    if (maxn > 1024) return HSS_EUNSUPPORTED;
    const TrsmItem* d = (const TrsmItem*)ar.push(items.data(), sizeof(TrsmItem) * items.size(), st);
    int* const* dip = (int* const*)ar.push(ip.data(), sizeof(int*) * ip.size(), st);
    if (!d || !dip) return HSS_ENOMEM;
    hipLaunchKernelGGL(perm_identity_kernel, dim3((unsigned)items.size()), dim3(256), 0, st, d, dip);
    HIP_TRY(hipGetLastError());
    HSS_TRY(btrsm(st, ar, items, true, true));
    HSS_TRY(btrsm(st, ar, items, false, false));
    return HSS_OK;
}
