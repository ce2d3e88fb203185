// Matrix-vector kernels of the ULV solve (the operation every ADMM iteration calls, Sec. 2.1.1 and
// Algorithm 3) and of the HSS mat-vec.  Both are streaming operations: every stored factor entry is read
// once per sweep and used for one multiply-add, so they are HBM-bandwidth bound.
//
// ULV solve, level by level:
//   up-sweep    node t:  [b_r'; c_e] = Mup_t b_t          (top k entries go to the parent, the rest stay)
//   root             :  x = Dinv b
//   down-sweep  node t:  x_t = Mdown_t [x_r; c_e]         (x_r handed down by the parent)
// with dense m_t x m_t operators built at factorization time.  A launch processes one level; a work
// list maps workgroups to (node, block of rows) so that ragged node sizes need no padding.
#include "common.h"
#include "solve.h"
#include <algorithm>

namespace {

typedef double v2d __attribute__((ext_vector_type(2)));

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// One wavefront computes R consecutive rows of Y = M X for one node and NR right-hand sides; lane l multiplies
// columns 2l, 2l+1 (+128 per chunk) of every row, and every matrix entry is used NR times.
// VEC: 16-byte loads (needs even m, n0, ld and 16-byte aligned pointers).
// NCH > 0 (VEC only): the level's widest node has at most 128 NCH columns; the lane's share of X is loaded
// first, then the rows are streamed front to back without a branch between the loads.  NCH = 0: chunk by
// chunk over all rows, any width up to 1024.
// A workgroup = 4 wavefronts = 4R rows; the work list gives (node, first row).
//
// Right-hand sides are interleaved: entry i of column j sits at v[i * NR + j].  The item tables hold the
// pointers of the single-column layout, all inside one pool; for NR > 1 a pointer p stands for
// pool + (p - pool) * NR.
template <int NR>
__device__ __forceinline__ const double* scaled(const double* p, const double* pool) {
    return (NR == 1 || p == nullptr) ? p : pool + (p - pool) * NR;
}
template <int NR>
__device__ __forceinline__ double* scaled(double* p, double* pool) {
    return (NR == 1 || p == nullptr) ? p : pool + (p - pool) * NR;
}

template <int R, bool VEC, int NR, int NCH>
__global__ __launch_bounds__(256) void solve_gemv_kernel(const SolveItem* __restrict__ items,
                                                         const int2* __restrict__ work, double* pool) {
    const int2 w = work[blockIdx.x];
    const SolveItem it = items[w.x];
    const int m = it.m;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const double* in0 = scaled<NR>(it.in0, pool);
    const double* in1 = scaled<NR>(it.in1, pool);
    double* out0 = scaled<NR>(it.out0, pool);
    double* out1 = scaled<NR>(it.out1, pool);
    if (it.M == nullptr) {   // nothing was eliminated at this node: hand the vectors through
        const int lo = w.y * NR, hi = (w.y + 4 * R < m ? w.y + 4 * R : m) * NR;
        for (int e = lo + tid; e < hi; e += 256) {
            const double v = e < it.n0 * NR ? in0[e] : in1[e - it.n0 * NR];
            if (e < it.nout0 * NR) out0[e] = v;
            else out1[e - it.nout0 * NR] = v;
        }
        return;
    }
    const int row0 = w.y + wave * R;
    if (row0 >= m) return;
    constexpr int KMAX = 16;   // m <= 1024
    double s[R][NR];
#pragma unroll
    for (int rr = 0; rr < R; ++rr)
#pragma unroll
        for (int j = 0; j < NR; ++j) s[rr][j] = 0.0;
    const double* rowp[R];
#pragma unroll
    for (int rr = 0; rr < R; ++rr) rowp[rr] = it.M + (size_t)(row0 + rr < m ? row0 + rr : m - 1) * it.ld;
    if constexpr (VEC && NCH > 0) {
        // the lane's share of X first (all column chunks), then the matrix rows one after the other: a wavefront
        // reads each row front to back, which the memory system serves measurably faster than chunk-major order
        double x0[NCH][NR], x1[NCH][NR];
#pragma unroll
        for (int k = 0; k < NCH; ++k) {
            const int c = 2 * lane + 128 * k;
#pragma unroll
            for (int j = 0; j < NR; ++j) x0[k][j] = x1[k][j] = 0.0;
            if (c < m) {            // c and n0 are even: both columns come from the same input
                const double* src = c < it.n0 ? in0 + (size_t)c * NR : in1 + (size_t)(c - it.n0) * NR;
#pragma unroll
                for (int q = 0; q < NR; ++q) {      // 2 NR consecutive doubles, 16 bytes at a time
                    const double2 t = *reinterpret_cast<const double2*>(src + 2 * q);
                    if (2 * q < NR) x0[k][2 * q] = t.x; else x1[k][2 * q - NR] = t.x;
                    if (2 * q + 1 < NR) x0[k][2 * q + 1] = t.y; else x1[k][2 * q + 1 - NR] = t.y;
                }
            }
        }
#pragma unroll
        for (int rr = 0; rr < R; ++rr) {
#pragma unroll
            for (int k = 0; k < NCH; ++k) {
                // no branch around the loads (a chunk past the end of a short row re-reads its start against
                // zeros): the compiler keeps all of them in flight
                const int c = 2 * lane + 128 * k;
                const int cc = c < m ? c : 0;
                // streamed once per sweep: non-temporal, so the factors do not displace the vectors in cache
                const v2d a = __builtin_nontemporal_load(reinterpret_cast<const v2d*>(rowp[rr] + cc));
#pragma unroll
                for (int j = 0; j < NR; ++j) s[rr][j] += a.x * x0[k][j] + a.y * x1[k][j];
            }
        }
    } else if (VEC) {
#pragma unroll
        for (int k = 0; k < KMAX / 2; ++k) {
            const int c = 2 * lane + 128 * k;
            if (128 * k < m) {          // uniform
                double x0[NR], x1[NR];
#pragma unroll
                for (int j = 0; j < NR; ++j) x0[j] = x1[j] = 0.0;
                if (c < m) {            // c and n0 are even: both columns come from the same input
                    const double* src = c < it.n0 ? in0 + (size_t)c * NR : in1 + (size_t)(c - it.n0) * NR;
#pragma unroll
                    for (int q = 0; q < NR; ++q) {      // 2 NR consecutive doubles, 16 bytes at a time
                        const double2 t = *reinterpret_cast<const double2*>(src + 2 * q);
                        if (2 * q < NR) x0[2 * q] = t.x; else x1[2 * q - NR] = t.x;
                        if (2 * q + 1 < NR) x0[2 * q + 1] = t.y; else x1[2 * q + 1 - NR] = t.y;
                    }
                }
                const int cc = c < m ? c : 0;
#pragma unroll
                for (int rr = 0; rr < R; ++rr) {
                    // streamed once per sweep: non-temporal, so the factors do not displace the vectors in cache
                    const v2d a = __builtin_nontemporal_load(reinterpret_cast<const v2d*>(rowp[rr] + cc));
#pragma unroll
                    for (int j = 0; j < NR; ++j) s[rr][j] += a.x * x0[j] + a.y * x1[j];
                }
            }
        }
    } else {
#pragma unroll
        for (int k = 0; k < KMAX; ++k) {
            const int c = lane + 64 * k;
            if (64 * k < m) {           // uniform
                double xv[NR];
#pragma unroll
                for (int j = 0; j < NR; ++j) xv[j] = 0.0;
                if (c < m) {
                    const double* src = c < it.n0 ? in0 + (size_t)c * NR : in1 + (size_t)(c - it.n0) * NR;
#pragma unroll
                    for (int j = 0; j < NR; ++j) xv[j] = src[j];
                }
                const int cc = c < m ? c : 0;
#pragma unroll
                for (int rr = 0; rr < R; ++rr) {
                    const double a = __builtin_nontemporal_load(rowp[rr] + cc);
#pragma unroll
                    for (int j = 0; j < NR; ++j) s[rr][j] += a * xv[j];
                }
            }
        }
    }
#pragma unroll
    for (int rr = 0; rr < R; ++rr)
#pragma unroll
        for (int j = 0; j < NR; ++j) s[rr][j] = wave_sum(s[rr][j]);
    if (lane == 0) {
#pragma unroll
        for (int rr = 0; rr < R; ++rr) {
            const int r = row0 + rr;
            if (r < m) {
                double* dst = r < it.nout0 ? out0 + (size_t)r * NR : out1 + (size_t)(r - it.nout0) * NR;
#pragma unroll
                for (int j = 0; j < NR; ++j) dst[j] = s[rr][j];
            }
        }
    }
}

// y = T x for the dense operator that stands for the top of the tree (all levels from the root down to a cut
// level merged into the inverse of the reduced matrix at the cut): T is M x M row-major, M even, M <= 512 NCH.
// A workgroup computes R rows for NR interleaved right-hand sides; thread t multiplies columns 2t, 2t+1 (+512 per
// chunk) of every row with its share of x held in registers, rows streamed front to back as in the level kernel.
template <int R, int NR, int NCH>
__global__ __launch_bounds__(256) void top_gemv_kernel(const double* __restrict__ T, int M, const double* __restrict__ in,
                                                       double* __restrict__ out) {
    __shared__ double red[4][R][NR];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int row0 = blockIdx.x * R;
    double x0[NCH][NR], x1[NCH][NR];
#pragma unroll
    for (int k = 0; k < NCH; ++k) {
        const int c = 2 * tid + 512 * k;
#pragma unroll
        for (int j = 0; j < NR; ++j) x0[k][j] = x1[k][j] = 0.0;
        if (c < M) {
            const double* src = in + (size_t)c * NR;
#pragma unroll
            for (int q = 0; q < NR; ++q) {      // 2 NR consecutive doubles, 16 bytes at a time
                const double2 t = *reinterpret_cast<const double2*>(src + 2 * q);
                if (2 * q < NR) x0[k][2 * q] = t.x; else x1[k][2 * q - NR] = t.x;
                if (2 * q + 1 < NR) x0[k][2 * q + 1] = t.y; else x1[k][2 * q + 1 - NR] = t.y;
            }
        }
    }
    double s[R][NR];
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
        const double* rowp = T + (size_t)(row0 + rr < M ? row0 + rr : M - 1) * M;
#pragma unroll
        for (int j = 0; j < NR; ++j) s[rr][j] = 0.0;
#pragma unroll
        for (int k = 0; k < NCH; ++k) {
            const int c = 2 * tid + 512 * k;
            const v2d a = __builtin_nontemporal_load(reinterpret_cast<const v2d*>(rowp + (c < M ? c : 0)));
#pragma unroll
            for (int j = 0; j < NR; ++j) s[rr][j] += a.x * x0[k][j] + a.y * x1[k][j];
        }
    }
#pragma unroll
    for (int rr = 0; rr < R; ++rr)
#pragma unroll
        for (int j = 0; j < NR; ++j) {
            const double v = wave_sum(s[rr][j]);
            if (lane == 0) red[wave][rr][j] = v;
        }
    __syncthreads();
    if (tid < R * NR) {
        const int rr = tid / NR, j = tid - rr * NR;
        if (row0 + rr < M) out[(size_t)(row0 + rr) * NR + j] = ((red[0][rr][j] + red[1][rr][j]) + red[2][rr][j]) + red[3][rr][j];
    }
}

// Batched y = alpha * A x + beta * y for the HSS mat-vec, A (M x N, N <= 1024) row-major: a wavefront computes
// four consecutive rows with the input vector in registers, as in the solve kernel; transposed products use a
// transposed copy of the generator, so every product streams rows.  Items whose generator is a permutation
// (a node that kept all its rows) only move entries.
template <bool VEC, int NCH>    // NCH: 128-column chunks covering the widest item (16-byte loads only)
__global__ __launch_bounds__(256) void bgemv_rows_kernel(const GemvItem* __restrict__ items, double alpha, double beta) {
    const GemvItem it = items[blockIdx.x];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (it.mode != GEMV_DENSE) {
        for (int j = blockIdx.y * 256 + tid; j < it.M; j += gridDim.y * 256) {
            const double v = alpha * (it.mode == GEMV_GATHER ? it.x[it.perm[j]] : it.x[j]);
            double* dst = it.mode == GEMV_GATHER ? it.y + j : it.y + it.perm[j];
            *dst = beta != 0.0 ? v + beta * (*dst) : v;
        }
        return;
    }
    constexpr int R = 4, KMAX = 16;
    const int N = it.N;
    for (int row0 = (blockIdx.y * 4 + wave) * R; row0 < it.M; row0 += gridDim.y * 4 * R) {
        double s[R] = {0.0, 0.0, 0.0, 0.0};
        const double* rowp[R];
#pragma unroll
        for (int rr = 0; rr < R; ++rr) rowp[rr] = it.A + (size_t)(row0 + rr < it.M ? row0 + rr : it.M - 1) * it.lda;
        if (VEC) {
            // row by row, no branch around the loads (see the solve kernel)
            double2 xv[NCH];
#pragma unroll
            for (int k = 0; k < NCH; ++k) {
                const int c = 2 * lane + 128 * k;
                xv[k] = make_double2(0.0, 0.0);
                if (c < N) xv[k] = *reinterpret_cast<const double2*>(it.x + c);
            }
#pragma unroll
            for (int rr = 0; rr < R; ++rr) {
#pragma unroll
                for (int k = 0; k < NCH; ++k) {
                    const int c = 2 * lane + 128 * k;
                    const v2d a = *reinterpret_cast<const v2d*>(rowp[rr] + (c < N ? c : 0));
                    s[rr] += a.x * xv[k].x + a.y * xv[k].y;
                }
            }
        } else {
#pragma unroll
            for (int k = 0; k < KMAX; ++k) {
                const int c = lane + 64 * k;
                if (64 * k < N) {           // uniform
                    const double xv = c < N ? it.x[c] : 0.0;
                    const int cc = c < N ? c : 0;
#pragma unroll
                    for (int rr = 0; rr < R; ++rr) s[rr] += rowp[rr][cc] * xv;
                }
            }
        }
#pragma unroll
        for (int rr = 0; rr < R; ++rr) s[rr] = wave_sum(s[rr]);
        if (lane < R && row0 + lane < it.M) {
            const double v = alpha * (lane == 0 ? s[0] : lane == 1 ? s[1] : lane == 2 ? s[2] : s[3]);
            double* y = it.y + row0 + lane;
            *y = beta != 0.0 ? v + beta * (*y) : v;
        }
    }
}

}  // namespace

int solve_level_launch(hipStream_t st, const SolveItem* items_dev, const int2* work_dev, int nwork, int rows_per_wave,
                       bool vec, int nrhs, double* pool, int maxm) {
    if (maxm > 1024) return HSS_EUNSUPPORTED;
    if (nwork <= 0) return HSS_OK;
    dim3 g((unsigned)nwork), b(256);
#define HSS_SOLVE_K(R, NR, NCH)                                                                                  \
    hipLaunchKernelGGL((solve_gemv_kernel<R, true, NR, NCH>), g, b, 0, st, items_dev, work_dev, pool)
#define HSS_SOLVE_GO(R, NR)                                                                                      \
    do {                                                                                                         \
        if (vec && (NR == 1 || R == 4) && nch == 2) HSS_SOLVE_K(R, NR, 2);                                       \
        else if (vec && (NR == 1 || R == 4) && nch == 4) HSS_SOLVE_K(R, NR, 4);                                  \
        else if (vec && NR == 1 && nch == 8) HSS_SOLVE_K(R, 1, 8);                                               \
        else if (vec) HSS_SOLVE_K(R, NR, 0);                                                                     \
        else hipLaunchKernelGGL((solve_gemv_kernel<R, false, NR, 0>), g, b, 0, st, items_dev, work_dev, pool); \
    } while (0)
#define HSS_SOLVE_CASE(R)                                                                                         \
    case R:                                                                                                       \
        if (nrhs == 1) HSS_SOLVE_GO(R, 1);                                                                        \
        else if (nrhs == 2) HSS_SOLVE_GO(R, 2);                                                                   \
        else HSS_SOLVE_GO(R, 4);                                                                                  \
        break;
    if (nrhs != 1 && nrhs != 2 && nrhs != 4) return HSS_EINVAL;
    // one right-hand side, 16-byte loads: the row-by-row variant unrolled for the level's widest node
    const int nch = maxm <= 256 ? 2 : (maxm <= 512 ? 4 : 8);
    switch (rows_per_wave) {
        HSS_SOLVE_CASE(1)
        HSS_SOLVE_CASE(2)
        HSS_SOLVE_CASE(4)
        default: return HSS_EINVAL;
    }
#undef HSS_SOLVE_CASE
#undef HSS_SOLVE_K
#undef HSS_SOLVE_GO
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}

int top_gemv_launch(hipStream_t st, const double* T, int M, const double* in, double* out, int nrhs) {
    if (M < 2 || (M & 1) || M > 4096) return HSS_EUNSUPPORTED;
    if (nrhs != 1 && nrhs != 2 && nrhs != 4) return HSS_EINVAL;
    const int nch = M <= 1024 ? 2 : (M <= 2048 ? 4 : 8);
#define HSS_TOP_K(R, NR, NCH)                                                                              \
    hipLaunchKernelGGL((top_gemv_kernel<R, NR, NCH>), dim3((unsigned)((M + R - 1) / R)), dim3(256), 0, st, T, M, in, out)
#define HSS_TOP_GO(R, NR)                        \
    do {                                         \
        if (nch == 2) HSS_TOP_K(R, NR, 2);       \
        else if (nch == 4) HSS_TOP_K(R, NR, 4);  \
        else HSS_TOP_K(R, NR, 8);                \
    } while (0)
    if (nrhs == 1) HSS_TOP_GO(4, 1);
    else if (nrhs == 2) HSS_TOP_GO(4, 2);
    else HSS_TOP_GO(2, 4);
#undef HSS_TOP_GO
#undef HSS_TOP_K
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}

int bgemv_launch(hipStream_t st, const GemvItem* items_dev, int nitems, int maxM, int maxN, bool vec, double alpha,
                 double beta) {
    if (nitems <= 0 || maxM <= 0) return HSS_OK;
    if (maxN > 1024) return HSS_EUNSUPPORTED;
    // enough workgroups to fill the chip, at most one per 16 rows
    int yc = (maxM + 15) / 16;
    while (yc > 1 && (int64_t)nitems * yc > 16384) yc = (yc + 1) / 2;
    const dim3 g((unsigned)nitems, (unsigned)yc), b(256);
    if (!vec) hipLaunchKernelGGL((bgemv_rows_kernel<false, 1>), g, b, 0, st, items_dev, alpha, beta);
    else if (maxN <= 256) hipLaunchKernelGGL((bgemv_rows_kernel<true, 2>), g, b, 0, st, items_dev, alpha, beta);
    else if (maxN <= 512) hipLaunchKernelGGL((bgemv_rows_kernel<true, 4>), g, b, 0, st, items_dev, alpha, beta);
    else hipLaunchKernelGGL((bgemv_rows_kernel<true, 8>), g, b, 0, st, items_dev, alpha, beta);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}
