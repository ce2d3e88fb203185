// Matrix-vector kernels of the ULV solve (the operation every ADMM iteration calls, Sec. 2.1.1 and
// Algorithm 3) and of the HSS mat-vec.  Both are streaming operations: every stored factor entry is read
// once per sweep and used for one multiply-add, so they are HBM-bandwidth bound.
//
// ULV solve, level by level:
//   up-sweep    node t:  [b_r'; c_e] = Mup_t b_t          (top k entries go to the parent, the rest stay)
//   root             :  x = Dinv b
//   down-sweep  node t:  x_t = Mdown_t [x_r; c_e]         (x_r handed down by the parent)
// with dense m_t x m_t operators built at factorization time.  A launch processes one level; a work
// list maps workgroups to (node, block of 32 rows) so that ragged node sizes need no padding.
#include "common.h"
#include "solve.h"
#include <algorithm>

namespace {

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

constexpr int RB = SOLVE_ROWS_PER_BLOCK;   // 32 rows per workgroup, 8 per wavefront

__global__ __launch_bounds__(256) void solve_gemv_kernel(const SolveItem* __restrict__ items,
                                                         const int2* __restrict__ work) {
    const int2 w = work[blockIdx.x];
    const SolveItem it = items[w.x];
    const int row0 = w.y;
    const int m = it.m;
    __shared__ double xs[1024];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (it.M == nullptr) {   // nothing was eliminated at this node: hand the vector through
        for (int r = row0 + tid; r < row0 + RB && r < m; r += 256) {
            double v = r < it.n0 ? it.in0[r] : it.in1[r - it.n0];
            if (r < it.nout0) it.out0[r] = v;
            else it.out1[r - it.nout0] = v;
        }
        return;
    }
    for (int c = tid; c < m; c += 256) xs[c] = c < it.n0 ? it.in0[c] : it.in1[c - it.n0];
    __syncthreads();
    const int rbase = row0 + wave * 8;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const int r = rbase + half * 4;
        if (r >= m) break;
        const double* a0 = it.M + (size_t)r * it.ld;
        // rows past the end alias the last valid row (their sums are discarded)
        const double* a1 = it.M + (size_t)(r + 1 < m ? r + 1 : m - 1) * it.ld;
        const double* a2 = it.M + (size_t)(r + 2 < m ? r + 2 : m - 1) * it.ld;
        const double* a3 = it.M + (size_t)(r + 3 < m ? r + 3 : m - 1) * it.ld;
        double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
        for (int c = lane; c < m; c += 64) {
            const double xv = xs[c];
            s0 += a0[c] * xv;
            s1 += a1[c] * xv;
            s2 += a2[c] * xv;
            s3 += a3[c] * xv;
        }
        s0 = wave_sum(s0); s1 = wave_sum(s1); s2 = wave_sum(s2); s3 = wave_sum(s3);
        if (lane < 4) {
            const int rr = r + lane;
            const double v = lane == 0 ? s0 : lane == 1 ? s1 : lane == 2 ? s2 : s3;
            if (rr < m) {
                if (rr < it.nout0) it.out0[rr] = v;
                else it.out1[rr - it.nout0] = v;
            }
        }
    }
}

// y = alpha * A x + beta * y, A is M x N row-major; one wavefront per 4 rows.
__global__ __launch_bounds__(256) void bgemv_n_kernel(const GemvItem* __restrict__ items, double alpha, double beta) {
    const GemvItem it = items[blockIdx.x];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int r = (blockIdx.y * 4 + wave) * 4; r < it.M; r += gridDim.y * 16) {
        double s[4] = {0.0, 0.0, 0.0, 0.0};
        const double* a[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) a[u] = it.A + (size_t)(r + u < it.M ? r + u : it.M - 1) * it.lda;
        for (int c = lane; c < it.N; c += 64) {
            const double xv = it.x[c];
#pragma unroll
            for (int u = 0; u < 4; ++u) s[u] += a[u][c] * xv;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) s[u] = wave_sum(s[u]);
        if (lane < 4 && r + lane < it.M) {
            double v = alpha * (lane == 0 ? s[0] : lane == 1 ? s[1] : lane == 2 ? s[2] : s[3]);
            double* y = it.y + r + lane;
            *y = beta != 0.0 ? v + beta * (*y) : v;
        }
    }
}

// y = alpha * A^T x + beta * y, A is M x N row-major; one workgroup per 64 columns, the four wavefronts
// split the rows and are combined through LDS in a fixed order.
__global__ __launch_bounds__(256) void bgemv_t_kernel(const GemvItem* __restrict__ items, double alpha, double beta) {
    const GemvItem it = items[blockIdx.x];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    __shared__ double part[4][64];
    for (int c0 = blockIdx.y * 64; c0 < it.N; c0 += gridDim.y * 64) {
        const int c = c0 + lane;
        double s = 0.0;
        if (c < it.N)
            for (int r = wave; r < it.M; r += 4) s += it.A[(size_t)r * it.lda + c] * it.x[r];
        part[wave][lane] = s;
        __syncthreads();
        if (wave == 0 && c < it.N) {
            double v = alpha * (((part[0][lane] + part[1][lane]) + part[2][lane]) + part[3][lane]);
            double* y = it.y + c;
            *y = beta != 0.0 ? v + beta * (*y) : v;
        }
        __syncthreads();
    }
}

}  // namespace

int solve_level_launch(hipStream_t st, const SolveItem* items_dev, const int2* work_dev, int nwork) {
    if (nwork <= 0) return HSS_OK;
    hipLaunchKernelGGL(solve_gemv_kernel, dim3((unsigned)nwork), dim3(256), 0, st, items_dev, work_dev);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}

int bgemv_launch(hipStream_t st, const GemvItem* items_dev, int nitems, int maxM, int maxN, bool trans, double alpha,
                 double beta) {
    if (nitems <= 0 || maxM <= 0 || maxN <= 0) return HSS_OK;
    if (!trans) {
        unsigned yc = (unsigned)std::min(64, (maxM + 15) / 16);
        hipLaunchKernelGGL(bgemv_n_kernel, dim3((unsigned)nitems, yc), dim3(256), 0, st, items_dev, alpha, beta);
    } else {
        unsigned yc = (unsigned)std::min(64, (maxN + 63) / 64);
        hipLaunchKernelGGL(bgemv_t_kernel, dim3((unsigned)nitems, yc), dim3(256), 0, st, items_dev, alpha, beta);
    }
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}
