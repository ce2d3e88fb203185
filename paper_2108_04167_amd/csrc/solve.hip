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

// One wavefront computes R consecutive rows of y = M x for one node; the input vector lives in registers
// (lane l holds the columns it multiplies), so a wavefront issues its loads of x and of its R matrix rows
// back to back and waits once.  VEC: 16-byte loads (needs even m, n0, ld and 16-byte aligned pointers).
// A workgroup = 4 wavefronts = 4R rows; the work list gives (node, first row).
template <int R, bool VEC>
__global__ __launch_bounds__(256) void solve_gemv_kernel(const SolveItem* __restrict__ items,
                                                         const int2* __restrict__ work) {
    const int2 w = work[blockIdx.x];
    const SolveItem it = items[w.x];
    const int m = it.m;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (it.M == nullptr) {   // nothing was eliminated at this node: hand the vector through
        for (int r = w.y + tid; r < w.y + 4 * R && r < m; r += 256) {
            double v = r < it.n0 ? it.in0[r] : it.in1[r - it.n0];
            if (r < it.nout0) it.out0[r] = v;
            else it.out1[r - it.nout0] = v;
        }
        return;
    }
    const int row0 = w.y + wave * R;
    if (row0 >= m) return;
    constexpr int KMAX = 16;   // m <= 1024
    double s[R];
#pragma unroll
    for (int rr = 0; rr < R; ++rr) s[rr] = 0.0;
    const double* rowp[R];
#pragma unroll
    for (int rr = 0; rr < R; ++rr) rowp[rr] = it.M + (size_t)(row0 + rr < m ? row0 + rr : m - 1) * it.ld;
    if (VEC) {
#pragma unroll
        for (int k = 0; k < KMAX / 2; ++k) {
            const int c = 2 * lane + 128 * k;
            if (128 * k < m) {          // uniform
                double2 xv = make_double2(0.0, 0.0);
                if (c < m) xv = c < it.n0 ? *reinterpret_cast<const double2*>(it.in0 + c)
                                          : *reinterpret_cast<const double2*>(it.in1 + (c - it.n0));
                const int cc = c < m ? c : 0;
#pragma unroll
                for (int rr = 0; rr < R; ++rr) {
                    // streamed once per sweep: non-temporal, so the factors do not displace the vectors in cache
                    const v2d a = __builtin_nontemporal_load(reinterpret_cast<const v2d*>(rowp[rr] + cc));
                    s[rr] += a.x * xv.x + a.y * xv.y;
                }
            }
        }
    } else {
#pragma unroll
        for (int k = 0; k < KMAX; ++k) {
            const int c = lane + 64 * k;
            if (64 * k < m) {           // uniform
                double xv = 0.0;
                if (c < m) xv = c < it.n0 ? it.in0[c] : it.in1[c - it.n0];
                const int cc = c < m ? c : 0;
#pragma unroll
                for (int rr = 0; rr < R; ++rr) s[rr] += __builtin_nontemporal_load(rowp[rr] + cc) * xv;
            }
        }
    }
#pragma unroll
    for (int rr = 0; rr < R; ++rr) s[rr] = wave_sum(s[rr]);
    if (lane == 0) {
#pragma unroll
        for (int rr = 0; rr < R; ++rr) {
            const int r = row0 + rr;
            if (r < m) {
                if (r < it.nout0) it.out0[r] = s[rr];
                else it.out1[r - it.nout0] = s[rr];
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

int solve_level_launch(hipStream_t st, const SolveItem* items_dev, const int2* work_dev, int nwork, int rows_per_wave,
                       bool vec) {
    if (nwork <= 0) return HSS_OK;
    dim3 g((unsigned)nwork), b(256);
#define HSS_SOLVE_CASE(R)                                                                                     \
    case R:                                                                                                   \
        if (vec) hipLaunchKernelGGL((solve_gemv_kernel<R, true>), g, b, 0, st, items_dev, work_dev);          \
        else hipLaunchKernelGGL((solve_gemv_kernel<R, false>), g, b, 0, st, items_dev, work_dev);             \
        break;
    switch (rows_per_wave) {
        HSS_SOLVE_CASE(1)
        HSS_SOLVE_CASE(2)
        HSS_SOLVE_CASE(4)
        HSS_SOLVE_CASE(8)
        default: return HSS_EINVAL;
    }
#undef HSS_SOLVE_CASE
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
