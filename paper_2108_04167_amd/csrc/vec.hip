// Vector kernels: the per-iteration ADMM updates (Algorithm 2 / Algorithm 3 inner loop), deterministic
// two-stage reductions (wavefront shuffles inside a workgroup, a fixed-order sum over workgroup
// partials), permutation gathers, and the label-assignment kernel of Algorithm 3.
//
// All ADMM vectors live in cluster-tree order inside the library.  Scalars produced on the device
// (w1 = e^T K_beta^{-1} e, w2 = w^T q) stay on the device: an iteration never synchronises with the host.
#include "common.h"
#include "vec.h"

namespace {

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Sum over the workgroup (256 threads); result valid in every thread.
__device__ __forceinline__ double block_sum(double v, double* sh /*[4]*/) {
    v = wave_sum(v);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    __syncthreads();
    if (lane == 0) sh[wave] = v;
    __syncthreads();
    return ((sh[0] + sh[1]) + sh[2]) + sh[3];
}

// Fixed-order sum of `count` partials (count <= VEC_BLOCKS), redundantly by every workgroup.
__device__ __forceinline__ double sum_partials(const double* __restrict__ part, int count, double* sh) {
    double v = 0.0;
    for (int i = threadIdx.x; i < count; i += 256) v += part[i];
    return block_sum(v, sh);
}

__global__ void gather_kernel(double* __restrict__ dst, const double* __restrict__ src, const int64_t* __restrict__ perm,
                              int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src[perm[i]];
}
__global__ void scatter_kernel(double* __restrict__ dst, const double* __restrict__ src, const int64_t* __restrict__ perm,
                               int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[perm[i]] = src[i];
}

// partial[b] = sum over the workgroup's grid-stride slice of a[i]*b[i] (b == nullptr: of a[i])
__global__ __launch_bounds__(256) void dot_partial_kernel(const double* __restrict__ a, const double* __restrict__ b,
                                                          int64_t n, double* __restrict__ partial) {
    __shared__ double sh[4];
    double v = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256)
        v += b ? a[i] * b[i] : a[i];
    v = block_sum(v, sh);
    if (threadIdx.x == 0) partial[blockIdx.x] = v;
}
__global__ __launch_bounds__(256) void finish_sum_kernel(const double* __restrict__ partial, int count,
                                                         double* __restrict__ out) {
    __shared__ double sh[4];
    double v = sum_partials(partial, count, sh);
    if (threadIdx.x == 0) *out = v;
}

// w <- y .* wbar  (Algorithm 3: w = Y K_beta^{-1} e)
__global__ void mul_kernel(double* __restrict__ dst, const double* __restrict__ a, const double* __restrict__ b, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = a[i] * b[i];
}

// The ADMM kernels run NR independent problems that differ only in the box bound C (one beta, one
// factorization): x, z, mu, rhs and sol hold NR interleaved columns (entry i of column j at [i * NR + j]),
// y and w are shared.  Partial sums of column j go to part[j * gridDim.x + workgroup].
//
// Start of a run: x = z = mu = 0, q = e, rhs = Y q = y, partial sums of w^T q.
template <int NR>
__global__ __launch_bounds__(256) void admm_start_kernel(AdmmVecs v, int64_t n, double* __restrict__ part_out) {
    __shared__ double sh[4];
    double acc = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
        const double yi = v.y[i];
#pragma unroll
        for (int j = 0; j < NR; ++j) {
            v.x[i * NR + j] = 0.0;
            v.z[i * NR + j] = 0.0;
            v.mu[i * NR + j] = 0.0;
            v.rhs[i * NR + j] = yi;
        }
        acc += v.w[i];
    }
    acc = block_sum(acc, sh);
    if (threadIdx.x == 0)
        for (int j = 0; j < NR; ++j) part_out[(size_t)j * gridDim.x + blockIdx.x] = acc;
}

// One iteration after the solve: sol holds K_beta^{-1} Y q^k.
//   x = Y sol - (w2 / w1) w;  z = clip(x - mu/beta, 0, C);  mu -= beta (x - z);
//   q = e + mu + beta z;  rhs = Y q;  partial sums of w^T q for the next iteration.
template <int NR>
__global__ __launch_bounds__(256) void admm_step_kernel(AdmmVecs v, int64_t n, CBox box, double beta,
                                                        const double* __restrict__ w1, const double* __restrict__ part_in,
                                                        int nparts, double* __restrict__ part_out) {
    __shared__ double sh[4];
    double ratio[NR], acc[NR];
#pragma unroll
    for (int j = 0; j < NR; ++j) {
        const double w2 = sum_partials(part_in + (size_t)j * nparts, nparts, sh);
        ratio[j] = w2 / (*w1);
        acc[j] = 0.0;
    }
    const double ibeta = 1.0 / beta;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
        const double yi = v.y[i], wi = v.w[i];
#pragma unroll
        for (int j = 0; j < NR; ++j) {
            const int64_t e = i * NR + j;
            const double C = box.c[j];
            const double mu = v.mu[e];
            const double x = yi * v.sol[e] - ratio[j] * wi;
            double z = x - mu * ibeta;
            z = z < 0.0 ? 0.0 : (z > C ? C : z);
            const double mun = mu - beta * (x - z);
            v.x[e] = x;
            v.z[e] = z;
            v.mu[e] = mun;
            const double q = 1.0 + mun + beta * z;
            v.rhs[e] = yi * q;
            acc[j] += wi * q;
        }
    }
#pragma unroll
    for (int j = 0; j < NR; ++j) {
        const double a = block_sum(acc[j], sh);
        if (threadIdx.x == 0) part_out[(size_t)j * gridDim.x + blockIdx.x] = a;
    }
}

// dst[i] = src[i * nr + j]: one column out of an interleaved block
__global__ void column_kernel(double* __restrict__ dst, const double* __restrict__ src, int64_t n, int nr, int j) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src[i * nr + j];
}
// dst[i * nr + j] = src[j * n + perm[i]] for j < ncols (0 beyond): columns in caller order -> interleaved,
// cluster-tree order; and back
__global__ void gather_cols_kernel(double* __restrict__ dst, const double* __restrict__ src,
                                   const int64_t* __restrict__ perm, int64_t n, int nr, int ncols) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int64_t p = perm[i];
    for (int j = 0; j < nr; ++j) dst[i * nr + j] = j < ncols ? src[(size_t)j * n + p] : 0.0;
}
__global__ void scatter_cols_kernel(double* __restrict__ dst, const double* __restrict__ src,
                                    const int64_t* __restrict__ perm, int64_t n, int nr, int ncols) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int64_t p = perm[i];
    for (int j = 0; j < ncols; ++j) dst[(size_t)j * n + p] = src[i * nr + j];
}

// ebar_i = 1 if 0 < z_i < C else 0
__global__ void margin_kernel(const double* __restrict__ z, double C, double* __restrict__ ebar, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) ebar[i] = (z[i] > 0.0 && z[i] < C) ? 1.0 : 0.0;
}
// partials of  sum_M y_j,  sum_i y_i z_i u_i,  |M|
__global__ __launch_bounds__(256) void bias_partial_kernel(const double* __restrict__ z, const double* __restrict__ y,
                                                           const double* __restrict__ u, const double* __restrict__ ebar,
                                                           int64_t n, double* __restrict__ partial /*[3][blocks]*/) {
    __shared__ double sh[4];
    double sy = 0.0, sz = 0.0, sc = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
        const double e = ebar[i];
        sy += e * y[i];
        sc += e;
        sz += y[i] * z[i] * u[i];
    }
    sy = block_sum(sy, sh);
    sz = block_sum(sz, sh);
    sc = block_sum(sc, sh);
    if (threadIdx.x == 0) {
        partial[blockIdx.x] = sy;
        partial[gridDim.x + blockIdx.x] = sz;
        partial[2 * gridDim.x + blockIdx.x] = sc;
    }
}
__global__ __launch_bounds__(256) void finish_sum3_kernel(const double* __restrict__ partial, int count,
                                                          double* __restrict__ out /*[3]*/) {
    __shared__ double sh[4];
    for (int k = 0; k < 3; ++k) {
        double v = sum_partials(partial + (size_t)k * count, count, sh);
        if (threadIdx.x == 0) out[k] = v;
    }
}

// y <- a*x + b*y;  y <- y + c*e? (generic helpers for the Lanczos recurrence of the definiteness guard)
__global__ void axpby_kernel(double* __restrict__ y, const double* __restrict__ x, double a, double b, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) y[i] = a * x[i] + b * y[i];
}
// w <- w - alpha v - beta vprev
// (alpha is read from device memory: the dot product that made it has not been seen by the host yet)
__global__ void lanczos_update_kernel(double* __restrict__ w, const double* __restrict__ v, const double* __restrict__ vp,
                                      const double* __restrict__ alpha_dev, double beta, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const double alpha = *alpha_dev;
    if (i < n) w[i] = w[i] - alpha * v[i] - beta * vp[i];
}

// Label assignment (Algorithm 3, last loop), the parts around the kernel product:
// Om[i * ld] = y_i z_i (cluster-tree order; z in caller order), and dec_j = S[j * ld] + b.
__global__ void zy_column_kernel(double* __restrict__ Om, int ld, const double* __restrict__ z, const double* __restrict__ yp,
                                 const int64_t* __restrict__ perm, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) Om[i * ld] = yp[i] * z[perm[i]];
}
__global__ void decision_finish_kernel(double* __restrict__ dec, const double* __restrict__ S, int ld, double bias,
                                       int64_t n_test) {
    int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j < n_test) dec[j] = S[j * ld] + bias;
}

// dst = src, 16 bytes per lane and access, grid-stride: the plain streaming copy whose known traffic
// calibrates bandwidth figures and the memory counters
__global__ __launch_bounds__(256) void stream_copy_kernel(const double2* __restrict__ src, double2* __restrict__ dst,
                                                          size_t n2) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n2; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

}  // namespace

namespace {
// partial[b * r + c] = sum over rows b*CENTRE_ROWS .. of X[row * ld + c]; columns in groups of at most 256; within a
// group of rc columns thread t adds column t % rc of every (256 / rc)-th row, then the partial sums of a column
// are added in order
__global__ __launch_bounds__(256) void col_partial_kernel(const double* __restrict__ X, int64_t n, int r, int ld,
                                                          double* __restrict__ partial) {
    __shared__ double red[256];
    const int64_t lo = (int64_t)blockIdx.x * CENTRE_ROWS;
    const int64_t hi = lo + CENTRE_ROWS < n ? lo + CENTRE_ROWS : n;
    for (int c0 = 0; c0 < r; c0 += 256) {
        const int rc = r - c0 < 256 ? r - c0 : 256;
        const int npl = 256 / rc;
        const int c = c0 + threadIdx.x % rc, pl = threadIdx.x / rc;
        double acc = 0.0;
        if (pl < npl)
            for (int64_t i = lo + pl; i < hi; i += npl) acc += X[i * ld + c];
        red[threadIdx.x] = acc;
        __syncthreads();
        if (threadIdx.x < rc) {
            double s = 0.0;
            for (int p = 0; p < npl; ++p) s += red[p * rc + threadIdx.x];
            partial[(size_t)blockIdx.x * r + c0 + threadIdx.x] = s;
        }
        __syncthreads();
    }
}
__global__ __launch_bounds__(256) void col_mean_kernel(const double* __restrict__ partial, int64_t chunks, int r, double n,
                                                       double* __restrict__ mean) {
    for (int c = threadIdx.x; c < r; c += 256) {
        double s = 0.0;
        for (int64_t b = 0; b < chunks; ++b) s += partial[b * r + c];
        mean[c] = s / n;
    }
}
__global__ __launch_bounds__(256) void centre_rows_kernel(double* __restrict__ X, int64_t n, int r, int ld,
                                                          const double* __restrict__ mean) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= n * r) return;
    const int64_t row = idx / r;
    const int c = (int)(idx - row * r);
    X[row * ld + c] -= mean[c];
}
}  // namespace

static unsigned eb(int64_t n) { return (unsigned)((n + 255) / 256); }

int vec_blocks(int64_t n) {
    int64_t b = (n + 255) / 256;
    if (b > VEC_BLOCKS) b = VEC_BLOCKS;
    if (b < 1) b = 1;
    return (int)b;
}

int vec_gather(hipStream_t st, double* dst, const double* src, const int64_t* perm, int64_t n) {
    hipLaunchKernelGGL(gather_kernel, dim3(eb(n)), dim3(256), 0, st, dst, src, perm, n);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}
int vec_scatter(hipStream_t st, double* dst, const double* src, const int64_t* perm, int64_t n) {
    hipLaunchKernelGGL(scatter_kernel, dim3(eb(n)), dim3(256), 0, st, dst, src, perm, n);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}
int vec_mul(hipStream_t st, double* dst, const double* a, const double* b, int64_t n) {
    hipLaunchKernelGGL(mul_kernel, dim3(eb(n)), dim3(256), 0, st, dst, a, b, n);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}
// *out_dev = sum a[i]*b[i] (b null: sum a[i]); partial_dev: at least VEC_BLOCKS doubles
int vec_dot(hipStream_t st, const double* a, const double* b, int64_t n, double* partial_dev, double* out_dev) {
    const int nb = vec_blocks(n);
    hipLaunchKernelGGL(dot_partial_kernel, dim3(nb), dim3(256), 0, st, a, b, n, partial_dev);
    hipLaunchKernelGGL(finish_sum_kernel, dim3(1), dim3(256), 0, st, partial_dev, nb, out_dev);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}
int vec_axpby(hipStream_t st, double* y, const double* x, double a, double b, int64_t n) {
    hipLaunchKernelGGL(axpby_kernel, dim3(eb(n)), dim3(256), 0, st, y, x, a, b, n);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}
int vec_lanczos_update(hipStream_t st, double* w, const double* v, const double* vp, const double* alpha_dev, double beta,
                       int64_t n) {
    hipLaunchKernelGGL(lanczos_update_kernel, dim3(eb(n)), dim3(256), 0, st, w, v, vp, alpha_dev, beta, n);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}
int admm_start(hipStream_t st, const AdmmVecs& v, int64_t n, int nr, double* part_out) {
    const dim3 g(vec_blocks(n)), b(256);
    if (nr == 1) hipLaunchKernelGGL(admm_start_kernel<1>, g, b, 0, st, v, n, part_out);
    else if (nr == 2) hipLaunchKernelGGL(admm_start_kernel<2>, g, b, 0, st, v, n, part_out);
    else if (nr == 4) hipLaunchKernelGGL(admm_start_kernel<4>, g, b, 0, st, v, n, part_out);
    else return HSS_EINVAL;
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}
int admm_step(hipStream_t st, const AdmmVecs& v, int64_t n, int nr, const CBox& box, double beta, const double* w1_dev,
              const double* part_in, double* part_out) {
    const int nb = vec_blocks(n);
    const dim3 g(nb), b(256);
    if (nr == 1) hipLaunchKernelGGL(admm_step_kernel<1>, g, b, 0, st, v, n, box, beta, w1_dev, part_in, nb, part_out);
    else if (nr == 2) hipLaunchKernelGGL(admm_step_kernel<2>, g, b, 0, st, v, n, box, beta, w1_dev, part_in, nb, part_out);
    else if (nr == 4) hipLaunchKernelGGL(admm_step_kernel<4>, g, b, 0, st, v, n, box, beta, w1_dev, part_in, nb, part_out);
    else return HSS_EINVAL;
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}
int vec_column(hipStream_t st, double* dst, const double* src, int64_t n, int nr, int j) {
    hipLaunchKernelGGL(column_kernel, dim3(eb(n)), dim3(256), 0, st, dst, src, n, nr, j);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}
int vec_gather_cols(hipStream_t st, double* dst, const double* src, const int64_t* perm, int64_t n, int nr, int ncols) {
    hipLaunchKernelGGL(gather_cols_kernel, dim3(eb(n)), dim3(256), 0, st, dst, src, perm, n, nr, ncols);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}
int vec_scatter_cols(hipStream_t st, double* dst, const double* src, const int64_t* perm, int64_t n, int nr, int ncols) {
    hipLaunchKernelGGL(scatter_cols_kernel, dim3(eb(n)), dim3(256), 0, st, dst, src, perm, n, nr, ncols);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}
int margin_indicator(hipStream_t st, const double* z, double C, double* ebar, int64_t n) {
    hipLaunchKernelGGL(margin_kernel, dim3(eb(n)), dim3(256), 0, st, z, C, ebar, n);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}
// out_dev[0] = sum_M y_j, out_dev[1] = sum_i y_i z_i u_i, out_dev[2] = |M|; partial_dev: 3*VEC_BLOCKS doubles
int bias_sums(hipStream_t st, const double* z, const double* y, const double* u, const double* ebar, int64_t n,
              double* partial_dev, double* out_dev) {
    const int nb = vec_blocks(n);
    hipLaunchKernelGGL(bias_partial_kernel, dim3(nb), dim3(256), 0, st, z, y, u, ebar, n, partial_dev);
    hipLaunchKernelGGL(finish_sum3_kernel, dim3(1), dim3(256), 0, st, partial_dev, nb, out_dev);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}
int zy_column(hipStream_t st, double* Om, int ld, const double* z, const double* yp, const int64_t* perm, int64_t n) {
    hipLaunchKernelGGL(zy_column_kernel, dim3(eb(n)), dim3(256), 0, st, Om, ld, z, yp, perm, n);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}
int decision_finish(hipStream_t st, double* dec, const double* S, int ld, double bias, int64_t n_test) {
    hipLaunchKernelGGL(decision_finish_kernel, dim3(eb(n_test)), dim3(256), 0, st, dec, S, ld, bias, n_test);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}
int column_means_launch(hipStream_t st, const double* X, int64_t n, int r, int ld, double* work, double* mean) {
    if (n < 1 || r < 1) return HSS_EINVAL;
    const int64_t chunks = (n + CENTRE_ROWS - 1) / CENTRE_ROWS;
    hipLaunchKernelGGL(col_partial_kernel, dim3((unsigned)chunks), dim3(256), 0, st, X, n, r, ld, work);
    hipLaunchKernelGGL(col_mean_kernel, dim3(1), dim3(256), 0, st, work, chunks, r, (double)n, mean);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}

int centre_rows_launch(hipStream_t st, double* X, int64_t n, int r, int ld, const double* mean) {
    hipLaunchKernelGGL(centre_rows_kernel, dim3(eb(n * r)), dim3(256), 0, st, X, n, r, ld, mean);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}

int stream_copy_launch(hipStream_t st, const double* src, double* dst, int64_t n) {
    hipLaunchKernelGGL(stream_copy_kernel, dim3(8192), dim3(256), 0, st, reinterpret_cast<const double2*>(src),
                       reinterpret_cast<double2*>(dst), (size_t)n / 2);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}
