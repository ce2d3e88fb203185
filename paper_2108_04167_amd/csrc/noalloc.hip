// hss_kernel_sample_noalloc: the kernel-sampling product S = K(F,F) * Omega for callers that may not allocate
// (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  Same kernels as
// hss_kernel_sample; the padded copies of F and Omega, the squared norms and the padded S live in one
// file-scope device array instead of per-call allocations.
//
// Every call on a GPU shares that GPU's array: calls that overlap on one GPU (two streams, two threads) race.
// Every part of the array a call reads is written by the same call first (the padding kernels write whole
// padded tiles, zeros included), so nothing of an earlier, larger call leaks into a later, smaller one.
#include "ctx.h"

namespace {

constexpr int64_t NA_MAX_N = 4096;       // points (rows of F, Omega, S)
constexpr int     NA_MAX_R = 96;         // features
constexpr int     NA_MAX_S = 128;        // columns of Omega
constexpr int64_t NA_NPAD = 4096;        // NA_MAX_N rounded up to the sampling kernel's row tile
constexpr int     NA_RPAD = 112;         // feature_pad(NA_MAX_R)
constexpr int     NA_SPAD = 128;
// Fp (n_pad x r_pad) | nu (n_pad) | Omega (n_pad x s_pad) | S (n_pad x s_pad) | feature means and their partial
// sums (512): 12.1 MB per GPU, held until the process ends
constexpr size_t  NA_MEAN_DOUBLES = 512;     // >= NA_MAX_R + centre_work_doubles(NA_MAX_N, NA_MAX_R) = 96 + 384
constexpr size_t  NA_DOUBLES = (size_t)NA_NPAD * (NA_RPAD + 1 + 2 * NA_SPAD) + NA_MEAN_DOUBLES;

static __device__ __align__(256) double scratch[NA_DOUBLES];

// The array's address on each device.  `scratch` itself is only a host-side stand-in for the symbol: the
// device address comes from hipGetSymbolAddress, asked once per device with that device current.
constexpr int NA_MAX_DEVICES = 64;
double* scratch_ptr[NA_MAX_DEVICES] = {};

// dst (n x s, tight) = src (n x ld), first s columns
__global__ void take_columns_kernel(double* __restrict__ dst, const double* __restrict__ src, int64_t n, int s, int ld) {
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n * s) return;
    const int64_t row = idx / s;
    const int c = (int)(idx - row * s);
    dst[idx] = src[row * ld + c];
}

}  // namespace

// Address of the scratch array on the current device (looked up on first use per device).
int noalloc_scratch_for_current_device(double** out) {
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= NA_MAX_DEVICES) return HSS_EUNSUPPORTED;
    if (!scratch_ptr[dev]) {
        double* p = nullptr;
        if (hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return HSS_EHIP;
        }
        scratch_ptr[dev] = p;
    }
    *out = scratch_ptr[dev];
    return HSS_OK;
}

extern "C" int hss_kernel_sample_noalloc(hss_ctx* ctx, const double* F_dev, int64_t n, int32_t r, double h,
                                         const double* Omega_dev, int32_t s, double* S_out_dev) {
    if (!ctx || !F_dev || !Omega_dev || !S_out_dev || n < 1 || r < 1 || s < 1 || !(h > 0.0)) return HSS_EINVAL;
    if (n > NA_MAX_N || r > NA_MAX_R || s > NA_MAX_S) return HSS_EUNSUPPORTED;
    double* base = nullptr;
    HSS_TRY(noalloc_scratch_for_current_device(&base));
    hipStream_t st = ctx->stream;
    const int64_t n_pad = round_up(n, 256);
    const int r_pad = feature_pad(r), s_pad = NA_SPAD;
    double* Fp = base;
    double* nu = Fp + (size_t)NA_NPAD * NA_RPAD;
    double* Om = nu + NA_NPAD;
    double* S = Om + (size_t)NA_NPAD * NA_SPAD;
    double* mean = S + (size_t)NA_NPAD * NA_SPAD;       // NA_MAX_R means, then the partial sums
    HSS_TRY(gather_pad_rows_launch(st, F_dev, nullptr, Fp, n, n_pad, r, r_pad));
    HSS_TRY(gather_pad_rows_launch(st, Omega_dev, nullptr, Om, n, n_pad, s, s_pad));
    HSS_TRY(column_means_launch(st, Fp, n, r, r_pad, mean + NA_MAX_R, mean));
    HSS_TRY(centre_rows_launch(st, Fp, n, r, r_pad, mean));
    HSS_TRY(row_norms_launch(st, Fp, nu, n_pad, r_pad));
    HSS_TRY(sample_launch(st, Fp, nu, Om, S, n_pad, r_pad, s_pad, h));
    const int64_t total = n * s;
    hipLaunchKernelGGL(take_columns_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, S_out_dev, S, n, s,
                       s_pad);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}
