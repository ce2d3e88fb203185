// Vector kernels (host entry points in vec.hip).
#pragma once
#include "common.h"

constexpr int VEC_BLOCKS = 1024;   // workgroups (and partial sums) of a reduction

struct AdmmVecs {
    double* x;
    double* z;
    double* mu;
    double* rhs;        // right-hand side of the next solve, Y q (written)
    const double* sol;  // solution of the last solve, K_beta^{-1} Y q (read)
    const double* y;    // labels, cluster-tree order
    const double* w;    // Y K_beta^{-1} e
};

int vec_blocks(int64_t n);
int vec_gather(hipStream_t st, double* dst, const double* src, const int64_t* perm, int64_t n);
int vec_scatter(hipStream_t st, double* dst, const double* src, const int64_t* perm, int64_t n);
int vec_mul(hipStream_t st, double* dst, const double* a, const double* b, int64_t n);
int vec_dot(hipStream_t st, const double* a, const double* b, int64_t n, double* partial_dev, double* out_dev);
int vec_axpby(hipStream_t st, double* y, const double* x, double a, double b, int64_t n);
int vec_lanczos_update(hipStream_t st, double* w, const double* v, const double* vp, const double* alpha_dev, double beta,
                       int64_t n);
struct CBox {
    double c[4];        // box bound C of each interleaved column
};
// nr in {1, 2, 4} interleaved columns (x, z, mu, rhs, sol); partials: nr * vec_blocks(n) doubles
int admm_start(hipStream_t st, const AdmmVecs& v, int64_t n, int nr, double* part_out);
int admm_step(hipStream_t st, const AdmmVecs& v, int64_t n, int nr, const CBox& box, double beta, const double* w1_dev,
              const double* part_in, double* part_out);
int vec_column(hipStream_t st, double* dst, const double* src, int64_t n, int nr, int j);
int vec_gather_cols(hipStream_t st, double* dst, const double* src, const int64_t* perm, int64_t n, int nr, int ncols);
int vec_scatter_cols(hipStream_t st, double* dst, const double* src, const int64_t* perm, int64_t n, int nr, int ncols);
int margin_indicator(hipStream_t st, const double* z, double C, double* ebar, int64_t n);
int bias_sums(hipStream_t st, const double* z, const double* y, const double* u, const double* ebar, int64_t n,
              double* partial_dev, double* out_dev);
int zy_column(hipStream_t st, double* Om, int ld, const double* z, const double* yp, const int64_t* perm, int64_t n);
int decision_finish(hipStream_t st, double* dec, const double* S, int ld, double bias, int64_t n_test);
int stream_copy_launch(hipStream_t st, const double* src, double* dst, int64_t n);   // n even, 16-byte aligned

// Centring of the feature rows before the kernel products (the Gaussian kernel sees differences of points only, so a
// common shift changes nothing in exact arithmetic, while the expansion ||f_i||^2 + ||f_j||^2 - 2 f_i . f_j loses
// as many digits as the norms exceed the distances by: data with an offset would lose them all).
constexpr int CENTRE_ROWS = 1024;            // rows per partial sum
inline int64_t centre_work_doubles(int64_t n, int r) { return (n + CENTRE_ROWS - 1) / CENTRE_ROWS * r; }
// mean[c] = (sum over the first n rows of X[row * ld + c]) / n for c < r, partial sums of 1024 rows added in a
// fixed order; work: centre_work_doubles(n, r) doubles
int column_means_launch(hipStream_t st, const double* X, int64_t n, int r, int ld, double* work, double* mean);
// X[row * ld + c] -= mean[c] for row < n, c < r
int centre_rows_launch(hipStream_t st, double* X, int64_t n, int r, int ld, const double* mean);
