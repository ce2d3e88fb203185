// ULV solve / HSS mat-vec kernels (host entry points in solve.hip).
#pragma once
#include "common.h"


struct SolveItem {           // y = M [in0(0:n0); in1(0:m-n0)];  y(0:nout0) -> out0, y(nout0:m) -> out1
    const double* M;         // m x m row-major (ld); null = identity (nothing eliminated at this node)
    const double* in0;
    const double* in1;
    double*       out0;
    double*       out1;
    int32_t m, ld, n0, nout0;
};

enum { GEMV_DENSE = 0, GEMV_GATHER = 1, GEMV_SCATTER = 2 };
struct GemvItem {            // y = alpha * op x + beta * y
    const double* A;         // GEMV_DENSE: M x N row-major, y(0:M) = A x(0:N)
    const double* x;
    double*       y;
    const int32_t* perm;     // GEMV_GATHER: y[j] = x[perm[j]];  GEMV_SCATTER: y[perm[j]] = x[j]   (j < M)
    int32_t M, N, lda, mode;
};

struct GemvItem32 {          // the same with the matrix in FP32 (vectors and sums FP64)
    const float*  A;
    const double* x;
    double*       y;
    const int32_t* perm;
    int32_t M, N, lda, mode;
};

// rows_per_wave in {1, 2, 4}: a workgroup (4 wavefronts) takes 4 * rows_per_wave rows of one node.
// nrhs in {1, 2, 4} interleaved right-hand sides; `pool` is the allocation all vector pointers of the item
// tables point into (a pointer p of the tables stands for pool + (p - pool) * nrhs).
// A work item stands for 4 * rows_per_wave rows; maxm = widest node of the table (<= 1024).
int solve_level_launch(hipStream_t st, const SolveItem* items_dev, const int2* work_dev, int nwork, int rows_per_wave,
                       bool vec, int nrhs, double* pool, int maxm);
// out = T in for the dense top-of-tree operator T (M x M row-major, M even, <= 4096); in / out hold nrhs
// interleaved right-hand sides
int top_gemv_launch(hipStream_t st, const double* T, int M, const double* in, double* out, int nrhs);
// vec: every M, N, lda of the table is even and every pointer 16-byte aligned
int bgemv_launch(hipStream_t st, const GemvItem* items_dev, int nitems, int maxM, int maxN, bool vec, double alpha,
                 double beta);
