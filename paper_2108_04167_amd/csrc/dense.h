// Batched dense building blocks (host drivers in dense.hip).
#pragma once
#include "common.h"

constexpr int LU_NB = 32;   // block size of the blocked LU / triangular solves

struct LUItem {
    double* A;      // n x n, row-major, leading dimension ld
    int*    ipiv;   // n interchanges (may be null without pivoting)
    int32_t n, ld;
};

struct TrsmItem {
    const double* T;   // triangular n x n
    double*       B;   // n x nrhs, overwritten by T^{-1} B
    int32_t n, nrhs, ldt, ldb;
};

enum { COPY_PLAIN = 0, COPY_TRANS = 1, COPY_IDENTITY = 2, COPY_ZERO = 3, COPY_PLAIN_ADD_DIAG = 4 };
struct CopyItem {
    const double* src;
    double*       dst;        // rows x cols
    int32_t rows, cols, lds, ldd, mode;
    int32_t pad;
    double  diag;             // added to the diagonal in mode COPY_PLAIN_ADD_DIAG
};

int bcopy(hipStream_t st, DescArena& ar, const std::vector<CopyItem>& items);
int bgemm_host(hipStream_t st, DescArena& ar, const std::vector<GemmItem>& items, bool ta, bool tb, double alpha,
               double beta);
int bgetrf(hipStream_t st, DescArena& ar, const std::vector<LUItem>& mats, bool pivot, double tiny, int* flags_dev);
int bchol(hipStream_t st, DescArena& ar, const std::vector<LUItem>& mats, double* scratch_dev, int* flags_dev);
int btrsm(hipStream_t st, DescArena& ar, const std::vector<TrsmItem>& items, bool lower, bool unit);
int bgetri(hipStream_t st, DescArena& ar, const std::vector<LUItem>& lus, const std::vector<double*>& X,
           const std::vector<int>& ldx);
