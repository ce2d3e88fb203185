// Small batched kernels of the HSS construction / ULV set-up (host entry points in levels.hip).
#pragma once
#include "common.h"

struct KBItem {               // out (nr x nc, ldo) = K(points ridx or r0.., points cidx or c0..)
    const int64_t* ridx;
    const int64_t* cidx;
    int64_t r0, c0;
    double* out;
    int32_t nr, nc, ldo, pad;
};

struct CompItem {             // complement of U = P [I; T]
    const double* U;          // m x k row-major, tight
    const int*    J;          // k skeleton rows
    double*       dst;        // (m-k) x m, leading dimension ldd, pre-zeroed
    int32_t m, k, ldd, pad;
};

int kernel_blocks(hipStream_t st, DescArena& ar, const std::vector<KBItem>& items, const double* Fp, int r_pad, double h);
int rowmap_launch(hipStream_t st, const int64_t* moff, const int64_t* koff, const int* jtmp, int kc, int nnodes,
                  int64_t* rowmap);
int copy_rows_launch(hipStream_t st, double* dst, int ldd, const double* src, int lds, const int64_t* rowmap,
                     int64_t nrows, int ncols);
int gather_index_launch(hipStream_t st, int64_t* skel, const int64_t* idx, const int64_t* rowmap, int64_t count);
int complement_launch(hipStream_t st, DescArena& ar, const std::vector<CompItem>& items);
int fill_launch(hipStream_t st, double* p, int64_t n, double v);
