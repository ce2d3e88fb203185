// Batched row interpolative decomposition of one tree level (host entry points in rowid.hip).
#pragma once
#include "common.h"

struct IdLevelArgs {
    double*        W;        // work copy of the level's sample rows (sum msz x ld), destroyed
    int            ld;       // = s_pad, a multiple of 128, <= 512
    const int64_t* moff;     // [nnodes+1] first row of every node
    int            kcap;     // rank cap
    int            kc;       // leading dimension of Lc and jtmp (>= kcap, >= 1)
    int            rows_per_block;
    double         rel, abs_tol;
    int*           done;     // [nnodes]
    double*        r11;      // [nnodes] norm of the first pivot row
    int*           jtmp;     // [nnodes x kc] pivot rows in order (local row indices)
    int*           rk;       // [nnodes] ranks (output)
    double*        Lc;       // [sum msz x kc] Gram-Schmidt coefficients
    int*           sel;      // [sum msz] 0 = not chosen, j+1 = chosen at step j
    const int*     active;   // [nnodes] or null: nodes with active[t] == 0 are left exactly as an earlier run of
                             // the same level left them (ranks, pivots, coefficients)
};

int id_init(hipStream_t st, const IdLevelArgs& a, int nnodes, int maxmsz, double* norms0);
int id_steps(hipStream_t st, const IdLevelArgs& a, int nnodes, int maxmsz, double* norms0, double* norms1);
int id_finish(hipStream_t st, const IdLevelArgs& a, int nnodes, int maxmsz, const int64_t* koff, const int64_t* uoff,
              double* U, int* J);
int id_chol(hipStream_t st, const IdLevelArgs& a, int nnodes, int maxmsz, double* G, const int64_t* goff_dev);
