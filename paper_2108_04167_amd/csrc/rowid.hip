// Batched row interpolative decomposition  A_t ~= U_t A_t(J_t, :)  of the sample blocks of all nodes
// of one tree level (per-node truncation of the HSS blocks, end of Sec. 3.2).
//
// Row-pivoted modified Gram-Schmidt, one kernel launch per pivot step for the whole level:
//   step j, node t:  p = argmax_i ||a_i||  over rows not yet chosen;  stop when
//                    ||a_p|| <= max(rel * ||a_p0||, abs) or j reaches the rank cap;
//                    q = a_p / ||a_p||;  every other live row:  r_ij = a_i . q,  a_i -= r_ij q,
//                    and its norm is recomputed from the updated row (no down-dating).
// Every workgroup of a node recomputes the argmax from the node's norm array (<= 1024 values), so no
// grid-wide synchronisation is needed; norms are double buffered between steps.  The coefficients
// r_ij form [L11; L21] (rows in pivot order / the rest), and T = L21 L11^{-1} gives
// U = P [I; T].  A node always keeps at least one row (rank >= 1).
#include "common.h"
#include "rowid.h"

namespace {

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Start of a run for the nodes taking part in it: norms0[i] = ||W_i||^2, sel[i] = 0, rank 0, not done.
// A node that sits the run out is marked done so that no step touches it.  One wavefront per row.
__global__ __launch_bounds__(256) void id_init_kernel(IdLevelArgs a, double* __restrict__ norms0) {
    const int node = blockIdx.x;
    const int64_t m0 = a.moff[node];
    const int msz = (int)(a.moff[node + 1] - m0);
    const bool act = !a.active || a.active[node];
    if (blockIdx.y == 0 && threadIdx.x == 0) {
        a.done[node] = act ? 0 : 1;
        if (act) a.rk[node] = 0;
    }
    if (!act) return;
    const int r0 = blockIdx.y * a.rows_per_block;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int rend = r0 + a.rows_per_block;
    if (rend > msz) rend = msz;
    for (int i = r0 + wave; i < rend; i += 4) {
        const double* w = a.W + (size_t)(m0 + i) * a.ld;
        double acc = 0.0;
        for (int c = lane; c < a.ld; c += 64) {
            double v = w[c];
            acc += v * v;
        }
        acc = wave_sum(acc);
        if (lane == 0) {
            norms0[m0 + i] = acc;
            a.sel[m0 + i] = 0;
        }
    }
}

template <int NPL>   // doubles per lane per row: ld == 64 * NPL
__global__ __launch_bounds__(256) void id_step_kernel(IdLevelArgs a, int j, const double* __restrict__ nin,
                                                      double* __restrict__ nout) {
    const int node = blockIdx.x;
    const int64_t m0 = a.moff[node];
    const int msz = (int)(a.moff[node + 1] - m0);
    const int lim = msz < a.kcap ? msz : a.kcap;
    if (j >= lim || a.done[node]) return;
    const int r0 = blockIdx.y * a.rows_per_block;
    if (r0 >= msz) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // argmax of the live norms of this node (ties -> lowest row)
    double bv = -2.0;
    int bi = 0x7fffffff;
    for (int i = tid; i < msz; i += 256) {
        double v = nin[m0 + i];
        if (v > bv) { bv = v; bi = i; }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        double ov = __shfl_xor(bv, off, 64);
        int oi = __shfl_xor(bi, off, 64);
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
    }
    __shared__ double sv[4];
    __shared__ int si[4];
    if (lane == 0) { sv[wave] = bv; si[wave] = bi; }
    __syncthreads();
    bv = sv[0]; bi = si[0];
#pragma unroll
    for (int w = 1; w < 4; ++w)
        if (sv[w] > bv || (sv[w] == bv && si[w] < bi)) { bv = sv[w]; bi = si[w]; }
    if (bi >= msz) {   // no comparable norm (NaN input): stop this node
        if (blockIdx.y == 0 && tid == 0) a.done[node] = 1;
        return;
    }
    const int p = bi;
    const double pv = sqrt(bv > 0.0 ? bv : 0.0);
    const double r11 = (j == 0) ? pv : a.r11[node];
    double thr = a.rel * r11;
    if (a.abs_tol > thr) thr = a.abs_tol;
    if (j > 0 && !(pv > thr)) {
        if (blockIdx.y == 0 && tid == 0) a.done[node] = 1;
        return;
    }
    if (blockIdx.y == 0 && tid == 0) {
        a.jtmp[(size_t)node * a.kc + j] = p;
        a.rk[node] = j + 1;
        if (j == 0) a.r11[node] = pv;
    }
    const double inv = pv > 0.0 ? 1.0 / pv : 0.0;
    double q[NPL];
    {
        const double* pr = a.W + (size_t)(m0 + p) * a.ld + lane;
#pragma unroll
        for (int u = 0; u < NPL; ++u) q[u] = pr[64 * u] * inv;
    }
    int rend = r0 + a.rows_per_block;
    if (rend > msz) rend = msz;
    for (int i = r0 + wave; i < rend; i += 4) {
        const int64_t gi = m0 + i;
        if (i == p) {
            if (lane == 0) {
                a.Lc[(size_t)gi * a.kc + j] = pv;
                nout[gi] = -1.0;
                a.sel[gi] = j + 1;
            }
            continue;
        }
        if (nin[gi] < 0.0) {
            if (lane == 0) nout[gi] = -1.0;
            continue;
        }
        double* ar = a.W + (size_t)gi * a.ld + lane;
        double x[NPL];
        double dot = 0.0;
#pragma unroll
        for (int u = 0; u < NPL; ++u) {
            x[u] = ar[64 * u];
            dot += x[u] * q[u];
        }
        dot = wave_sum(dot);
        double nn = 0.0;
#pragma unroll
        for (int u = 0; u < NPL; ++u) {
            x[u] -= dot * q[u];
            nn += x[u] * x[u];
            ar[64 * u] = x[u];
        }
        nn = wave_sum(nn);
        if (lane == 0) {
            a.Lc[(size_t)gi * a.kc + j] = dot;
            nout[gi] = nn;
        }
    }
}

// The same decomposition from the Gram matrix G = A A^T of a node (msz x msz, built by a batched GEMM): pivoted
// Cholesky of G picks the same rows as row-pivoted Gram-Schmidt of A and its factor holds the same coefficients
// r_ij, but a step touches one row of G instead of every row of A.  One workgroup per node runs all steps:
//   step j: p = argmax of the running diagonal d (rows not yet chosen), stop test as above with |a_p| = sqrt(d_p);
//           l_i = (G[p][i] - sum_{q in panel} l_iq l_pq) / sqrt(d_p),  d_i -= l_i^2;
//   after NB steps (a panel, kept in LDS) the coefficients go to Lc and G -= Lp Lp^T.
// The diagonal is down-dated, so |a_p| carries an absolute error of about 1e-7 |a_p0|: the host uses this
// kernel only when the relative stop threshold is well above that.
template <int NB>
__global__ __launch_bounds__(512) void id_chol_kernel(IdLevelArgs a, double* __restrict__ G, const int64_t* __restrict__ goff,
                                                      int maxm) {
    extern __shared__ double sm[];
    constexpr int LDP = NB + 1;
    const int node = blockIdx.x;
    if (a.active && !a.active[node]) return;
    const int64_t m0 = a.moff[node];
    const int msz = (int)(a.moff[node + 1] - m0);
    const int lim = msz < a.kcap ? msz : a.kcap;
    double* Gn = G + goff[node];
    double* Lp = sm;                                    // [maxm][LDP]
    double* red_v = sm + (size_t)maxm * LDP;            // [2][8]
    int* red_i = reinterpret_cast<int*>(red_v + 16);    // [2][8]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i0 = tid, i1 = tid + 512;                 // the rows this thread owns
    double d0 = i0 < msz ? Gn[(size_t)i0 * msz + i0] : 0.0;
    double d1 = i1 < msz ? Gn[(size_t)i1 * msz + i1] : 0.0;
    int s0 = 0, s1 = 0;                                 // step + 1 at which the row was chosen
    double thr = 0.0;
    int rank = 0, par = 0;
    bool stop = false;
    for (int p0 = 0; p0 < lim && !stop; p0 += NB) {
        int nb = 0;
        for (int jj = 0; jj < NB && p0 + jj < lim; ++jj) {
            const int j = p0 + jj;
            double bv = -1.0;
            int bi = 0x7fffffff;
            if (i0 < msz && s0 == 0 && d0 > bv) { bv = d0; bi = i0; }
            if (i1 < msz && s1 == 0 && d1 > bv) { bv = d1; bi = i1; }
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) {
                const double ov = __shfl_xor(bv, off, 64);
                const int oi = __shfl_xor(bi, off, 64);
                if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
            }
            if (lane == 0) { red_v[par * 8 + wave] = bv; red_i[par * 8 + wave] = bi; }
            __syncthreads();            // also orders the previous step's writes of Lp before this step's reads
            bv = red_v[par * 8];
            bi = red_i[par * 8];
#pragma unroll
            for (int w = 1; w < 8; ++w) {
                const double ov = red_v[par * 8 + w];
                const int oi = red_i[par * 8 + w];
                if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
            }
            par ^= 1;
            if (bi >= msz) { stop = true; break; }      // no comparable value (NaN input)
            const int p = bi;
            const double pv = sqrt(bv > 0.0 ? bv : 0.0);
            if (j == 0) {
                thr = a.rel * pv;
                if (a.abs_tol > thr) thr = a.abs_tol;
                if (tid == 0) a.r11[node] = pv;
            } else if (!(pv > thr)) {
                stop = true;
                break;
            }
            if (tid == 0) a.jtmp[(size_t)node * a.kc + j] = p;
            const double inv = pv > 0.0 ? 1.0 / pv : 0.0;
            const double* Lpp = Lp + (size_t)p * LDP;
            // G is symmetric and only its lower triangle is kept up to date: entry (p, i) is read at
            // (max(p, i), min(p, i))
            if (i0 < msz) {
                double l = 0.0;
                if (i0 == p) { l = pv; s0 = j + 1; }
                else if (s0 == 0) {
                    double c = i0 < p ? Gn[(size_t)p * msz + i0] : Gn[(size_t)i0 * msz + p];
                    const double* Li = Lp + (size_t)i0 * LDP;
                    for (int q = 0; q < jj; ++q) c -= Li[q] * Lpp[q];
                    l = c * inv;
                    d0 -= l * l;
                }
                Lp[(size_t)i0 * LDP + jj] = l;
            }
            if (i1 < msz) {
                double l = 0.0;
                if (i1 == p) { l = pv; s1 = j + 1; }
                else if (s1 == 0) {
                    double c = i1 < p ? Gn[(size_t)p * msz + i1] : Gn[(size_t)i1 * msz + p];
                    const double* Li = Lp + (size_t)i1 * LDP;
                    for (int q = 0; q < jj; ++q) c -= Li[q] * Lpp[q];
                    l = c * inv;
                    d1 -= l * l;
                }
                Lp[(size_t)i1 * LDP + jj] = l;
            }
            rank = j + 1;
            nb = jj + 1;
        }
        __syncthreads();
        if (nb == 0) break;
        // the panel's coefficients: rows of Lc, columns p0 .. p0 + nb
        for (int i = tid; i < msz; i += 512) {
            double* dst = a.Lc + (size_t)(m0 + i) * a.kc + p0;
            const double* src = Lp + (size_t)i * LDP;
            for (int q = 0; q < nb; ++q) dst[q] = src[q];
        }
        if (stop || p0 + nb >= lim) break;
        // G -= Lp Lp^T on the tiles that hold a part of the lower triangle: thread (ty, tx) of a 32 x 16 arrangement
        // owns rows ty + 32 u and columns tx + 16 v of a 128 x 64 tile
        const int ty = tid >> 4, tx = tid & 15;
        for (int rb = 0; rb < msz; rb += 128)
            for (int cb = 0; cb < msz && cb < rb + 128; cb += 64) {
                double acc[4][4];
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc[u][v] = 0.0;
                const int rbase = rb + ty, cbase = cb + tx;
                for (int q = 0; q < nb; ++q) {
                    double av[4], bw[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int r = rbase + 32 * u;
                        av[u] = Lp[(size_t)(r < msz ? r : 0) * LDP + q];
                    }
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int cc = cbase + 16 * v;
                        bw[v] = Lp[(size_t)(cc < msz ? cc : 0) * LDP + q];
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u)
#pragma unroll
                        for (int v = 0; v < 4; ++v) acc[u][v] += av[u] * bw[v];
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int r = rbase + 32 * u;
                    if (r >= msz) continue;
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int cc = cbase + 16 * v;
                        if (cc < msz) Gn[(size_t)r * msz + cc] -= acc[u][v];
                    }
                }
            }
        __threadfence_block();
        __syncthreads();
    }
    // which step chose which row; rank
    if (i0 < msz) a.sel[m0 + i0] = s0;
    if (i1 < msz) a.sel[m0 + i1] = s1;
    if (tid == 0) a.rk[node] = rank;
}

// T = L21 L11^{-1} row by row (a wavefront per group of four rows, a row's coefficients spread over the lanes),
// and assembly of U (msz x k, row-major at uoff[node]) and of the compact skeleton list J.
template <int KU>   // kc <= 64 * KU
__global__ __launch_bounds__(256) void id_finish_kernel(IdLevelArgs a, const int64_t* __restrict__ koff,
                                                        const int64_t* __restrict__ uoff, double* __restrict__ U,
                                                        int* __restrict__ J) {
    const int node = blockIdx.x;
    const int64_t m0 = a.moff[node];
    const int msz = (int)(a.moff[node + 1] - m0);
    const int k = a.rk[node];
    const int r0 = blockIdx.y * a.rows_per_block;
    if (r0 >= msz) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int* jt = a.jtmp + (size_t)node * a.kc;
    if (blockIdx.y == 0)
        for (int c = tid; c < k; c += 256) J[koff[node] + c] = jt[c];
    double* Un = U + uoff[node];
    int rend = r0 + a.rows_per_block;
    if (rend > msz) rend = msz;
    // A wavefront takes every fourth row of the block.  Rows that were chosen as pivots become unit vectors; the
    // others go through the back substitution RB at a time, so that every row of L11 that is fetched serves RB rows
    // (the arithmetic of a row is the same whatever its group).
    constexpr int RB = 4;
    int grp[RB];
    int ng = 0;
    auto substitute = [&]() {
        if (ng == 0) return;
        double l[RB][KU];
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            const double* lr = a.Lc + (size_t)(m0 + grp[r < ng ? r : 0]) * a.kc;
#pragma unroll
            for (int u = 0; u < KU; ++u) {
                const int c = lane + 64 * u;
                l[r][u] = (r < ng && c < k) ? lr[c] : 0.0;
            }
        }
        // back substitution  t L11 = l,  columns from k-1 down to 0; L11[j][c] = Lc[row of pivot j][c], c <= j
#pragma unroll
        for (int uu = 0; uu < KU; ++uu) {
            const int u = KU - 1 - uu;
            if (64 * u >= k) continue;
            for (int jj = 63; jj >= 0; --jj) {
                const int j = 64 * u + jj;
                if (j >= k) continue;
                const double* Lj = a.Lc + (size_t)(m0 + jt[j]) * a.kc;
                const double diag = Lj[j];
                double tj[RB];
#pragma unroll
                for (int r = 0; r < RB; ++r) {
                    double t = __shfl(l[r][u], jj, 64);
                    t = diag != 0.0 ? t / diag : 0.0;
                    if (lane == jj) l[r][u] = t;
                    tj[r] = t;
                }
#pragma unroll
                for (int w = 0; w < KU; ++w) {
                    if (w <= u) {
                        const int c = lane + 64 * w;
                        if (c < j) {
                            const double v = Lj[c];
#pragma unroll
                            for (int r = 0; r < RB; ++r) l[r][w] -= tj[r] * v;
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            if (r >= ng) continue;
            double* urow = Un + (size_t)grp[r] * k;
#pragma unroll
            for (int u = 0; u < KU; ++u) {
                const int c = lane + 64 * u;
                if (c < k) urow[c] = l[r][u];
            }
        }
        ng = 0;
    };
    for (int i = r0 + wave; i < rend; i += 4) {
        const int s = a.sel[m0 + i];
        if (s > 0) {
            double* urow = Un + (size_t)i * k;
            for (int c = lane; c < k; c += 64) urow[c] = (c == s - 1) ? 1.0 : 0.0;
            continue;
        }
        grp[ng++] = i;
        if (ng == RB) substitute();
    }
    substitute();
}

}  // namespace

int id_init(hipStream_t st, const IdLevelArgs& a, int nnodes, int maxmsz, double* norms0) {
    if (nnodes <= 0 || maxmsz <= 0) return HSS_OK;
    const unsigned yc = (unsigned)((maxmsz + a.rows_per_block - 1) / a.rows_per_block);
    hipLaunchKernelGGL(id_init_kernel, dim3((unsigned)nnodes, yc), dim3(256), 0, st, a, norms0);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}

int id_steps(hipStream_t st, const IdLevelArgs& a, int nnodes, int maxmsz, double* norms0, double* norms1) {
    const int steps = maxmsz < a.kcap ? maxmsz : a.kcap;
    const unsigned yc = (unsigned)((maxmsz + a.rows_per_block - 1) / a.rows_per_block);
    dim3 grid((unsigned)nnodes, yc);
    for (int j = 0; j < steps; ++j) {
        const double* nin = (j & 1) ? norms1 : norms0;
        double* nout = (j & 1) ? norms0 : norms1;
        switch (a.ld / 64) {
            case 2: hipLaunchKernelGGL(id_step_kernel<2>, grid, dim3(256), 0, st, a, j, nin, nout); break;
            case 4: hipLaunchKernelGGL(id_step_kernel<4>, grid, dim3(256), 0, st, a, j, nin, nout); break;
            case 6: hipLaunchKernelGGL(id_step_kernel<6>, grid, dim3(256), 0, st, a, j, nin, nout); break;
            case 8: hipLaunchKernelGGL(id_step_kernel<8>, grid, dim3(256), 0, st, a, j, nin, nout); break;
            case 10: hipLaunchKernelGGL(id_step_kernel<10>, grid, dim3(256), 0, st, a, j, nin, nout); break;
            case 12: hipLaunchKernelGGL(id_step_kernel<12>, grid, dim3(256), 0, st, a, j, nin, nout); break;
            case 14: hipLaunchKernelGGL(id_step_kernel<14>, grid, dim3(256), 0, st, a, j, nin, nout); break;
            case 16: hipLaunchKernelGGL(id_step_kernel<16>, grid, dim3(256), 0, st, a, j, nin, nout); break;
            default: return HSS_EUNSUPPORTED;
        }
    }
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}

int id_finish(hipStream_t st, const IdLevelArgs& a, int nnodes, int maxmsz, const int64_t* koff, const int64_t* uoff,
              double* U, int* J) {
    const unsigned yc = (unsigned)((maxmsz + a.rows_per_block - 1) / a.rows_per_block);
    dim3 grid((unsigned)nnodes, yc);
    const int ku = (a.kc + 63) / 64;
    switch (ku) {
        case 1: hipLaunchKernelGGL(id_finish_kernel<1>, grid, dim3(256), 0, st, a, koff, uoff, U, J); break;
        case 2: hipLaunchKernelGGL(id_finish_kernel<2>, grid, dim3(256), 0, st, a, koff, uoff, U, J); break;
        case 3: case 4: hipLaunchKernelGGL(id_finish_kernel<4>, grid, dim3(256), 0, st, a, koff, uoff, U, J); break;
        case 5: case 6: case 7: case 8:
            hipLaunchKernelGGL(id_finish_kernel<8>, grid, dim3(256), 0, st, a, koff, uoff, U, J); break;
        default: return HSS_EUNSUPPORTED;
    }
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}

// All pivot steps of every node of the level from the nodes' Gram matrices (G: msz x msz per node at goff,
// destroyed).  Fills Lc, jtmp, sel, rk, r11 like id_init + id_steps.
int id_chol(hipStream_t st, const IdLevelArgs& a, int nnodes, int maxmsz, double* G, const int64_t* goff_dev) {
    if (nnodes <= 0) return HSS_OK;
    if (maxmsz > 1024) return HSS_EUNSUPPORTED;
    const int nb = maxmsz <= 512 ? 32 : 16;
    const size_t smem = sizeof(double) * ((size_t)maxmsz * (nb + 1) + 16) + sizeof(int) * 16;
    if (nb == 32) {
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(id_chol_kernel<32>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
        hipLaunchKernelGGL(id_chol_kernel<32>, dim3((unsigned)nnodes), dim3(512), smem, st, a, G, goff_dev, maxmsz);
    } else {
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(id_chol_kernel<16>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
        hipLaunchKernelGGL(id_chol_kernel<16>, dim3((unsigned)nnodes), dim3(512), smem, st, a, G, goff_dev, maxmsz);
    }
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}
