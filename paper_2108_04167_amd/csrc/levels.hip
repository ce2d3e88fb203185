// Small batched kernels of the level-by-level HSS construction and of the ULV set-up:
// entries of K on index lists (leaf diagonal blocks D and the coupling blocks B, which are entries of
// K itself), row gathers, skeleton index propagation, and the complement basis of an
// interpolative basis.
#include "common.h"
#include "levels.h"
#include <algorithm>

namespace {

// out[i][j] = exp(-||f_ri - f_cj||^2 / (2 h^2)) by direct differences (kernel definition, Sec. 1.1).
// 16 x 16 outputs per workgroup; the 32 points involved are staged in LDS, KB_CHUNK features at a time (the squared
// distance is accumulated feature by feature in index order whatever the chunking).
constexpr int KB_CHUNK = 112;
__global__ __launch_bounds__(256) void kernel_block_kernel(const KBItem* __restrict__ items, const double* __restrict__ Fp,
                                                           int r_pad, int tilesC, double inv2h2) {
    const KBItem it = items[blockIdx.x];
    const int tr = blockIdx.y / tilesC, tc = blockIdx.y % tilesC;
    const int i0 = tr * 16, j0 = tc * 16;
    if (i0 >= it.nr || j0 >= it.nc) return;
    constexpr int ldf = KB_CHUNK + 1;
    __shared__ double Fr[16 * ldf];
    __shared__ double Fc[16 * ldf];
    const int tid = threadIdx.x;
    const int li = tid >> 4, lj = tid & 15;
    double d2 = 0.0;
    for (int f0 = 0; f0 < r_pad; f0 += KB_CHUNK) {
        const int fw = r_pad - f0 < KB_CHUNK ? r_pad - f0 : KB_CHUNK;
        for (int idx = tid; idx < 16 * fw; idx += 256) {
            int q = idx / fw, f = idx - q * fw;
            int i = i0 + q, j = j0 + q;
            double a = 0.0, b = 0.0;
            if (i < it.nr) {
                int64_t g = it.ridx ? it.ridx[i] : it.r0 + i;
                a = Fp[g * r_pad + f0 + f];
            }
            if (j < it.nc) {
                int64_t g = it.cidx ? it.cidx[j] : it.c0 + j;
                b = Fp[g * r_pad + f0 + f];
            }
            Fr[q * ldf + f] = a;
            Fc[q * ldf + f] = b;
        }
        __syncthreads();
        for (int f = 0; f < fw; ++f) {
            double d = Fr[li * ldf + f] - Fc[lj * ldf + f];
            d2 += d * d;
        }
        __syncthreads();
    }
    const int i = i0 + li, j = j0 + lj;
    if (i < it.nr && j < it.nc) it.out[(size_t)i * it.ldo + j] = exp(-d2 * inv2h2);
}

// rowmap[koff[t] + j] = moff[t] + jtmp[t*kc + j]   (global row, within the level, of skeleton j of node t)
__global__ void rowmap_kernel(const int64_t* __restrict__ moff, const int64_t* __restrict__ koff,
                              const int* __restrict__ jtmp, int kc, int nnodes, int64_t* __restrict__ rowmap) {
    const int node = blockIdx.x;
    if (node >= nnodes) return;
    const int k = (int)(koff[node + 1] - koff[node]);
    for (int j = threadIdx.x; j < k; j += blockDim.x) rowmap[koff[node] + j] = moff[node] + jtmp[(size_t)node * kc + j];
}

// dst[q, :] = src[rowmap[q], :]
__global__ void copy_rows_kernel(double* __restrict__ dst, int ldd, const double* __restrict__ src, int lds,
                                 const int64_t* __restrict__ rowmap, int64_t nrows, int ncols) {
    int64_t row = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (row >= nrows) return;
    const int lane = threadIdx.x & 63;
    const double* s = src + (size_t)rowmap[row] * lds;
    double* d = dst + (size_t)row * ldd;
    for (int c = lane; c < ncols; c += 64) d[c] = s[c];
}

// skel[q] = idx ? idx[rowmap[q]] : rowmap[q]
__global__ void gather_index_kernel(int64_t* __restrict__ skel, const int64_t* __restrict__ idx,
                                    const int64_t* __restrict__ rowmap, int64_t count) {
    int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= count) return;
    int64_t g = rowmap[q];
    skel[q] = idx ? idx[g] : g;
}

// Transposed complement of an interpolative basis U = P [I; T] (m x k):  the (m-k) x m matrix PT0 with
// PT0 U = 0, PT0[o][N_o] = 1 and PT0[o][J_j] = -U[N_o][j], where N lists the rows that are not
// skeletons in increasing order.  One workgroup per node; dst must be zeroed beforehand.
__global__ __launch_bounds__(256) void complement_kernel(const CompItem* __restrict__ items) {
    const CompItem it = items[blockIdx.x];
    const int m = it.m, k = it.k;
    if (k >= m) return;
    __shared__ int ord[1024];
    for (int i = threadIdx.x; i < m; i += 256) ord[i] = 0;
    __syncthreads();
    for (int j = threadIdx.x; j < k; j += 256) ord[it.J[j]] = -1;
    __syncthreads();
    if (threadIdx.x == 0) {
        int o = 0;
        for (int i = 0; i < m; ++i)
            if (ord[i] == 0) ord[i] = o++;
            else ord[i] = -1;
    }
    __syncthreads();
    for (int i = threadIdx.x >> 6; i < m; i += 4) {
        const int o = ord[i];
        if (o < 0) continue;
        const int lane = threadIdx.x & 63;
        double* prow = it.dst + (size_t)o * it.ldd;
        if (lane == 0) prow[i] = 1.0;
        for (int j = lane; j < k; j += 64) prow[it.J[j]] = -it.U[(size_t)i * k + j];
    }
}

__global__ void fill_kernel(double* __restrict__ p, int64_t n, double v) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

}  // namespace

int kernel_blocks(hipStream_t st, DescArena& ar, const std::vector<KBItem>& items, const double* Fp, int r_pad, double h) {
    if (items.empty()) return HSS_OK;
    int mr = 0, mc = 0;
    for (auto& it : items) {
        mr = std::max(mr, it.nr);
        mc = std::max(mc, it.nc);
    }
    if (mr == 0 || mc == 0) return HSS_OK;
    const int tilesR = (mr + 15) / 16, tilesC = (mc + 15) / 16;
    if ((int64_t)tilesR * tilesC > 65535) return HSS_EUNSUPPORTED;
    const KBItem* d = (const KBItem*)ar.push(items.data(), sizeof(KBItem) * items.size(), st);
    if (!d) return HSS_ENOMEM;
    hipLaunchKernelGGL(kernel_block_kernel, dim3((unsigned)items.size(), (unsigned)(tilesR * tilesC)), dim3(256), 0, st,
                       d, Fp, r_pad, tilesC, 1.0 / (2.0 * h * h));
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}

int rowmap_launch(hipStream_t st, const int64_t* moff, const int64_t* koff, const int* jtmp, int kc, int nnodes,
                  int64_t* rowmap) {
    if (nnodes <= 0) return HSS_OK;
    hipLaunchKernelGGL(rowmap_kernel, dim3((unsigned)nnodes), dim3(256), 0, st, moff, koff, jtmp, kc, nnodes, rowmap);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}

int copy_rows_launch(hipStream_t st, double* dst, int ldd, const double* src, int lds, const int64_t* rowmap,
                     int64_t nrows, int ncols) {
    if (nrows <= 0) return HSS_OK;
    hipLaunchKernelGGL(copy_rows_kernel, dim3((unsigned)((nrows + 3) / 4)), dim3(256), 0, st, dst, ldd, src, lds, rowmap,
                       nrows, ncols);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}

int gather_index_launch(hipStream_t st, int64_t* skel, const int64_t* idx, const int64_t* rowmap, int64_t count) {
    if (count <= 0) return HSS_OK;
    hipLaunchKernelGGL(gather_index_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st, skel, idx, rowmap,
                       count);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}

int complement_launch(hipStream_t st, DescArena& ar, const std::vector<CompItem>& items) {
    if (items.empty()) return HSS_OK;
    for (auto& it : items)
        if (it.m > 1024) return HSS_EUNSUPPORTED;
    const CompItem* d = (const CompItem*)ar.push(items.data(), sizeof(CompItem) * items.size(), st);
    if (!d) return HSS_ENOMEM;
    hipLaunchKernelGGL(complement_kernel, dim3((unsigned)items.size()), dim3(256), 0, st, d);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}

int fill_launch(hipStream_t st, double* p, int64_t n, double v) {
    if (n <= 0) return HSS_OK;
    hipLaunchKernelGGL(fill_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, n, v);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}
