// Cluster tree by balanced coordinate bisection (the clustering/reordering preprocess the compression
// relies on, Sec. 1.2), built on the device level by level.
//
// Node rule: split coordinate = the lowest one whose population variance over the node is at least
// (1 - 1e-9) times the largest (variances that differ only by the rounding of their sums count as tied),
// points sorted by (coordinate value, original index), lower half to the left child.
//
// One level = five small kernels (two-pass variance with per-chunk partial sums recombined in a fixed
// order, so the result does not depend on scheduling) and one device-wide merge sort of 16-byte keys
// (node, value, original index): nodes are contiguous equal-width ranges of the index array, so sorting
// the whole array by that key sorts every node in place.
#include "common.h"
#include "ctx.h"
#include <rocprim/device/device_merge_sort.hpp>
#include <algorithm>

namespace {

constexpr int TREE_CHUNK = 256;   // points per partial sum
constexpr int SEG_SHIFT = 40;     // key word = (node << 40) | original index

struct TreeKey {
    double  v;
    int64_t k;
};

struct TreeKeyLess {
    __host__ __device__ bool operator()(const TreeKey& a, const TreeKey& b) const {
        const int64_t sa = a.k >> SEG_SHIFT, sb = b.k >> SEG_SHIFT;
        if (sa != sb) return sa < sb;
        if (a.v != b.v) return a.v < b.v;
        return a.k < b.k;
    }
};

__global__ __launch_bounds__(256) void tree_iota_kernel(int64_t* idx, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) idx[i] = i;
}

// partial[block][c] = sum over the block's chunk of points of F[idx][c] (MODE 0) or of
// (F[idx][c] - mean[node][c])^2 (MODE 1).  Thread t works on coordinate t % r of every (256 / r)-th point.
template <int MODE>
__global__ __launch_bounds__(256) void tree_partial_kernel(const double* __restrict__ F, int r,
                                                           const int64_t* __restrict__ idx, int64_t w, int chunks,
                                                           const double* __restrict__ mean, double* __restrict__ partial) {
    const int64_t node = blockIdx.x / chunks;
    const int ch = blockIdx.x % chunks;
    const int npl = 256 / r;
    const int c = threadIdx.x % r, pl = threadIdx.x / r;
    __shared__ double red[256];
    double acc = 0.0;
    const int64_t lo = node * w + (int64_t)ch * TREE_CHUNK;
    const int64_t hi = lo + TREE_CHUNK < (node + 1) * w ? lo + TREE_CHUNK : (node + 1) * w;
    if (pl < npl) {
        const double m = MODE ? mean[node * r + c] : 0.0;
        for (int64_t i = lo + pl; i < hi; i += npl) {
            const double d = F[idx[i] * r + c] - m;
            acc += MODE ? d * d : d;
        }
    }
    red[threadIdx.x] = acc;
    __syncthreads();
    if (threadIdx.x < r) {
        double s = 0.0;
        for (int p = 0; p < npl; ++p) s += red[p * r + threadIdx.x];
        partial[(size_t)blockIdx.x * r + threadIdx.x] = s;
    }
}

// mean[node][c] = (sum of the node's partials, in chunk order) / w
__global__ __launch_bounds__(128) void tree_mean_kernel(const double* __restrict__ partial, int r, int chunks, double w,
                                                        double* __restrict__ mean) {
    const int c = threadIdx.x;
    if (c >= r) return;
    const double* p = partial + (size_t)blockIdx.x * chunks * r + c;
    double s = 0.0;
    for (int ch = 0; ch < chunks; ++ch) s += p[(size_t)ch * r];
    mean[(size_t)blockIdx.x * r + c] = s / w;
}

// best[node] = lowest coordinate whose summed squared deviation reaches (1 - 1e-9) x the largest.  A sum that is
// not finite (a NaN or an infinity among the features, or squares that overflow) sets *bad: at the root this
// covers every entry of F.
__global__ __launch_bounds__(128) void tree_best_kernel(const double* __restrict__ partial, int r, int chunks,
                                                        int* __restrict__ best, int* __restrict__ bad) {
    __shared__ double var[128];
    const int c = threadIdx.x;
    if (c < r) {
        const double* p = partial + (size_t)blockIdx.x * chunks * r + c;
        double s = 0.0;
        for (int ch = 0; ch < chunks; ++ch) s += p[(size_t)ch * r];
        var[c] = s;
        if (!(s <= 1.7976931348623157e308)) atomicOr(bad, 1);
    }
    __syncthreads();
    if (c == 0) {
        double bv = 0.0;
        for (int k = 0; k < r; ++k) bv = var[k] > bv ? var[k] : bv;
        const double thr = bv * (1.0 - 1e-9);
        int b = 0;
        while (b < r - 1 && !(var[b] >= thr)) ++b;
        best[blockIdx.x] = b;
    }
}

__global__ __launch_bounds__(256) void tree_keys_kernel(const double* __restrict__ F, int r, const int64_t* __restrict__ idx,
                                                        int64_t n, int64_t w, const int* __restrict__ best,
                                                        TreeKey* __restrict__ keys) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const int64_t node = i / w;
    const int64_t o = idx[i];
    const double v = F[o * r + best[node]];
    keys[i] = TreeKey{v, (node << SEG_SHIFT) | o};
}

__global__ __launch_bounds__(256) void tree_unpack_kernel(const TreeKey* __restrict__ keys, int64_t n,
                                                          int64_t* __restrict__ idx) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) idx[i] = keys[i].k & ((int64_t(1) << SEG_SHIFT) - 1);
}

}  // namespace

// perm_dev[i] = original index of the i-th point in leaf order.  n = leaf * 2^L, F_dev is n x r row-major.
// *bad_dev (an int the caller zeroed) is set when F holds a value that is not finite.
int build_cluster_tree(hipStream_t st, const double* F_dev, int64_t n, int r, int leaf, int64_t* perm_dev, int* bad_dev) {
    if (r < 1 || r > 128 || n < 1 || n >= (int64_t(1) << SEG_SHIFT)) return HSS_EINVAL;
    const unsigned nb = (unsigned)((n + 255) / 256);
    hipLaunchKernelGGL(tree_iota_kernel, dim3(nb), dim3(256), 0, st, perm_dev, n);
    HIP_TRY(hipGetLastError());
    if (n <= leaf) return HSS_OK;
    DevBuf partial, mean, best, keys_a, keys_b, tmp;
    const int64_t max_blocks = (n + TREE_CHUNK - 1) / TREE_CHUNK + n / (2 * (int64_t)leaf) + 1;
    HSS_TRY(partial.reserve(sizeof(double) * (size_t)max_blocks * r));
    HSS_TRY(mean.reserve(sizeof(double) * (size_t)(n / leaf) * r));
    HSS_TRY(best.reserve(sizeof(int) * (size_t)(n / leaf)));
    HSS_TRY(keys_a.reserve(sizeof(TreeKey) * (size_t)n));
    HSS_TRY(keys_b.reserve(sizeof(TreeKey) * (size_t)n));
    size_t tmp_bytes = 0;
    HIP_TRY(rocprim::merge_sort(nullptr, tmp_bytes, keys_a.as<TreeKey>(), keys_b.as<TreeKey>(), (size_t)n, TreeKeyLess(), st));
    HSS_TRY(tmp.reserve(std::max<size_t>(tmp_bytes, 16)));
    for (int64_t w = n; w > leaf; w /= 2) {
        const int64_t nodes = n / w;
        const int chunks = (int)((w + TREE_CHUNK - 1) / TREE_CHUNK);
        const unsigned grid = (unsigned)(nodes * chunks);
        hipLaunchKernelGGL((tree_partial_kernel<0>), dim3(grid), dim3(256), 0, st, F_dev, r, perm_dev, w, chunks,
                           (const double*)nullptr, partial.as<double>());
        hipLaunchKernelGGL(tree_mean_kernel, dim3((unsigned)nodes), dim3(128), 0, st, partial.as<double>(), r, chunks,
                           (double)w, mean.as<double>());
        hipLaunchKernelGGL((tree_partial_kernel<1>), dim3(grid), dim3(256), 0, st, F_dev, r, perm_dev, w, chunks,
                           mean.as<double>(), partial.as<double>());
        hipLaunchKernelGGL(tree_best_kernel, dim3((unsigned)nodes), dim3(128), 0, st, partial.as<double>(), r, chunks,
                           best.as<int>(), bad_dev);
        hipLaunchKernelGGL(tree_keys_kernel, dim3(nb), dim3(256), 0, st, F_dev, r, perm_dev, n, w, best.as<int>(),
                           keys_a.as<TreeKey>());
        HIP_TRY(hipGetLastError());
        HIP_TRY(rocprim::merge_sort(tmp.p, tmp_bytes, keys_a.as<TreeKey>(), keys_b.as<TreeKey>(), (size_t)n, TreeKeyLess(), st));
        hipLaunchKernelGGL(tree_unpack_kernel, dim3(nb), dim3(256), 0, st, keys_b.as<TreeKey>(), n, perm_dev);
        HIP_TRY(hipGetLastError());
    }
    HIP_TRY(hipStreamSynchronize(st));   // the work buffers above are released on return
    return HSS_OK;
}
