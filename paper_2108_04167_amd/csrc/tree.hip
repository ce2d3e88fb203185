// Cluster trees by balanced bisection (the clustering/reordering preprocess the compression relies on,
// Sec. 1.1 last paragraph / Sec. 1.2), built on the device level by level: along a coordinate axis (default) or
// along the line between the centres of a 2-means pass (data-driven, second half of this file).
//
// Node rule: split coordinate = the lowest one whose population variance over the node is at least
// (1 - 1e-9) times the largest (variances that differ only by the rounding of their sums count as tied),
// points sorted by (coordinate value, original index), lower half to the left child.
//
// One level = five small kernels (two-pass variance with per-chunk partial sums recombined in a fixed
// order, so the result does not depend on scheduling) and one device-wide merge sort of 16-byte keys
// (node, value, original index): nodes are contiguous ranges of the index array (offsets in `noff`; shape of the
// tree: see tree_depth), so sorting the whole array by that key sorts every node in place.
#include "common.h"
#include "ctx.h"
#include <rocprim/device/device_merge_sort.hpp>
#include <algorithm>

namespace {

constexpr int TREE_CHUNK = 256;   // points per partial sum
constexpr int SEG_SHIFT = 40;     // key word = (node << 40) | original index
constexpr int TREE_RMAX = 512;    // most coordinates (one thread each in the per-node kernels)

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
// (F[idx][c] - mean[node][c])^2 (MODE 1).  The coordinates are taken in groups of at most 256; within a group of rc
// coordinates thread t works on coordinate t % rc of every (256 / rc)-th point.
template <int MODE>
__global__ __launch_bounds__(256) void tree_partial_kernel(const double* __restrict__ F, int r,
                                                           const int64_t* __restrict__ idx,
                                                           const int64_t* __restrict__ noff, int chunks,
                                                           const double* __restrict__ mean, double* __restrict__ partial) {
    const int64_t node = blockIdx.x / chunks;
    const int ch = blockIdx.x % chunks;
    __shared__ double red[256];
    const int64_t lo = noff[node] + (int64_t)ch * TREE_CHUNK, end = noff[node + 1];   // lo >= end: an empty chunk
    const int64_t hi = lo + TREE_CHUNK < end ? lo + TREE_CHUNK : end;
    for (int c0 = 0; c0 < r; c0 += 256) {
        const int rc = r - c0 < 256 ? r - c0 : 256;
        const int npl = 256 / rc;
        const int c = c0 + threadIdx.x % rc, pl = threadIdx.x / rc;
        double acc = 0.0;
        if (pl < npl) {
            const double m = MODE ? mean[node * r + c] : 0.0;
            for (int64_t i = lo + pl; i < hi; i += npl) {
                const double d = F[idx[i] * r + c] - m;
                acc += MODE ? d * d : d;
            }
        }
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

// mean[node][c] = (sum of the node's partials, in chunk order) / (points of the node)
__global__ __launch_bounds__(TREE_RMAX) void tree_mean_kernel(const double* __restrict__ partial, int r, int chunks,
                                                        const int64_t* __restrict__ noff, double* __restrict__ mean) {
    const int c = threadIdx.x;
    if (c >= r) return;
    const double* p = partial + (size_t)blockIdx.x * chunks * r + c;
    double s = 0.0;
    for (int ch = 0; ch < chunks; ++ch) s += p[(size_t)ch * r];
    mean[(size_t)blockIdx.x * r + c] = s / (double)(noff[blockIdx.x + 1] - noff[blockIdx.x]);
}

// best[node] = lowest coordinate whose summed squared deviation reaches (1 - 1e-9) x the largest.  A sum that is
// not finite (a NaN or an infinity among the features, or squares that overflow) sets *bad: at the root this
// covers every entry of F.
__global__ __launch_bounds__(TREE_RMAX) void tree_best_kernel(const double* __restrict__ partial, int r, int chunks,
                                                        int* __restrict__ best, int* __restrict__ bad) {
    __shared__ double var[TREE_RMAX];
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
                                                        int64_t n, const int64_t* __restrict__ noff, int64_t nodes,
                                                        const int* __restrict__ best, TreeKey* __restrict__ keys) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const int64_t node = segment_of(noff, nodes, i);
    const int64_t o = idx[i];
    const double v = F[o * r + best[node]];
    keys[i] = TreeKey{v, (node << SEG_SHIFT) | o};
}

__global__ __launch_bounds__(256) void tree_unpack_kernel(const TreeKey* __restrict__ keys, int64_t n,
                                                          int64_t* __restrict__ idx) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) idx[i] = keys[i].k & ((int64_t(1) << SEG_SHIFT) - 1);
}

// ---------------------------------------------------------------------------------------------------------
// Data-driven rule: a node is split along the line between the two centres of a 2-means pass over its points.
// Nothing in it depends on a summation order: centres are means from EXACT integer sums of the features in fixed
// point (rint(value * scale), |.| <= 2^38, added with integer atomics), every other quantity is computed per point
// with each operation rounded on its own (no fused multiply-add) and only compared or sorted across points, ties to
// the lowest original index.
//   c = mean of the node; a = farthest point from c; b = farthest point from a; (ca, cb) = (a, b);
//   `iters` times: A = {dist2(., ca) <= dist2(., cb)}, B = the rest; unless one is empty (ca, cb) = (mean A, mean B);
//   sort by (sum_f (x_f - ca_f)(cb_f - ca_f), original index), lower half to the left child.
typedef unsigned long long u64;

// From here on no multiply is fused with an add: the per-point quantities below must round exactly like the
// same operations written one after the other anywhere else.
#pragma clang fp contract(off)

__device__ __forceinline__ double dist2_seq(const double* __restrict__ x, const double* __restrict__ c, int r) {
    double acc = 0.0;
    for (int f = 0; f < r; ++f) {
        const double diff = x[f] - c[f];
        const double sq = diff * diff;
        acc = acc + sq;
    }
    return acc;
}

// *amax_bits = max over all entries of the bit pattern of |F| (order-preserving for non-negative doubles; an
// infinity or a NaN gives a pattern at or above that of infinity)
__global__ __launch_bounds__(256) void tm_amax_kernel(const double* __restrict__ F, int64_t count, u64* amax_bits) {
    u64 m = 0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)gridDim.x * 256) {
        const u64 b = (u64)__double_as_longlong(fabs(F[i]));
        m = b > m ? b : m;
    }
    for (int off = 32; off > 0; off >>= 1) {
        const u64 o = __shfl_xor(m, off, 64);
        m = o > m ? o : m;
    }
    if ((threadIdx.x & 63) == 0) atomicMax(amax_bits, m);
}

// qsum[(node*2 + side)*r + c] += sum of rint(F * scale) over the chunk's points on that side; cnt[node*2 + side]
// += their number.  side == nullptr: every point counts as side 0.  Coordinates in groups of at most 256, as in
// tree_partial_kernel; the integer sums are exact, so the grouping does not show in the result.
__global__ __launch_bounds__(256) void tm_sum_kernel(const double* __restrict__ F, int r, const int64_t* __restrict__ idx,
                                                     const int64_t* __restrict__ noff, int chunks, double scale,
                                                     const unsigned char* __restrict__ side, u64* __restrict__ qsum,
                                                     u64* __restrict__ cnt) {
    const int64_t node = blockIdx.x / chunks;
    const int ch = blockIdx.x % chunks;
    __shared__ long long red[2][256];
    const int64_t lo = noff[node] + (int64_t)ch * TREE_CHUNK, end = noff[node + 1];   // lo >= end: an empty chunk
    const int64_t hi = lo + TREE_CHUNK < end ? lo + TREE_CHUNK : end;
    for (int c0 = 0; c0 < r; c0 += 256) {
        const int rc = r - c0 < 256 ? r - c0 : 256;
        const int npl = 256 / rc;
        const int c = c0 + threadIdx.x % rc, pl = threadIdx.x / rc;
        long long acc0 = 0, acc1 = 0, n0 = 0, n1 = 0;
        if (pl < npl) {
            for (int64_t i = lo + pl; i < hi; i += npl) {
                const long long q = (long long)rint(F[idx[i] * r + c] * scale);
                const int sd = side ? side[i] : 0;
                if (sd) { acc1 += q; ++n1; }
                else { acc0 += q; ++n0; }
            }
        }
        red[0][threadIdx.x] = acc0;
        red[1][threadIdx.x] = acc1;
        __syncthreads();
        if (threadIdx.x < rc) {
            long long s0 = 0, s1 = 0;
            for (int p = 0; p < npl; ++p) {
                s0 += red[0][p * rc + threadIdx.x];
                s1 += red[1][p * rc + threadIdx.x];
            }
            atomicAdd(qsum + (size_t)(node * 2) * r + c0 + threadIdx.x, (u64)s0);
            atomicAdd(qsum + (size_t)(node * 2 + 1) * r + c0 + threadIdx.x, (u64)s1);
        }
        __syncthreads();
        if (c0 == 0) {
            // the number of points per side: coordinate 0's threads saw every point of the chunk once
            red[0][threadIdx.x] = (c == 0 && pl < npl) ? n0 : 0;
            red[1][threadIdx.x] = (c == 0 && pl < npl) ? n1 : 0;
            __syncthreads();
            if (threadIdx.x == 0) {
                long long s0 = 0, s1 = 0;
                for (int p = 0; p < npl; ++p) {
                    s0 += red[0][p * rc];
                    s1 += red[1][p * rc];
                }
                atomicAdd(cnt + node * 2, (u64)s0);
                atomicAdd(cnt + node * 2 + 1, (u64)s1);
            }
            __syncthreads();
        }
    }
}

// ctr[(node*2 + side)*r + c] = ((double)sum / (double)count) / scale.  both == 0: side 0 only (the node's mean);
// both == 1: both sides, and only when neither is empty (an empty side leaves the centres as they are).
__global__ __launch_bounds__(TREE_RMAX) void tm_centre_kernel(const u64* __restrict__ qsum, const u64* __restrict__ cnt, int r,
                                                        double scale, int both, double* __restrict__ ctr) {
    const int64_t node = blockIdx.x;
    const int c = threadIdx.x;
    if (c >= r) return;
    const long long n0 = (long long)cnt[node * 2], n1 = (long long)cnt[node * 2 + 1];
    if (both && (n0 == 0 || n1 == 0)) return;
    ctr[(size_t)(node * 2) * r + c] = ((double)(long long)qsum[(size_t)(node * 2) * r + c] / (double)n0) / scale;
    if (both) ctr[(size_t)(node * 2 + 1) * r + c] = ((double)(long long)qsum[(size_t)(node * 2 + 1) * r + c] / (double)n1) / scale;
}

// d2[i] = dist2(point i, centre 0 of its node); dmax[node] = max of their bit patterns
__global__ __launch_bounds__(256) void tm_far1_kernel(const double* __restrict__ F, int r, const int64_t* __restrict__ idx,
                                                      int64_t n, const int64_t* __restrict__ noff, int64_t nodes,
                                                      const double* __restrict__ ctr, double* __restrict__ d2,
                                                      u64* __restrict__ dmax) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const int64_t node = segment_of(noff, nodes, i);
    const double v = dist2_seq(F + idx[i] * r, ctr + (size_t)(node * 2) * r, r);
    d2[i] = v;
    atomicMax(dmax + node, (u64)__double_as_longlong(v));
}
// amin[node] = lowest original index among the points that reach the maximum
__global__ __launch_bounds__(256) void tm_far2_kernel(const int64_t* __restrict__ idx, int64_t n,
                                                      const int64_t* __restrict__ noff, int64_t nodes,
                                                      const double* __restrict__ d2, const u64* __restrict__ dmax,
                                                      u64* __restrict__ amin) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const int64_t node = segment_of(noff, nodes, i);
    if ((u64)__double_as_longlong(d2[i]) == dmax[node]) atomicMin(amin + node, (u64)idx[i]);
}
// centre `which` of every node = the point amin[node]
__global__ __launch_bounds__(TREE_RMAX) void tm_take_point_kernel(const double* __restrict__ F, int r, const u64* __restrict__ amin,
                                                            int which, double* __restrict__ ctr) {
    const int64_t node = blockIdx.x;
    const int c = threadIdx.x;
    if (c < r) ctr[(size_t)(node * 2 + which) * r + c] = F[(int64_t)amin[node] * r + c];
}
// side[i] = 0 if dist2(point, ca) <= dist2(point, cb) else 1
__global__ __launch_bounds__(256) void tm_assign_kernel(const double* __restrict__ F, int r, const int64_t* __restrict__ idx,
                                                        int64_t n, const int64_t* __restrict__ noff, int64_t nodes,
                                                        const double* __restrict__ ctr, unsigned char* __restrict__ side) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const int64_t node = segment_of(noff, nodes, i);
    const double* x = F + idx[i] * r;
    const double da = dist2_seq(x, ctr + (size_t)(node * 2) * r, r);
    const double db = dist2_seq(x, ctr + (size_t)(node * 2 + 1) * r, r);
    side[i] = da <= db ? 0 : 1;
}
// sort key of point i: (node, sum_f (x_f - ca_f) (cb_f - ca_f), original index)
__global__ __launch_bounds__(256) void tm_keys_kernel(const double* __restrict__ F, int r, const int64_t* __restrict__ idx,
                                                      int64_t n, const int64_t* __restrict__ noff, int64_t nodes,
                                                      const double* __restrict__ ctr, TreeKey* __restrict__ keys) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const int64_t node = segment_of(noff, nodes, i);
    const int64_t o = idx[i];
    const double* x = F + o * r;
    const double* ca = ctr + (size_t)(node * 2) * r;
    const double* cb = ca + r;
    double p = 0.0;
    for (int f = 0; f < r; ++f) {
        const double d = cb[f] - ca[f];
        const double t = (x[f] - ca[f]) * d;
        p = p + t;
    }
    keys[i] = TreeKey{p, (node << SEG_SHIFT) | o};
}

// Node offsets of the levels 0 .. L-1 of the tree over n points, level after level, in device memory (level l at
// d + start[l], 2^l + 1 entries).  The host copy lives as long as the object: the upload is asynchronous.
struct LevelOffsets {
    DevBuf d;
    std::vector<int64_t> h;
    std::vector<size_t> start;
    const int64_t* level(int l) const { return d.as<int64_t>() + start[l]; }
};
int upload_level_offsets(hipStream_t st, int64_t n, int L, LevelOffsets& lo) {
    lo.h.clear();
    lo.start.assign(L, 0);
    for (int l = 0; l < L; ++l) {
        const std::vector<int64_t> off = level_offsets(n, l);
        lo.start[l] = lo.h.size();
        lo.h.insert(lo.h.end(), off.begin(), off.end());
    }
    HSS_TRY(lo.d.reserve(sizeof(int64_t) * std::max<size_t>(lo.h.size(), 1)));
    if (!lo.h.empty()) HIP_TRY(hipMemcpyAsync(lo.d.p, lo.h.data(), sizeof(int64_t) * lo.h.size(), hipMemcpyHostToDevice, st));
    return HSS_OK;
}

}  // namespace

int build_cluster_tree_2means(hipStream_t st, const double* F_dev, int64_t n, int r, int leaf, int iters,
                              int64_t* perm_dev, int* bad_dev) {
    if (r < 1 || r > TREE_RMAX || n < 1 || n >= (int64_t(1) << 24) || iters < 0) return HSS_EINVAL;
    const unsigned nb = (unsigned)((n + 255) / 256);
    hipLaunchKernelGGL(tree_iota_kernel, dim3(nb), dim3(256), 0, st, perm_dev, n);
    HIP_TRY(hipGetLastError());
    DevBuf amaxd;
    HSS_TRY(amaxd.reserve(sizeof(u64)));
    HIP_TRY(hipMemsetAsync(amaxd.p, 0, sizeof(u64), st));
    hipLaunchKernelGGL(tm_amax_kernel, dim3(1024), dim3(256), 0, st, F_dev, n * r, amaxd.as<u64>());
    HIP_TRY(hipGetLastError());
    u64 abits = 0;
    HIP_TRY(hipMemcpyAsync(&abits, amaxd.p, sizeof(u64), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    double amax;
    memcpy(&amax, &abits, sizeof(double));
    if (!(amax <= 1.7976931348623157e308)) {       // an infinity or a NaN among the features
        const int one = 1;
        HIP_TRY(hipMemcpyAsync(bad_dev, &one, sizeof(int), hipMemcpyHostToDevice, st));
        HIP_TRY(hipStreamSynchronize(st));
        return HSS_OK;
    }
    const int L = tree_depth(n, leaf);
    if (L == 0) return HSS_OK;
    int e = 0;
    if (amax > 0.0) (void)frexp(amax, &e);          // amax < 2^e
    const double scale = ldexp(1.0, 38 - e);
    const int64_t maxnodes = int64_t(1) << (L - 1);
    LevelOffsets lo;
    HSS_TRY(upload_level_offsets(st, n, L, lo));
    DevBuf qsum, cnt, ctr, dmax, amin, d2, side, keys_a, keys_b, tmp;
    HSS_TRY(qsum.reserve(sizeof(u64) * (size_t)maxnodes * 2 * r));
    HSS_TRY(cnt.reserve(sizeof(u64) * (size_t)maxnodes * 2));
    HSS_TRY(ctr.reserve(sizeof(double) * (size_t)maxnodes * 2 * r));
    HSS_TRY(dmax.reserve(sizeof(u64) * (size_t)maxnodes));
    HSS_TRY(amin.reserve(sizeof(u64) * (size_t)maxnodes));
    HSS_TRY(d2.reserve(sizeof(double) * (size_t)n));
    HSS_TRY(side.reserve((size_t)n));
    HSS_TRY(keys_a.reserve(sizeof(TreeKey) * (size_t)n));
    HSS_TRY(keys_b.reserve(sizeof(TreeKey) * (size_t)n));
    size_t tmp_bytes = 0;
    HIP_TRY(rocprim::merge_sort(nullptr, tmp_bytes, keys_a.as<TreeKey>(), keys_b.as<TreeKey>(), (size_t)n, TreeKeyLess(), st));
    HSS_TRY(tmp.reserve(std::max<size_t>(tmp_bytes, 16)));
    for (int l = 0; l < L; ++l) {
        const int64_t nodes = int64_t(1) << l;
        const int64_t w = (n + nodes - 1) / nodes;                   // the largest node of the level
        const int chunks = (int)((w + TREE_CHUNK - 1) / TREE_CHUNK);
        const unsigned grid = (unsigned)(nodes * chunks);
        const int64_t* noff = lo.level(l);
        auto sums = [&](const unsigned char* sd, int both) -> int {
            HIP_TRY(hipMemsetAsync(qsum.p, 0, sizeof(u64) * (size_t)nodes * 2 * r, st));
            HIP_TRY(hipMemsetAsync(cnt.p, 0, sizeof(u64) * (size_t)nodes * 2, st));
            hipLaunchKernelGGL(tm_sum_kernel, dim3(grid), dim3(256), 0, st, F_dev, r, perm_dev, noff, chunks, scale, sd,
                               qsum.as<u64>(), cnt.as<u64>());
            hipLaunchKernelGGL(tm_centre_kernel, dim3((unsigned)nodes), dim3(TREE_RMAX), 0, st, qsum.as<u64>(), cnt.as<u64>(), r,
                               scale, both, ctr.as<double>());
            HIP_TRY(hipGetLastError());
            return HSS_OK;
        };
        auto farthest_into = [&](int which) -> int {      // centre `which` = the point farthest from centre 0
            HIP_TRY(hipMemsetAsync(dmax.p, 0, sizeof(u64) * (size_t)nodes, st));
            HIP_TRY(hipMemsetAsync(amin.p, 0xff, sizeof(u64) * (size_t)nodes, st));
            hipLaunchKernelGGL(tm_far1_kernel, dim3(nb), dim3(256), 0, st, F_dev, r, perm_dev, n, noff, nodes,
                               ctr.as<double>(), d2.as<double>(), dmax.as<u64>());
            hipLaunchKernelGGL(tm_far2_kernel, dim3(nb), dim3(256), 0, st, perm_dev, n, noff, nodes, d2.as<double>(),
                               dmax.as<u64>(), amin.as<u64>());
            hipLaunchKernelGGL(tm_take_point_kernel, dim3((unsigned)nodes), dim3(TREE_RMAX), 0, st, F_dev, r, amin.as<u64>(), which,
                               ctr.as<double>());
            HIP_TRY(hipGetLastError());
            return HSS_OK;
        };
        HSS_TRY(sums(nullptr, 0));          // centre 0 = mean of the node
        HSS_TRY(farthest_into(0));          // centre 0 = a
        HSS_TRY(farthest_into(1));          // centre 1 = b
        for (int it = 0; it < iters; ++it) {
            hipLaunchKernelGGL(tm_assign_kernel, dim3(nb), dim3(256), 0, st, F_dev, r, perm_dev, n, noff, nodes,
                               ctr.as<double>(), side.as<unsigned char>());
            HSS_TRY(sums(side.as<unsigned char>(), 1));
        }
        hipLaunchKernelGGL(tm_keys_kernel, dim3(nb), dim3(256), 0, st, F_dev, r, perm_dev, n, noff, nodes,
                           ctr.as<double>(), keys_a.as<TreeKey>());
        HIP_TRY(hipGetLastError());
        HIP_TRY(rocprim::merge_sort(tmp.p, tmp_bytes, keys_a.as<TreeKey>(), keys_b.as<TreeKey>(), (size_t)n, TreeKeyLess(), st));
        hipLaunchKernelGGL(tree_unpack_kernel, dim3(nb), dim3(256), 0, st, keys_b.as<TreeKey>(), n, perm_dev);
        HIP_TRY(hipGetLastError());
    }
    HIP_TRY(hipStreamSynchronize(st));   // the work buffers above are released on return
    return HSS_OK;
}

// perm_dev[i] = original index of the i-th point in leaf order.  F_dev is n x r row-major; any n >= 1.
// *bad_dev (an int the caller zeroed) is set when F holds a value that is not finite.
int build_cluster_tree(hipStream_t st, const double* F_dev, int64_t n, int r, int leaf, int64_t* perm_dev, int* bad_dev) {
    if (r < 1 || r > TREE_RMAX || n < 1 || n >= (int64_t(1) << SEG_SHIFT)) return HSS_EINVAL;
    const unsigned nb = (unsigned)((n + 255) / 256);
    hipLaunchKernelGGL(tree_iota_kernel, dim3(nb), dim3(256), 0, st, perm_dev, n);
    HIP_TRY(hipGetLastError());
    const int L = tree_depth(n, leaf);
    if (L == 0) return HSS_OK;
    DevBuf partial, mean, best, keys_a, keys_b, tmp;
    const int64_t maxnodes = int64_t(1) << (L - 1);
    const int64_t max_blocks = (n + TREE_CHUNK - 1) / TREE_CHUNK + 2 * maxnodes;   // sum over nodes of ceil(size / chunk)
    LevelOffsets lo;
    HSS_TRY(upload_level_offsets(st, n, L, lo));
    HSS_TRY(partial.reserve(sizeof(double) * (size_t)max_blocks * r));
    HSS_TRY(mean.reserve(sizeof(double) * (size_t)maxnodes * r));
    HSS_TRY(best.reserve(sizeof(int) * (size_t)maxnodes));
    HSS_TRY(keys_a.reserve(sizeof(TreeKey) * (size_t)n));
    HSS_TRY(keys_b.reserve(sizeof(TreeKey) * (size_t)n));
    size_t tmp_bytes = 0;
    HIP_TRY(rocprim::merge_sort(nullptr, tmp_bytes, keys_a.as<TreeKey>(), keys_b.as<TreeKey>(), (size_t)n, TreeKeyLess(), st));
    HSS_TRY(tmp.reserve(std::max<size_t>(tmp_bytes, 16)));
    for (int l = 0; l < L; ++l) {
        const int64_t nodes = int64_t(1) << l;
        const int64_t w = (n + nodes - 1) / nodes;                   // the largest node of the level
        const int chunks = (int)((w + TREE_CHUNK - 1) / TREE_CHUNK);
        const unsigned grid = (unsigned)(nodes * chunks);
        const int64_t* noff = lo.level(l);
        hipLaunchKernelGGL((tree_partial_kernel<0>), dim3(grid), dim3(256), 0, st, F_dev, r, perm_dev, noff, chunks,
                           (const double*)nullptr, partial.as<double>());
        hipLaunchKernelGGL(tree_mean_kernel, dim3((unsigned)nodes), dim3(TREE_RMAX), 0, st, partial.as<double>(), r, chunks,
                           noff, mean.as<double>());
        hipLaunchKernelGGL((tree_partial_kernel<1>), dim3(grid), dim3(256), 0, st, F_dev, r, perm_dev, noff, chunks,
                           mean.as<double>(), partial.as<double>());
        hipLaunchKernelGGL(tree_best_kernel, dim3((unsigned)nodes), dim3(TREE_RMAX), 0, st, partial.as<double>(), r, chunks,
                           best.as<int>(), bad_dev);
        hipLaunchKernelGGL(tree_keys_kernel, dim3(nb), dim3(256), 0, st, F_dev, r, perm_dev, n, noff, nodes,
                           best.as<int>(), keys_a.as<TreeKey>());
        HIP_TRY(hipGetLastError());
        HIP_TRY(rocprim::merge_sort(tmp.p, tmp_bytes, keys_a.as<TreeKey>(), keys_b.as<TreeKey>(), (size_t)n, TreeKeyLess(), st));
        hipLaunchKernelGGL(tree_unpack_kernel, dim3(nb), dim3(256), 0, st, keys_b.as<TreeKey>(), n, perm_dev);
        HIP_TRY(hipGetLastError());
    }
    HIP_TRY(hipStreamSynchronize(st));   // the work buffers above are released on return
    return HSS_OK;
}
