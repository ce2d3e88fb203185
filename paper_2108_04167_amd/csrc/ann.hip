// Neighbour-based sampling for the HSS construction (the paper's own compressor, Sec. 3.1 first bullet: the columns
// of the dominating approximate nearest neighbours of a node's points stand for its off-diagonal block row, instead
// of a random sample K Omega).
//
// 1. Approximate nearest neighbours of every point (points in cluster-tree order):
//      tree 0 = the cells of the cluster-tree order itself (the nodes of one level of the cluster tree),
//      trees 1 .. T-1 = random projection trees of the same shape (a set is split at the median of the projections
//      on a random direction, the lower ceil(p/2) of its p points to the left, down to the cell level; one merge
//      sort of (node, projection, point) keys per level);
//      inside every cell an exact search: one wavefront per point keeps the point's list (k <= 64 entries, one per
//      lane, ascending by (distance, index)), computes the distances to 64 candidates at a time (features read
//      coalesced from a transposed copy), drops the point itself and entries already listed, sorts the 64 by a
//      bitonic network over the lanes and merges them into the list.  The lists of the trees merge by running the
//      search of every tree on the lists the previous trees left.
//    Distances and projections are accumulated feature by feature with every operation rounded on its own (no fused
//    multiply-add), so the lists are a function of the cells alone.
// 2. Sample columns of the nodes of a tree level: every neighbour-list entry of every row point of a node that lies
//    outside the node's index range is a candidate scored by its distance; distinct candidates (smallest distance
//    kept), the s smallest by (distance, index): two device-wide merge sorts of 16-byte keys per level.
#include "ctx.h"
#include <rocprim/device/device_merge_sort.hpp>
#include <algorithm>
#include <cmath>

namespace {

#pragma clang fp contract(off)

constexpr double ANN_INF = __builtin_huge_val();   // +infinity
constexpr int SEG_SHIFT = 40;
constexpr int ANN_RMAX = 512;                      // most features (a point's row is staged in LDS per wavefront)

struct PKey {          // projection-tree sort key
    double  v;
    int64_t k;         // (node << 40) | point
};
struct PKeyLess {
    __host__ __device__ bool operator()(const PKey& a, const PKey& b) const {
        const int64_t sa = a.k >> SEG_SHIFT, sb = b.k >> SEG_SHIFT;
        if (sa != sb) return sa < sb;
        if (a.v != b.v) return a.v < b.v;
        return a.k < b.k;
    }
};

struct CKey {          // candidate column of a node
    double  d;         // squared distance to the closest row point that lists it
    int32_t node;      // INT32_MAX: not a candidate
    int32_t cand;
};
struct CKeyByCand {    // (node, candidate, distance)
    __host__ __device__ bool operator()(const CKey& a, const CKey& b) const {
        if (a.node != b.node) return a.node < b.node;
        if (a.cand != b.cand) return a.cand < b.cand;
        return a.d < b.d;
    }
};
struct CKeyByDist {    // (node, distance, candidate)
    __host__ __device__ bool operator()(const CKey& a, const CKey& b) const {
        if (a.node != b.node) return a.node < b.node;
        if (a.d != b.d) return a.d < b.d;
        return a.cand < b.cand;
    }
};

__global__ __launch_bounds__(256) void iota_kernel(int64_t* idx, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) idx[i] = i;
}

__global__ __launch_bounds__(256) void list_clear_kernel(int32_t* __restrict__ idx, double* __restrict__ dist, int64_t count) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < count) {
        idx[i] = -1;
        dist[i] = ANN_INF;
    }
}

// Ft[f * n + pos] = feature f of point order[pos] of the cluster-tree order, i.e. F[perm[order[pos]] * r + f]: the
// caller's values as given (the centred copy differs from them in the last bits, and the lists are defined on these)
__global__ __launch_bounds__(256) void transpose_gather_kernel(const double* __restrict__ F, int r,
                                                               const int64_t* __restrict__ perm,
                                                               const int64_t* __restrict__ order, int64_t n,
                                                               double* __restrict__ Ft) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n * r) return;
    const int f = (int)(i / n);
    const int64_t pos = i - (int64_t)f * n;
    Ft[i] = F[perm[order[pos]] * r + f];
}

// key of position i: (node, sum_f x_f dir[node][f], point)
__global__ __launch_bounds__(256) void proj_keys_kernel(const double* __restrict__ F, int r,
                                                        const int64_t* __restrict__ perm,
                                                        const int64_t* __restrict__ order, int64_t n,
                                                        const int64_t* __restrict__ noff, int64_t nodes,
                                                        const double* __restrict__ dirs, PKey* __restrict__ keys) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const int64_t node = segment_of(noff, nodes, i);
    const int64_t o = order[i];
    const double* x = F + perm[o] * r;
    const double* d = dirs + node * r;
    double p = 0.0;
    for (int f = 0; f < r; ++f) {
        const double t = x[f] * d[f];
        p = p + t;
    }
    keys[i] = PKey{p, (node << SEG_SHIFT) | o};
}
__global__ __launch_bounds__(256) void proj_unpack_kernel(const PKey* __restrict__ keys, int64_t n, int64_t* __restrict__ order) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) order[i] = keys[i].k & ((int64_t(1) << SEG_SHIFT) - 1);
}

__device__ __forceinline__ bool key_less(double da, int ia, double db, int ib) {
    return da < db || (da == db && ia < ib);
}

// Exact search inside the cells of one tree, merged into the lists (see the file header).
__global__ __launch_bounds__(256) void knn_cell_kernel(const double* __restrict__ Ft, int r, int64_t n,
                                                       const int64_t* __restrict__ order,
                                                       const int64_t* __restrict__ celloff, int64_t ncells, int k,
                                                       int32_t* __restrict__ nbr_idx, double* __restrict__ nbr_dist) {
    __shared__ double xs[4][ANN_RMAX];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int64_t pos = (int64_t)blockIdx.x * 4 + wave;
    const bool live = pos < n;
    if (!live) pos = n - 1;                       // keeps the wavefront in step with the barrier below; nothing is stored
    for (int f = lane; f < r; f += 64) xs[wave][f] = Ft[(size_t)f * n + pos];
    __syncthreads();
    const int64_t pid = order[pos];
    double ld = lane < k ? nbr_dist[pid * k + lane] : ANN_INF;
    int li = lane < k ? nbr_idx[pid * k + lane] : -1;
    if (li < 0) { ld = ANN_INF; li = 0x7fffffff; }
    const int64_t mycell = segment_of(celloff, ncells, pos);
    const int64_t c0 = celloff[mycell], c1 = celloff[mycell + 1];
    for (int64_t base = c0; base < c1; base += 64) {
        const int64_t cp = base + lane;
        bool valid = cp < c1 && cp != pos;
        double d = ANN_INF;
        int ci = 0x7fffffff;
        if (valid) {
            ci = (int)order[cp];
            double acc = 0.0;
            for (int f = 0; f < r; ++f) {
                const double diff = xs[wave][f] - Ft[(size_t)f * n + cp];
                const double sq = diff * diff;
                acc = acc + sq;
            }
            d = acc;
        }
        // already listed?  lower bound of (d, ci) in the sorted list by bisection over the lanes
        int lo = 0, hi = 64;
#pragma unroll
        for (int s = 0; s < 7; ++s) {             // 64 -> 32 -> ... -> 1 -> 0 positions left
            const bool go = lo < hi;
            const int mid = go ? (lo + hi) >> 1 : 0;
            const double md = __shfl(ld, mid, 64);
            const int mi = __shfl(li, mid, 64);
            const bool less = key_less(md, mi, d, ci);
            lo = (go && less) ? mid + 1 : lo;
            hi = (go && !less) ? mid : hi;
        }
        {
            const int at = lo < 64 ? lo : 63;
            const double md = __shfl(ld, at, 64);
            const int mi = __shfl(li, at, 64);
            if (lo < 64 && md == d && mi == ci) valid = false;
        }
        if (!valid) { d = ANN_INF; ci = 0x7fffffff; }
        // bitonic sort of the 64 candidates, ascending
#pragma unroll
        for (int k2 = 2; k2 <= 64; k2 <<= 1) {
#pragma unroll
            for (int j = k2 >> 1; j > 0; j >>= 1) {
                const double pd = __shfl_xor(d, j, 64);
                const int pi = __shfl_xor(ci, j, 64);
                const bool up = (lane & k2) == 0 || k2 == 64;
                const bool lower = (lane & j) == 0;
                const bool take_min = up == lower;
                const bool p_less = key_less(pd, pi, d, ci);
                if (take_min ? p_less : !p_less) { d = pd; ci = pi; }
            }
        }
        // the 64 smallest of list + candidates: list[l] against candidates[63 - l], then a bitonic merge
        {
            const double rd = __shfl(d, 63 - lane, 64);
            const int ri = __shfl(ci, 63 - lane, 64);
            if (key_less(rd, ri, ld, li)) { ld = rd; li = ri; }
        }
#pragma unroll
        for (int j = 32; j > 0; j >>= 1) {
            const double pd = __shfl_xor(ld, j, 64);
            const int pi = __shfl_xor(li, j, 64);
            const bool lower = (lane & j) == 0;
            const bool p_less = key_less(pd, pi, ld, li);
            if (lower ? p_less : !p_less) { ld = pd; li = pi; }
        }
    }
    if (live && lane < k) {
        const bool real = ld < ANN_INF;
        nbr_idx[pid * k + lane] = real ? li : -1;
        nbr_dist[pid * k + lane] = real ? ld : ANN_INF;
    }
}

// Candidate entries of a level: entry (q, j) = neighbour j of the point behind row q of the level
__global__ __launch_bounds__(256) void cand_fill_kernel(const int64_t* __restrict__ rowpoint, const int32_t* __restrict__ rownode,
                                                        int64_t rows, int k, const int64_t* __restrict__ span,
                                                        const int32_t* __restrict__ nbr_idx, const double* __restrict__ nbr_dist,
                                                        CKey* __restrict__ keys) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= rows * k) return;
    const int64_t q = e / k;
    const int j = (int)(e - q * k);
    const int64_t pid = rowpoint ? rowpoint[q] : q;
    const int node = rownode[q];
    const int cand = nbr_idx[pid * k + j];
    const int64_t lo = span[node], hi = span[node + 1];     // the points under the node
    CKey key{ANN_INF, 0x7fffffff, 0x7fffffff};
    if (cand >= 0 && (cand < lo || cand >= hi)) key = CKey{nbr_dist[pid * k + j], node, cand};
    keys[e] = key;
}
// after the sort by (node, candidate, distance): every repeat of a (node, candidate) pair is dropped
__global__ __launch_bounds__(256) void cand_unique_kernel(const CKey* __restrict__ in, int64_t count, CKey* __restrict__ out) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= count) return;
    CKey key = in[e];
    if (e > 0 && key.node != 0x7fffffff) {
        const CKey prev = in[e - 1];
        if (prev.node == key.node && prev.cand == key.cand) key = CKey{ANN_INF, 0x7fffffff, 0x7fffffff};
    }
    out[e] = key;
}
// after the sort by (node, distance, candidate): first and one-past-last entry of every node
__global__ __launch_bounds__(256) void cand_segments_kernel(const CKey* __restrict__ keys, int64_t count,
                                                            int64_t* __restrict__ seg_lo, int64_t* __restrict__ seg_hi) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= count) return;
    const int node = keys[e].node;
    if (node == 0x7fffffff) return;
    if (e == 0 || keys[e - 1].node != node) seg_lo[node] = e;
    if (e + 1 == count || keys[e + 1].node != node) seg_hi[node] = e + 1;
}
// cols[node * s + j] = j-th candidate of the node (j < min(s, number of candidates)); ncols[node] = that minimum
__global__ __launch_bounds__(256) void cand_take_kernel(const CKey* __restrict__ keys, const int64_t* __restrict__ seg_lo,
                                                        const int64_t* __restrict__ seg_hi, int s, int64_t* __restrict__ cols,
                                                        int32_t* __restrict__ ncols) {
    const int node = blockIdx.x;
    const int64_t lo = seg_lo[node], cnt = seg_hi[node] - lo;
    const int take = (int)(cnt < s ? cnt : s);
    if (threadIdx.x == 0) ncols[node] = take;
    for (int j = threadIdx.x; j < take; j += 256) cols[(size_t)node * s + j] = keys[lo + j].cand;
}

// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11) on the host, from the published round function and constants.
void philox_host(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1, uint32_t (&out)[4]) {
    const uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
    for (int round = 0; round < 10; ++round) {
        const uint64_t p0 = (uint64_t)M0 * c0, p1 = (uint64_t)M1 * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n1 = (uint32_t)p1, n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1,
                       n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += W0; k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

}  // namespace

// Component f of the random direction of node `node` at level `level` of projection tree `tree`: uniform in (-1, 1),
// from the Philox block with counter (f / 2, node, level, tree) and key (seed low word, seed high word ^ 0xA511E9B3):
// its first / second 53-bit uniform for even / odd f, as ((double)bits + 0.5) * 2^-52 - 1.
double ann_direction_component(uint64_t seed, int tree, int level, int64_t node, int f) {
    uint32_t o[4];
    philox_host((uint32_t)(f / 2), (uint32_t)node, (uint32_t)level, (uint32_t)tree, (uint32_t)seed,
                (uint32_t)(seed >> 32) ^ 0xA511E9B3u, o);
    const uint64_t bits = (f & 1) ? (((uint64_t)o[2] << 32 | o[3]) >> 11) : (((uint64_t)o[0] << 32 | o[1]) >> 11);
    return ((double)bits + 0.5) * (1.0 / 4503599627370496.0) - 1.0;
}

// Neighbour lists of the n points of the context (cluster-tree order) into c->nbr_idx / c->nbr_dist (n x k).
int ann_search(hss_ctx* c, const double* F, int k, int cell, int trees, uint64_t seed) {
    hipStream_t st = c->stream;
    const int64_t n = c->n;
    const int r = c->r;
    const int64_t* perm = c->perm.as<int64_t>();
    if (k < 1 || k > 64 || trees < 1 || cell < 2 || n >= (int64_t(1) << 31) || r > ANN_RMAX) return HSS_EINVAL;
    // cells: the nodes of the deepest level of the cluster tree whose nodes all hold at least `cell` points (the
    // root if none does); every projection tree is split down to the same level
    int lc = c->L;
    while (lc > 0 && (n >> lc) < cell) --lc;
    const int64_t ncells = int64_t(1) << lc;
    // offsets of the nodes of levels 0 .. lc, level after level (level l at start[l])
    std::vector<int64_t> offs;
    std::vector<size_t> start(lc + 1);
    for (int l = 0; l <= lc; ++l) {
        const std::vector<int64_t> o = level_offsets(n, l);
        start[l] = offs.size();
        offs.insert(offs.end(), o.begin(), o.end());
    }
    DevBuf offd;
    HSS_TRY(offd.reserve(sizeof(int64_t) * offs.size()));
    HIP_TRY(hipMemcpyAsync(offd.p, offs.data(), sizeof(int64_t) * offs.size(), hipMemcpyHostToDevice, st));
    HSS_TRY(c->nbr_idx.reserve(sizeof(int32_t) * (size_t)n * k));
    HSS_TRY(c->nbr_dist.reserve(sizeof(double) * (size_t)n * k));
    c->ann_k = k;
    DevBuf order, Ft, keys_a, keys_b, tmp, dirs;
    HSS_TRY(order.reserve(sizeof(int64_t) * (size_t)n));
    HSS_TRY(Ft.reserve(sizeof(double) * (size_t)n * r));
    const unsigned nb = (unsigned)((n + 255) / 256);
    const int64_t cnt = n * k;
    hipLaunchKernelGGL(list_clear_kernel, dim3((unsigned)((cnt + 255) / 256)), dim3(256), 0, st, c->nbr_idx.as<int32_t>(),
                       c->nbr_dist.as<double>(), cnt);
    HIP_TRY(hipGetLastError());
    size_t tmp_bytes = 0;
    if (trees > 1 && lc > 0) {
        HSS_TRY(keys_a.reserve(sizeof(PKey) * (size_t)n));
        HSS_TRY(keys_b.reserve(sizeof(PKey) * (size_t)n));
        HIP_TRY(rocprim::merge_sort(nullptr, tmp_bytes, keys_a.as<PKey>(), keys_b.as<PKey>(), (size_t)n, PKeyLess(), st));
        HSS_TRY(tmp.reserve(std::max<size_t>(tmp_bytes, 16)));
        HSS_TRY(dirs.reserve(sizeof(double) * (size_t)ncells * r));
    }
    std::vector<double> dh;
    for (int t = 0; t < trees; ++t) {
        hipLaunchKernelGGL(iota_kernel, dim3(nb), dim3(256), 0, st, order.as<int64_t>(), n);
        HIP_TRY(hipGetLastError());
        if (t > 0) {
            if (lc == 0) break;                       // one cell holds everything: further trees add nothing
            for (int level = 0; level < lc; ++level) {
                const int64_t nodes = int64_t(1) << level;
                dh.resize((size_t)nodes * r);
                for (int64_t node = 0; node < nodes; ++node)
                    for (int f = 0; f < r; ++f) dh[(size_t)node * r + f] = ann_direction_component(seed, t, level, node, f);
                HIP_TRY(hipMemcpyAsync(dirs.p, dh.data(), sizeof(double) * dh.size(), hipMemcpyHostToDevice, st));
                hipLaunchKernelGGL(proj_keys_kernel, dim3(nb), dim3(256), 0, st, F, r, perm,
                                   order.as<int64_t>(), n, offd.as<int64_t>() + start[level], nodes, dirs.as<double>(),
                                   keys_a.as<PKey>());
                HIP_TRY(hipGetLastError());
                HIP_TRY(rocprim::merge_sort(tmp.p, tmp_bytes, keys_a.as<PKey>(), keys_b.as<PKey>(), (size_t)n, PKeyLess(), st));
                hipLaunchKernelGGL(proj_unpack_kernel, dim3(nb), dim3(256), 0, st, keys_b.as<PKey>(), n, order.as<int64_t>());
                HIP_TRY(hipGetLastError());
                HIP_TRY(hipStreamSynchronize(st));    // dh is reused by the next level
            }
        }
        const int64_t tot = n * r;
        hipLaunchKernelGGL(transpose_gather_kernel, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, st, F, r, perm,
                           order.as<int64_t>(), n, Ft.as<double>());
        hipLaunchKernelGGL(knn_cell_kernel, dim3((unsigned)((n + 3) / 4)), dim3(256), 0, st, Ft.as<double>(), r, n,
                           order.as<int64_t>(), offd.as<int64_t>() + start[lc], ncells, k, c->nbr_idx.as<int32_t>(),
                           c->nbr_dist.as<double>());
        HIP_TRY(hipGetLastError());
    }
    HIP_TRY(hipStreamSynchronize(st));                // the work buffers are released on return
    return HSS_OK;
}

// Sample columns of the N nodes of tree level `level`.  rowpoint: point behind each of the level's `rows` rows (null:
// row q is point q, the leaf level); rownode_host: node of each row.  cols_dev: N x s point indices; ncols_host: how
// many of them each node has.
int ann_select_columns(hss_ctx* c, AnnWork& wk, const int64_t* rowpoint, const std::vector<int32_t>& rownode_host,
                       int64_t rows, int N, int level, int s, int64_t* cols_dev, std::vector<int32_t>& ncols_host) {
    hipStream_t st = c->stream;
    const int k = c->ann_k;
    const int64_t count = rows * k;
    DevBuf &rn = wk.rn, &keys_a = wk.keys_a, &keys_b = wk.keys_b, &tmp = wk.tmp, &seg_lo = wk.seg_lo, &seg_hi = wk.seg_hi,
           &ncd = wk.ncd;      // grown on demand, reused by every level of a compression
    HSS_TRY(rn.reserve(sizeof(int32_t) * (size_t)rows));
    HSS_TRY(keys_a.reserve(sizeof(CKey) * (size_t)count));
    HSS_TRY(keys_b.reserve(sizeof(CKey) * (size_t)count));
    HSS_TRY(seg_lo.reserve(sizeof(int64_t) * (size_t)N));
    HSS_TRY(seg_hi.reserve(sizeof(int64_t) * (size_t)N));
    HSS_TRY(ncd.reserve(sizeof(int32_t) * (size_t)N));
    const std::vector<int64_t> span_host = level_offsets(c->n, level);   // points under node t: span[t] .. span[t+1]-1
    HSS_TRY(wk.span.reserve(sizeof(int64_t) * span_host.size()));
    HIP_TRY(hipMemcpyAsync(wk.span.p, span_host.data(), sizeof(int64_t) * span_host.size(), hipMemcpyHostToDevice, st));
    size_t tb1 = 0, tb2 = 0;
    HIP_TRY(rocprim::merge_sort(nullptr, tb1, keys_a.as<CKey>(), keys_b.as<CKey>(), (size_t)count, CKeyByCand(), st));
    HIP_TRY(rocprim::merge_sort(nullptr, tb2, keys_a.as<CKey>(), keys_b.as<CKey>(), (size_t)count, CKeyByDist(), st));
    HSS_TRY(tmp.reserve(std::max<size_t>(std::max(tb1, tb2), 16)));
    HIP_TRY(hipMemcpyAsync(rn.p, rownode_host.data(), sizeof(int32_t) * (size_t)rows, hipMemcpyHostToDevice, st));
    const unsigned gb = (unsigned)((count + 255) / 256);
    hipLaunchKernelGGL(cand_fill_kernel, dim3(gb), dim3(256), 0, st, rowpoint, rn.as<int32_t>(), rows, k,
                       wk.span.as<int64_t>(), c->nbr_idx.as<int32_t>(), c->nbr_dist.as<double>(), keys_a.as<CKey>());
    HIP_TRY(hipGetLastError());
    HIP_TRY(rocprim::merge_sort(tmp.p, tb1, keys_a.as<CKey>(), keys_b.as<CKey>(), (size_t)count, CKeyByCand(), st));
    hipLaunchKernelGGL(cand_unique_kernel, dim3(gb), dim3(256), 0, st, keys_b.as<CKey>(), count, keys_a.as<CKey>());
    HIP_TRY(hipGetLastError());
    HIP_TRY(rocprim::merge_sort(tmp.p, tb2, keys_a.as<CKey>(), keys_b.as<CKey>(), (size_t)count, CKeyByDist(), st));
    HIP_TRY(hipMemsetAsync(seg_lo.p, 0, sizeof(int64_t) * (size_t)N, st));
    HIP_TRY(hipMemsetAsync(seg_hi.p, 0, sizeof(int64_t) * (size_t)N, st));
    hipLaunchKernelGGL(cand_segments_kernel, dim3(gb), dim3(256), 0, st, keys_b.as<CKey>(), count, seg_lo.as<int64_t>(),
                       seg_hi.as<int64_t>());
    hipLaunchKernelGGL(cand_take_kernel, dim3((unsigned)N), dim3(256), 0, st, keys_b.as<CKey>(), seg_lo.as<int64_t>(),
                       seg_hi.as<int64_t>(), s, cols_dev, ncd.as<int32_t>());
    HIP_TRY(hipGetLastError());
    ncols_host.resize(N);
    HIP_TRY(hipMemcpyAsync(ncols_host.data(), ncd.p, sizeof(int32_t) * (size_t)N, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));                // ncols_host is read by the caller right away
    return HSS_OK;
}
