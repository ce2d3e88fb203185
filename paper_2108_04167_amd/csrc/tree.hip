// Cluster tree by balanced coordinate bisection (the clustering/reordering preprocess the compression
// relies on, Sec. 1.2).  Host code: the tree is a prerequisite of the hot path, not part of it.
//
// Node rule: split coordinate = the one with the largest population variance over the node (ties ->
// lowest coordinate), points sorted by (coordinate value, original index), lower half to the left child.
#include "common.h"
#include <algorithm>
#include <thread>

namespace {

void split_node(const double* F, int r, int64_t* idx, int64_t cnt) {
    int best = 0;
    double bestv = -1.0;
    for (int c = 0; c < r; ++c) {
        double mean = 0.0;
        for (int64_t i = 0; i < cnt; ++i) mean += F[idx[i] * r + c];
        mean /= (double)cnt;
        double var = 0.0;
        for (int64_t i = 0; i < cnt; ++i) {
            double d = F[idx[i] * r + c] - mean;
            var += d * d;
        }
        var /= (double)cnt;
        if (var > bestv) {
            bestv = var;
            best = c;
        }
    }
    const int c = best;
    std::sort(idx, idx + cnt, [F, r, c](int64_t a, int64_t b) {
        double va = F[a * r + c], vb = F[b * r + c];
        if (va != vb) return va < vb;
        return a < b;
    });
}

}  // namespace

// perm[i] = original index of the i-th point in leaf order.  n = leaf * 2^L.
int build_cluster_tree(const double* F_host, int64_t n, int r, int leaf, int64_t* perm) {
    for (int64_t i = 0; i < n; ++i) perm[i] = i;
    unsigned hw = std::thread::hardware_concurrency();
    int nthreads = (int)std::min<unsigned>(16, hw ? hw : 4);
    for (int64_t width = n; width > leaf; width /= 2) {
        const int64_t nodes = n / width;
        if (nodes == 1 || nthreads <= 1) {
            for (int64_t t = 0; t < nodes; ++t) split_node(F_host, r, perm + t * width, width);
        } else {
            const int nt = (int)std::min<int64_t>(nthreads, nodes);
            std::vector<std::thread> th;
            th.reserve(nt);
            for (int w = 0; w < nt; ++w)
                th.emplace_back([=]() {
                    for (int64_t t = w; t < nodes; t += nt) split_node(F_host, r, perm + t * width, width);
                });
            for (auto& x : th) x.join();
        }
    }
    return HSS_OK;
}
