// Cluster tree by balanced coordinate bisection (the clustering/reordering preprocess the compression
// relies on, Sec. 1.2).  Host code: the tree is a prerequisite of the hot path, not part of it.
//
// Node rule: split coordinate = the one with the largest population variance over the node (ties ->
// lowest coordinate), points sorted by (coordinate value, original index), lower half to the left child.
#include "common.h"
#include <algorithm>
#include <thread>

namespace {

struct KeyIdx {
    double  v;
    int64_t i;
};

// Variance of every coordinate over the node in two row-major passes (mean, then squared deviations, both
// summed in the node's current point order), then a sort of (value, original index) pairs.
void split_node(const double* F, int r, int64_t* idx, int64_t cnt, std::vector<double>& mean, std::vector<double>& var,
                std::vector<KeyIdx>& keys) {
    mean.assign(r, 0.0);
    var.assign(r, 0.0);
    for (int64_t i = 0; i < cnt; ++i) {
        const double* f = F + idx[i] * r;
        for (int c = 0; c < r; ++c) mean[c] += f[c];
    }
    for (int c = 0; c < r; ++c) mean[c] /= (double)cnt;
    for (int64_t i = 0; i < cnt; ++i) {
        const double* f = F + idx[i] * r;
        for (int c = 0; c < r; ++c) {
            const double d = f[c] - mean[c];
            var[c] += d * d;
        }
    }
    int best = 0;
    double bestv = -1.0;
    for (int c = 0; c < r; ++c) {
        const double v = var[c] / (double)cnt;
        if (v > bestv) {
            bestv = v;
            best = c;
        }
    }
    keys.resize(cnt);
    for (int64_t i = 0; i < cnt; ++i) keys[i] = KeyIdx{F[idx[i] * r + best], idx[i]};
    std::sort(keys.begin(), keys.end(), [](const KeyIdx& a, const KeyIdx& b) {
        if (a.v != b.v) return a.v < b.v;
        return a.i < b.i;
    });
    for (int64_t i = 0; i < cnt; ++i) idx[i] = keys[i].i;
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
            std::vector<double> mean, var;
            std::vector<KeyIdx> keys;
            for (int64_t t = 0; t < nodes; ++t) split_node(F_host, r, perm + t * width, width, mean, var, keys);
        } else {
            const int nt = (int)std::min<int64_t>(nthreads, nodes);
            std::vector<std::thread> th;
            th.reserve(nt);
            for (int w = 0; w < nt; ++w)
                th.emplace_back([=]() {
                    std::vector<double> mean, var;
                    std::vector<KeyIdx> keys;
                    for (int64_t t = w; t < nodes; t += nt) split_node(F_host, r, perm + t * width, width, mean, var, keys);
                });
            for (auto& x : th) x.join();
        }
    }
    return HSS_OK;
}
