// Internal declarations shared by the translation units of libhsssvm (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#include <mutex>
#include <vector>

#include "../../include/hss_svm.h"

#define HIP_TRY(expr)                                         \
    do {                                                      \
        hipError_t e__ = (expr);                              \
        if (e__ != hipSuccess) return HSS_EHIP;               \
    } while (0)

#define HSS_TRY(expr)                                         \
    do {                                                      \
        int rc__ = (expr);                                    \
        if (rc__ < 0) return rc__;                            \
    } while (0)

typedef double v4d __attribute__((ext_vector_type(4)));

static inline int64_t round_up(int64_t a, int64_t b) { return (a + b - 1) / b * b; }
// Feature count after zero padding: the sampling kernel issues its Gram k-steps (4 features each) in
// 7 equal groups per column block, so it wants a multiple of 28.
static inline int feature_pad(int r) { return (int)round_up(r, 28); }

// ---------------------------------------------------------------------------------------------
// Shape of the cluster tree for any number of points n and largest leaf size `leaf`: depth L = the smallest one
// with ceil(n / 2^L) <= leaf; a node of p points (a contiguous range of the tree order) gives its first ceil(p/2)
// points to the left child and the other floor(p/2) to the right one.  All leaves are on level L, their sizes
// differ by at most one, and n = leaf * 2^L gives leaves of exactly `leaf` points.
static inline int tree_depth(int64_t n, int leaf) {
    int L = 0;
    while (((n + (int64_t(1) << L) - 1) >> L) > leaf) ++L;
    return L;
}
// offsets (2^l + 1 of them) of the nodes of level l in the tree order
static inline std::vector<int64_t> level_offsets(int64_t n, int l) {
    std::vector<int64_t> off{0, n};
    for (int d = 0; d < l; ++d) {
        std::vector<int64_t> nxt;
        nxt.reserve(2 * off.size());
        nxt.push_back(0);
        for (size_t t = 0; t + 1 < off.size(); ++t) {
            nxt.push_back(off[t] + (off[t + 1] - off[t] + 1) / 2);
            nxt.push_back(off[t + 1]);
        }
        off.swap(nxt);
    }
    return off;
}
// the segment t with off[t] <= i < off[t+1] (off ascending, off[0] <= i < off[nseg])
__device__ __forceinline__ int64_t segment_of(const int64_t* __restrict__ off, int64_t nseg, int64_t i) {
    int64_t lo = 0, hi = nseg;
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if (off[mid] <= i) lo = mid;
        else hi = mid;
    }
    return lo;
}

// ---------------------------------------------------------------------------------------------
// Block cache of one context.  A compression and a factorization reserve a few hundred device buffers, and the next
// compression on the same context releases and reserves nearly all of them again at the same sizes; hipMalloc of
// a block of 16 MB and more costs 0.15 - 0.35 ms and hipFree of a gigabyte 0.3 - 3 ms, which added up to a tenth of
// a whole training run at n = 65 536.  While a call on a context is running (CacheScope), a DevBuf that releases
// its block hands it to the context's cache, and a reservation takes the smallest cached block that is large
// enough and at most a quarter larger.  All device work of a context is ordered on its one stream, so a block
// may change hands without the device-wide wait that hipFree implies.  The cache holds at most `cap` bytes,
// drops blocks that two compressions in a row did not use, and is emptied when the context is destroyed.  When an
// allocation fails anywhere in the process, the caches of ALL contexts are emptied before it is tried again (a
// cached block is idle by definition, and hipFree waits for whatever its context still has in flight), so what
// one context keeps can never be the reason another one runs out of memory.
struct BlockCache {
    struct Blk { void* p; size_t bytes; int epoch; };
    std::mutex mu;                       // a failed allocation of another context (another thread) may empty this one
    std::vector<Blk> blocks;
    size_t held = 0;
    int epoch = 0;
    size_t cap = size_t(16) << 30;       // option "block_cache_mib"; 0 keeps nothing
    struct Registry {
        std::mutex mu;
        std::vector<BlockCache*> all;
    };
    static Registry& registry() {
        static Registry* r = new Registry;      // never destroyed: contexts may outlive the library's static objects
        return *r;
    }
    BlockCache() {
        Registry& r = registry();
        std::lock_guard<std::mutex> g(r.mu);
        r.all.push_back(this);
    }
    BlockCache(const BlockCache&) = delete;
    BlockCache& operator=(const BlockCache&) = delete;
    ~BlockCache() {
        {
            Registry& r = registry();
            std::lock_guard<std::mutex> g(r.mu);
            for (size_t i = 0; i < r.all.size(); ++i)
                if (r.all[i] == this) {
                    r.all[i] = r.all.back();
                    r.all.pop_back();
                    break;
                }
        }
        flush();
    }
    void flush() {
        std::lock_guard<std::mutex> g(mu);
        for (const Blk& b : blocks) (void)hipFree(b.p);
        blocks.clear();
        held = 0;
    }
    void set_cap(size_t bytes) {
        {
            std::lock_guard<std::mutex> g(mu);
            cap = bytes;
        }
        flush();
    }
    // every cache of the process; returns whether anything was freed
    static bool flush_all() {
        Registry& r = registry();
        std::lock_guard<std::mutex> g(r.mu);
        bool any = false;
        for (BlockCache* c : r.all) {
            {
                std::lock_guard<std::mutex> gc(c->mu);
                any = any || !c->blocks.empty();
            }
            c->flush();
        }
        return any;
    }
    // a new compression starts: blocks that the last two did not take are freed
    void next_epoch() {
        std::lock_guard<std::mutex> g(mu);
        ++epoch;
        size_t w = 0;
        for (size_t i = 0; i < blocks.size(); ++i) {
            if (blocks[i].epoch + 2 <= epoch) {
                (void)hipFree(blocks[i].p);
                held -= blocks[i].bytes;
            } else {
                blocks[w++] = blocks[i];
            }
        }
        blocks.resize(w);
    }
    bool give(void* p, size_t bytes) {
        std::lock_guard<std::mutex> g(mu);
        if (bytes > cap || held + bytes > cap) return false;
        blocks.push_back(Blk{p, bytes, epoch});
        held += bytes;
        return true;
    }
    void* take(size_t nbytes, size_t* got) {
        std::lock_guard<std::mutex> g(mu);
        const size_t limit = nbytes + nbytes / 4 + (size_t(64) << 10);
        int best = -1;
        for (int i = 0; i < (int)blocks.size(); ++i)
            if (blocks[i].bytes >= nbytes && blocks[i].bytes <= limit && (best < 0 || blocks[i].bytes < blocks[best].bytes))
                best = i;
        if (best < 0) return nullptr;
        void* p = blocks[best].p;
        *got = blocks[best].bytes;
        held -= blocks[best].bytes;
        blocks[best] = blocks.back();
        blocks.pop_back();
        return p;
    }
};
// the cache of the context whose call is running on this thread (null outside such a call)
inline thread_local BlockCache* tl_block_cache = nullptr;
struct CacheScope {
    BlockCache* prev;
    explicit CacheScope(BlockCache* c) : prev(tl_block_cache) { tl_block_cache = c; }
    ~CacheScope() { tl_block_cache = prev; }
    CacheScope(const CacheScope&) = delete;
    CacheScope& operator=(const CacheScope&) = delete;
};

// ---------------------------------------------------------------------------------------------
// Device buffer with ownership.
struct DevBuf {
    void*  p = nullptr;
    size_t bytes = 0;
    DevBuf() = default;
    DevBuf(const DevBuf&) = delete;
    DevBuf& operator=(const DevBuf&) = delete;
    DevBuf(DevBuf&& o) noexcept : p(o.p), bytes(o.bytes) { o.p = nullptr; o.bytes = 0; }
    DevBuf& operator=(DevBuf&& o) noexcept {
        if (this != &o) {
            release();
            p = o.p; bytes = o.bytes;
            o.p = nullptr; o.bytes = 0;
        }
        return *this;
    }
    ~DevBuf() { release(); }
    void release() {
        if (p && !(tl_block_cache && tl_block_cache->give(p, bytes))) (void)hipFree(p);
        p = nullptr;
        bytes = 0;
    }
    // (re)allocate when the current block is too small; contents are not preserved
    int reserve(size_t nbytes) {
        if (nbytes <= bytes && p) return HSS_OK;
        release();
        if (nbytes == 0) nbytes = 8;
        if (tl_block_cache) {
            size_t got = 0;
            if (void* q = tl_block_cache->take(nbytes, &got)) {
                p = q;
                bytes = got;
                return HSS_OK;
            }
        }
        if (hipMalloc(&p, nbytes) != hipSuccess) {
            p = nullptr;
            (void)hipGetLastError();
            // give back what the caches of this process hold and try once more
            if (!BlockCache::flush_all()) return HSS_ENOMEM;
            if (hipMalloc(&p, nbytes) != hipSuccess) {
                p = nullptr;
                (void)hipGetLastError();
                return HSS_ENOMEM;
            }
        }
        bytes = nbytes;
        return HSS_OK;
    }
    template <class T> T* as() const { return reinterpret_cast<T*>(p); }
};

// ---------------------------------------------------------------------------------------------
// Upload arena for small descriptor tables: pinned host staging + device mirror.  push() copies
// a table into the staging area and enqueues an async H2D copy; the returned device pointer is
// valid for kernels enqueued afterwards on the same stream.  reset() may be called only after
// the stream has been synchronised.
struct DescArena {
    char*  h = nullptr;
    char*  d = nullptr;
    size_t cap = 0, used = 0;
    ~DescArena() { release(); }
    void release() {
        if (h) (void)hipHostFree(h);
        if (d) (void)hipFree(d);
        h = d = nullptr;
        cap = used = 0;
    }
    int init(size_t bytes) {
        release();
        if (hipHostMalloc((void**)&h, bytes, hipHostMallocDefault) != hipSuccess) return HSS_ENOMEM;
        if (hipMalloc((void**)&d, bytes) != hipSuccess) return HSS_ENOMEM;
        cap = bytes;
        used = 0;
        return HSS_OK;
    }
    void reset() { used = 0; }
    // returns device pointer or nullptr when full
    void* push(const void* src, size_t bytes, hipStream_t st) {
        size_t off = (used + 255) & ~size_t(255);
        if (off + bytes > cap) return nullptr;
        memcpy(h + off, src, bytes);
        if (hipMemcpyAsync(d + off, h + off, bytes, hipMemcpyHostToDevice, st) != hipSuccess) return nullptr;
        used = off + bytes;
        return d + off;
    }
};

// ---------------------------------------------------------------------------------------------
// Batched ragged GEMM on the FP64 matrix cores:  C = alpha * op(A) * op(B) + beta * C  per item.
// All matrices row-major.  op(A) is M x K, op(B) is K x N, C is M x N.  Items with M, N or K == 0
// are legal (K == 0 scales C by beta).
struct GemmItem {
    const double* A;
    const double* B;
    double*       C;
    int32_t M, N, K;
    int32_t lda, ldb, ldc;
};
int bgemm(hipStream_t st, const GemmItem* items_dev, int nitems, int maxM, int maxN, bool transA, bool transB,
          double alpha, double beta);

// ---------------------------------------------------------------------------------------------
// Sampling S = K(Fp,Fp) * Omega (fused Gram + exp + contraction on the matrix cores).
// Fp: n_pad x r_pad (zero padded), nu: n_pad squared norms, Om/S: n_pad x s_pad, n_pad % 256 == 0,
// r_pad % 28 == 0 (<= 112), s_pad % 128 == 0.
int sample_launch(hipStream_t st, const double* Fp, const double* nu, const double* Om, double* S,
                  int64_t n_pad, int r_pad, int s_pad, double h);
int sample_launch_rect(hipStream_t st, const double* Fr, const double* nur, int64_t nr_pad, const double* Fp,
                       const double* nu, int64_t n_pad, const double* Om, double* S, int r_pad, int s_pad, double h);
// The same for a window of `width` columns (a multiple of 128) of arrays with leading dimension ld.
int sample_launch_window(hipStream_t st, const double* Fr, const double* nur, int64_t nr_pad, const double* Fp,
                         const double* nu, int64_t n_pad, const double* Om, double* S, int r_pad, int width, int ld,
                         double h);
// The same product for any padded feature count: the fused kernel up to 112 features, row stripes of the kernel matrix
// in HBM beyond (sample_wide.hip; allocates its stripe and drains the stream)
int sample_wide_launch(hipStream_t st, const double* Fr, const double* nur, int64_t nr_pad, const double* Fp,
                       const double* nu, int64_t n_pad, const double* Om, double* S, int r_pad, int width, int ld,
                       double h);
int kernel_product_launch(hipStream_t st, const double* Fr, const double* nur, int64_t nr_pad, const double* Fp,
                          const double* nu, int64_t n_pad, const double* Om, double* S, int r_pad, int width, int ld,
                          double h);
constexpr int MAX_FEATURES = 384;        // r accepted by the compression (padded to 392)
// S (nr_pad x 16) = K(rows, cols) V for a block V (n_pad x 16) of at most 16 used columns (sample_narrow.hip); `work`
// is grown to hold partial results when the rows are few
int sample_narrow_launch(hipStream_t st, const double* Fr, const double* nur, int64_t nr_pad, const double* Fp,
                         const double* nu, int64_t n_pad, const double* V, double* S, int r_pad, double h, DevBuf& work);
int row_norms_launch(hipStream_t st, const double* Fp, double* nu, int64_t n_pad, int r_pad);
// Fp[i, :] = F[perm[i], :] zero padded to r_pad columns; rows >= n are zeroed.  perm == nullptr: identity.
int gather_pad_rows_launch(hipStream_t st, const double* F, const int64_t* perm, double* Fp, int64_t n, int64_t n_pad,
                           int r, int r_pad);
// Omega (n_pad x s_pad): standard normals for rows < n and columns < s, zeros elsewhere.
int omega_fill_launch(hipStream_t st, double* Om, int64_t n, int64_t n_pad, int s, int s_pad, uint64_t seed);
