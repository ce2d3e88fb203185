/*
 * hss_svm.h -- C ABI of the shifted-kernel-solve path of the ADMM + HSS nonlinear-SVM trainer
 * (Cipolla & Gondzio, "Training very large scale nonlinear SVMs using ADMM coupled with HSS
 * kernel approximations").
 *
 * The library runs on one AMD gfx950 GPU.  It trains
 *
 *        min_x  1/2 x^T Y K Y x - e^T x     s.t.  y^T x = 0,  0 <= x <= C            (eq. 1)
 *
 * with the Gaussian kernel K_ij = exp(-||f_i - f_j||^2 / (2 h^2)) (Sec. 1.1 / Sec. 3.3), following
 * Algorithm 3: HSS compression of K, shift by beta*I, ULV factorization, then closed-form ADMM
 * iterations (Algorithm 2) that each apply (K~ + beta I)^{-1} once.  What is cached follows Sec. 3.2:
 * the compression depends only on (F, h), the factorization on (F, h, beta), an ADMM run on
 * (F, h, beta, C).
 *
 * Conventions
 *   - "dev" pointers are device (HBM) addresses valid on the GPU that was current at hss_create;
 *     "host" pointers are ordinary host memory.  All floating point data is IEEE double.
 *   - F is point-major: the r features of point i are F[i*r .. i*r+r-1] (the paper's r x d matrix
 *     F_train stored column by column).  y holds exactly -1.0 or +1.0.
 *   - Every vector that crosses this boundary (rhs, x, z, mu, y, decision values) is in the
 *     caller's original point order.  The cluster-tree permutation is internal.
 *   - The caller owns every buffer it passes.  The library copies what it needs during the call,
 *     except F, which hss_compress copies into its own permuted storage as well: nothing of the
 *     caller's is retained after a call returns.
 *   - Work is enqueued on the HIP stream given to hss_create (borrowed, never destroyed).  Calls
 *     that return host scalars or need ranks on the host synchronise that stream; all others are
 *     asynchronous with respect to the host.
 *   - Return value: 0 = ok; < 0 = error, nothing useful was written; > 0 = bitwise OR of HSS_W*
 *     warnings, results were written.  No call aborts, throws, or prints.
 *   - A context is not thread-safe.  Calls on one context must not overlap.
 */
#ifndef HSS_SVM_H
#define HSS_SVM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hss_ctx hss_ctx;

/* errors */
#define HSS_OK            0
#define HSS_EINVAL       (-1)  /* bad argument: n, r, leaf, tol, h, beta, C out of range; null pointer              */
#define HSS_ESTATE       (-2)  /* call out of order: solve before factor, factor before compress, ...            */
#define HSS_ENOMEM       (-3)  /* device or host allocation failed                                                */
#define HSS_EHIP         (-4)  /* a HIP runtime call failed                                                       */
#define HSS_EUNSUPPORTED (-5)  /* size outside what the kernels are built for (see hss_compress)                 */
/* warnings (bit mask) */
#define HSS_WRANK      1   /* some node hit the rank cap: the requested tolerance is not guaranteed               */
#define HSS_WPIVOT     2   /* a tiny pivot was met while factoring: K~ + beta I is close to singular               */
#define HSS_WNOMARGIN  4   /* the margin set {j : 0 < z_j < C} is empty: bias returned as 0                        */
#define HSS_WSHIFT     8   /* the definiteness guard added delta > 0 to the diagonal of K~ (see hss_compress)      */

const char* hss_strerror(int code);

/* Create / destroy a context.  hip_stream: a hipStream_t (0 = the null stream); borrowed.
 * Device memory: a context owns its tree, generators, factors and work space.  Device blocks that a call releases
 * (the work space of a compression or factorization, the state of the previous compression) are kept by the
 * context, up to 16 GiB, and handed to later allocations of about the same size, so that repeated calls with the
 * same problem shape allocate next to nothing; blocks that two compressions in a row did not use are freed; when an
 * allocation fails in any context of the process, the kept blocks of every context are freed before it is tried
 * again; hss_destroy frees everything, after which nothing the library allocated for the context remains.
 * One context is used by one thread at a time (different contexts may be used by different threads). */
int  hss_create(hss_ctx** out, void* hip_stream);
void hss_destroy(hss_ctx* ctx);

/* Options (hss_set_i64 unless marked f64); set before hss_compress unless stated otherwise.
 *
 * Sampling and truncation (end of Sec. 3.2: randomized sampling with oversampling, every block truncated to the
 * tolerance; Sec. 3.1 first bullet: neighbour-based sampling)
 *   "sample_width" s     number of sample columns (default 128; padded with zero columns to a multiple of 128 inside)
 *   "oversample"   p     rank cap is s - p unless "max_rank" is set (default s/2: with ranks that hit the cap a small
 *                        p over-fits the sample and the nested bases amplify the error level by level)
 *   "max_rank"           explicit rank cap per node (default 0 = s - p)
 *   "seed"               seed of the counter-based generator (Omega, random projection directions; default 0)
 *   "abs_tol" (f64)      absolute pivot threshold of the interpolative decompositions (default 1e-8)
 *   "adaptive_start" s0  > 0: adaptive sample width.  The decompositions of a tree level first see the leading s0
 *                        columns of the sample; while a node of the level is cut by the sample's rank cap (w - p at
 *                        width w, p = "oversample", default w/2) rather than by the tolerance, and columns are left,
 *                        "adaptive_step" more columns of Omega are sampled (for all rows, and carried up through the
 *                        finished levels) and the cut nodes -- only those -- are decomposed again.  "sample_width"
 *                        (or the width of a caller's Omega) is then the LARGEST width, and the final rank cap is
 *                        min("max_rank", s - p(s)).  s0, the step and s must be multiples of 128.  Default 0: off, all
 *                        s columns are sampled at once.
 *   "adaptive_step"      columns added per widening (default 128)
 *   "sampling"           0 (default): random sample S = K Omega.  1: neighbour-based, the paper's own compressor: the
 *                        sample of a node's block row is K(rows, N) with N the "sample_width" closest distinct
 *                        approximate nearest neighbours of the node's row points that lie outside the node -- entries
 *                        of K itself, no product with a random matrix and no O(n^2) work.  Ignored by
 *                        hss_compress_with_samples; the adaptive width does not apply; n < 2^31.
 *   "ann_neighbours" k   neighbours per point, 1 .. 64 (default 64)
 *   "ann_trees"          search trees (default 3): tree 0 = the cells of the cluster-tree order, the others random
 *                        projection trees (directions uniform in (-1,1)^r from Philox4x32-10 keyed by "seed"); with a
 *                        single tree no search leaves a cell and nodes above the cell size get no column at all
 *   "ann_cell"           points per cell, searched exhaustively (default 512): the cells are the nodes of the deepest
 *                        tree level whose nodes all hold at least that many points (the root if none does)
 *
 * Cluster tree (the clustering preprocess of Sec. 1.1 / 1.2; shape: see hss_compress)
 *   "clustering"         0 (default): a node is split at the median of the coordinate of largest variance.
 *                        1: data-driven -- along the line between the two centres of a 2-means pass over the node
 *                        (started from the point farthest from the node's mean and the point farthest from that
 *                        one), at the median of the projections.  The rule is free of summation order (centres from
 *                        exact fixed-point sums, the rest per point); n < 2^24.
 *   "clustering_iterations"  Lloyd steps of that pass, 0 .. 64 (default 2)
 *
 * Definiteness
 *   "psd_guard"          1 (default): after compression estimate lambda_min(K~) (Lanczos on the HSS mat-vec until the
 *                        smallest Ritz value settles, at most 512 steps) and, if negative, add
 *                        delta = 1.1*|lambda_min| to the diagonal so that the approximate problem (eq. 8) stays
 *                        convex, as Algorithm 3 presupposes; 0: off
 *
 * Factorization, solve, iteration (may be set any time before the call they affect)
 *   "merge_top"          1 (default): the ULV solve replaces the levels from the root down to a cut level by one
 *                        product with the inverse of the reduced matrix at the cut (chosen at factorization time so
 *                        that a solve takes the least modelled time; at most 4096 rows); 0: every level is a launch
 *                        of its own.  Takes effect at the next hss_ulv_factor.
 *   "cache_basis"        1 (default): the parts of the ULV factorization that depend on the generators only -- the
 *                        orthogonal change of basis of every node, the reduced bases, the parents' off-diagonal
 *                        blocks -- are kept from the first factorization of a compression and reused by later ones
 *                        with another beta (Sec. 3.2: what is computed once is reused across the grid); the factors
 *                        are bit-identical either way.  0: recomputed every time.
 *   "graph"              1: admm_svm_train records two iterations (all launches of two ULV solves and two vector
 *                        updates) into a HIP graph and replays it, on a stream of the library's own that is ordered
 *                        after / before the context's stream by events; 0 (default): every launch is issued eagerly
 *                        on the context's stream.  The iterates are the same either way; the replay measured 3 - 35 %
 *                        slower per iteration than eager launches on gfx950.
 *   "block_cache_mib"    how many MiB of released device blocks the context keeps for later allocations of the same
 *                        size (default 16384; see hss_create).  0: keeps nothing -- every release is a hipFree, every
 *                        reservation a hipMalloc.  Setting the option frees what is kept at that moment.  Results do
 *                        not depend on it.
 * Unknown keys and values out of range return HSS_EINVAL. */
int hss_set_i64(hss_ctx* ctx, const char* key, int64_t v);
int hss_set_f64(hss_ctx* ctx, const char* key, double v);

/* S = K(F,F) * Omega without forming K (the randomized range sampling the compression is built on,
 * end of Sec. 3.2).  F (dev, n x r), Omega (dev, n x s row-major), S_out (dev, n x s row-major), rows in
 * the order of F.  Stand-alone: needs no prior call and leaves the context's compressed matrix alone.
 * 1 <= r <= 384, s >= 1 (more than 112 features after padding to a multiple of 28: through row stripes of the kernel
 * matrix in HBM instead of the fused kernel, see hss_compress). */
int hss_kernel_sample(hss_ctx* ctx, const double* F_dev, int64_t n, int32_t r, double h,
                      const double* Omega_dev, int32_t s, double* S_out_dev);

/* hss_kernel_sample for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, same result as
 * hss_kernel_sample, but the padded work copies live in a fixed 12.1 MB device array inside the library
 * (one per GPU, held until the process ends) and the call makes no hipMalloc / hipFree and does not
 * synchronise: it is asynchronous on the context's stream.  Limits: n <= 4096, r <= 96, s <= 128;
 * larger sizes return HSS_EUNSUPPORTED and write nothing.  All calls on one GPU share the array: calls
 * that overlap in time on one GPU (other streams, other threads, other contexts) race, and S_out of a call
 * is final only when its stream has reached the end of that call.  The array's device address is looked up
 * when the first context is created on a GPU (or, failing that, by the first call on that GPU). */
int hss_kernel_sample_noalloc(hss_ctx* ctx, const double* F_dev, int64_t n, int32_t r, double h,
                              const double* Omega_dev, int32_t s, double* S_out_dev);

/* HSS compression of K(F,F) (Algorithm 3, first line): cluster tree (balanced bisection; option "clustering"),
 * sampling of the off-diagonal block rows (S = K Omega, or the neighbour-based sample; option "sampling"),
 * interpolative decompositions level by level.  F (dev, n x r), y (dev, n).  Any n >= 1; `leaf` = the largest leaf
 * size, 2 <= leaf <= 1024; 1 <= r <= 384, h > 0, 0 < tol <= 10
 * (tol/10 is the relative truncation threshold below; tol = 10 keeps one pivot per block, the loosest setting of the
 * paper's Table 1: relative 1, absolute 0.1 through "abs_tol").
 * Shape of the tree: depth L = the smallest one with ceil(n / 2^L) <= leaf; a node of p points gives the lower
 * ceil(p/2) of them (in the order of its split) to the left child and the rest to the right one.  All leaves are on
 * level L and hold floor or ceil of n / 2^L points (n = leaf * 2^L: exactly `leaf` each).
 * The kernel products work on the points minus their feature means (the kernel of Sec. 1.1 sees differences only;
 * points far from the origin would otherwise lose digits in ||f_i||^2 + ||f_j||^2 - 2 f_i . f_j).
 * Up to 112 features (after padding to a multiple of 28) the products with K run in the fused Gram + exp + contraction
 * kernels and K is never stored; wider data goes through row stripes of K in HBM (batched GEMM for the Gram stripe,
 * elementwise exp, batched GEMM with Omega; a work buffer of at most 8 GB), at about half the rate.  Pivots of each decomposition are kept while
 * |R_jj| > max(tol/10 * |R_00|, abs_tol), up to the rank cap.  Rank cap <= 512 and s <= 2048 (s <= 1024 for
 * tol < 3e-5), EUNSUPPORTED beyond.
 * Drops any previous compression and factorization held by the context.
 * hss_compress draws Omega itself (Philox4x32-10 + Box-Muller, option "seed");
 * hss_compress_with_samples takes Omega (dev, n x s row-major, rows in the order of F) from the caller. */
int hss_compress(hss_ctx* ctx, const double* F_dev, const double* y_dev, int64_t n, int32_t r,
                 double h, int32_t leaf, double tol);
int hss_compress_with_samples(hss_ctx* ctx, const double* F_dev, const double* y_dev, int64_t n, int32_t r,
                              double h, int32_t leaf, double tol, const double* Omega_dev, int32_t s);

/* Achieved compression error, estimated on nprobe (1..128) Gaussian probe vectors z_j drawn by the library's
 * counter-based generator from `seed`:  sqrt( sum_j ||K~ z_j - K z_j||^2 / sum_j ||K z_j||^2 ), an estimate of
 * ||K~ - K||_F / ||K||_F (the quantity the tolerance of Sec. 3.2 / eq. (9) speaks of), with K z_j from the exact
 * kernel (one pass of the fused kernel product: its 16-column form up to 16 probes, 128-column blocks of the sampling
 * kernel beyond) and K~ without the guard's shift.
 * rel_err_out (host).  Needs a compressed context.  Synchronous. */
int hss_error_estimate(hss_ctx* ctx, int32_t nprobe, uint64_t seed, double* rel_err_out);

/* ULV factorization of K~ + beta I (Algorithm 3, lines 2-3).  beta > 0.  May be called again with another
 * beta without recompressing; replaces the previous factors. */
int hss_ulv_factor(hss_ctx* ctx, double beta);

/* rhs <- (K~ + beta I)^{-1} rhs, in place.  rhs (dev, n x nrhs, column-major: each right-hand side is
 * a contiguous n-vector).  nrhs >= 1; up to four right-hand sides share one pass over the factors. */
int hss_ulv_solve(hss_ctx* ctx, double* rhs_inout_dev, int32_t nrhs);

/* y_out <- K~ x (with the guard's diagonal shift included).  x, y_out (dev, n); may not alias. */
int hss_matvec(hss_ctx* ctx, const double* x_dev, double* y_out_dev);

/* ADMM (Algorithm 2 with the precomputation of Algorithm 3), maxit iterations from x = z = mu = 0, then
 * the averaged bias of eq. (7) with the sign that satisfies the margin condition
 * (b = mean over M of y_j - (K~ Y z)_j).  If beta differs from the factored beta the library
 * re-factors first.  x_out, z_out, mu_out (dev, n each; any may be null).  bias_out, n_margin_out
 * (host; may be null).  The model is z (Algorithm 3 uses z for the bias and the labels). */
int admm_svm_train(hss_ctx* ctx, double C, double beta, int32_t maxit,
                   double* x_out_dev, double* z_out_dev, double* mu_out_dev,
                   double* bias_out_host, int64_t* n_margin_out_host);

/* The same for nC box bounds C_list[0..nC) (host) and one beta: the hyper-parameter sweep the caching of
 * Sec. 3.2 is meant for (compression once per h, factorization once per beta, then one ADMM run per C).
 * The runs are independent and share the factorization, w = Y K_beta^{-1} e and w1; they advance in lockstep,
 * up to four at a time as interleaved right-hand sides of one ULV sweep, so the factors are read once per
 * iteration for four runs.  Every run's iterates equal those of admm_svm_train with that C.
 * x_out, z_out, mu_out (dev, nC x n, run j at offset j*n; any may be null); bias_out, n_margin_out
 * (host, nC entries; may be null).  Returns the OR of the runs' warnings. */
int admm_svm_train_multi(hss_ctx* ctx, const double* C_list, int32_t nC, double beta, int32_t maxit,
                         double* x_out_dev, double* z_out_dev, double* mu_out_dev,
                         double* bias_out, int64_t* n_margin_out);

/* dec_j = sum_i y_i z_i K(f_i, g_j) + bias with the exact kernel (label loop of Algorithm 3).
 * G (dev, n_test x r), z (dev, n), dec_out (dev, n_test). */
int svm_decision(hss_ctx* ctx, const double* G_dev, int64_t n_test, const double* z_dev, double bias,
                 double* dec_out_dev);

/* dst[0..n) = src[0..n): a plain streaming copy (16-byte accesses) on the context's stream, with exactly
 * 8n bytes read and 8n written.  It is the measurement reference of this library: the bandwidth a trivial
 * kernel reaches on the device at hand, and the known traffic that turns raw memory-counter readings into
 * bytes (the roofline of the ULV solve, the operation of Sec. 2.1.1 that every iteration repeats, is quoted
 * against both).  src, dst (dev, 16-byte aligned, not overlapping), n even and >= 2.  Asynchronous. */
int hss_stream_copy(hss_ctx* ctx, const double* src_dev, double* dst_dev, int64_t n);

typedef struct hss_stats_t {
    int64_t n, r, leaf, levels;        /* levels = L (leaves are level L, root level 0)                    */
    int64_t sample_width, rank_cap;
    int64_t rank_max, rank_sum;        /* over all non-root nodes                                           */
    int64_t nodes_at_cap;              /* nodes whose rank hit the cap                                      */
    int64_t generator_bytes;           /* D, U, B as stored                                                 */
    int64_t factor_bytes;              /* bytes of the dense operators one solve reads (up-sweep, root, down-sweep) */
    int64_t factor_bytes_compact;      /* the same sweeps with the factors counted in compact form: per node
                                          m k (reflectors) + (m-k)^2 (LU of D_ee) + k (m-k) (D_re), read twice     */
    double  sample_flops;              /* 2 n^2 (s + r) of the last sampling                                */
    double  delta;                     /* diagonal shift added by the definiteness guard                    */
    double  beta;                      /* factored beta, or -1                                              */
    double  t_tree, t_sample, t_levels, t_guard, t_factor;   /* seconds, last call of each phase            */
    double  t_sample_kernel;           /* seconds of the K*Omega kernel alone (HIP events on the stream)      */
    int32_t warnings;                  /* OR of HSS_W* seen since the last compress                         */
    int32_t reserved;
    int64_t sample_width_used;         /* columns of the sample the decompositions ended up using (adaptive width) */
    int64_t nodes_redone;              /* node decompositions repeated after the sample was widened              */
} hss_stats_t;
int hss_stats(hss_ctx* ctx, hss_stats_t* out_host);

/* Export of the generators to host memory (the seam the parity tests use to run the oracle on the
 * same compressed matrix).  Nodes are in heap order: root 0, children of t are 2t+1, 2t+2, leaves last.
 *   perm   int64[n]           perm[i] = original index of the i-th point in cluster-tree order
 *   sizes  int32[nnodes]      node size m_t (leaf size at leaves, k_a + k_b above)
 *   ranks  int32[nnodes]      k_t (0 at the root)
 *   D      double[sum m_t^2 over the leaves, at most n*leaf]  leaf diagonal blocks (m_t x m_t row-major, one after
 *                             the other, left to right), WITHOUT the guard's shift
 *   U      double[sum m_t k_t]      row-major (m_t x k_t) per non-root node, heap order
 *   J      int32[sum k_t]           skeleton rows of each node (local row indices), heap order
 *   B      double[sum k_a k_b]      row-major (k_a x k_b) per inner node t with children a, b, heap order
 * hss_export_sizes fills nnodes, u_len, j_len, b_len (host int64 each); hss_export fills the arrays
 * (host) and *delta_out (host): the represented matrix is the HSS matrix of (D, U, B) plus delta I. */
int hss_export_sizes(hss_ctx* ctx, int64_t* nnodes, int64_t* u_len, int64_t* j_len, int64_t* b_len);
int hss_export(hss_ctx* ctx, int64_t* perm, int32_t* sizes, int32_t* ranks, double* D, double* U,
               int32_t* J, double* B, double* delta_out);

/* The neighbour lists of the last neighbour-based compression ("sampling" = 1), for tests and inspection:
 * *k_out (host) = neighbours per point; idx_out (host, int32[n * k]) and dist_out (host, double[n * k]), either
 * may be null: entry j of point i (points in cluster-tree order, i.e. point i is perm[i] of hss_export) is the
 * cluster-tree index of its j-th neighbour and the squared distance to it, ascending by (distance, index), -1 /
 * +infinity where fewer than k were found.  HSS_ESTATE without such a compression.  Synchronous. */
int hss_export_neighbours(hss_ctx* ctx, int32_t* k_out, int32_t* idx_out, double* dist_out);

/* The inverse of hss_export: puts the context into the compressed state from generators in HOST memory
 * (same arrays, same layout and node order as hss_export writes), for the points F_dev (n x r) and labels
 * y_dev in DEVICE memory and the kernel width h.  Nothing is sampled or decomposed and the definiteness
 * guard does not run: the represented matrix is the HSS matrix of (D, U, B) plus delta I with the caller's
 * delta >= 0 (Sec. 3.2: the compressed matrix depends on (F, h) only, so it can be computed once and kept).
 * The arrays are copied; the caller keeps ownership.  Checked on the host: perm is a permutation of 0..n-1;
 * sizes/ranks describe the tree of hss_compress for this n and `leaf` (leaf sizes as stated there), inner size = sum
 * of the children's ranks, 1 <= rank <= size below the root and rank 0 at the root; every J lists distinct rows of its node and
 * U is interpolative on them (row J_j of U_t is exactly the j-th unit vector); labels are +-1.  Violations return HSS_EINVAL, ranks above 512 HSS_EUNSUPPORTED; the context is then not
 * compressed.  Returns 0 or HSS_WSHIFT (delta > 0).  Synchronous. */
int hss_import(hss_ctx* ctx, const double* F_dev, const double* y_dev, int64_t n, int32_t r, double h, int32_t leaf,
               const int64_t* perm, const int32_t* sizes, const int32_t* ranks, const double* D, const double* U,
               const int32_t* J, const double* B, double delta);

#ifdef __cplusplus
}
#endif
#endif /* HSS_SVM_H */
