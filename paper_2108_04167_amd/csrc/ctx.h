// The context behind the opaque hss_ctx handle: options, the cluster tree, the HSS generators, the ULV
// factors and the fixed work vectors of the solve / mat-vec / ADMM loop.
#pragma once
#include "common.h"
#include "dense.h"
#include "levels.h"
#include "rowid.h"
#include "solve.h"
#include "vec.h"
#include <new>
#include <string>

struct Level {
    int N = 0;                              // nodes at this level (2^l)
    std::vector<int> msz, rk;               // node sizes and ranks (rk = 0 at the root)
    std::vector<int64_t> moff, koff;        // prefix sums of msz, rk              [N+1]
    std::vector<int64_t> uoff, boff;        // prefix sums of msz*rk, k_a*k_b       [N+1]
    int maxm = 0, maxk = 0;
    DevBuf d_moff, d_koff, d_uoff;          // device copies of the prefix sums
    // generators
    DevBuf U;                               // (msz x rk) row-major per node, at uoff
    DevBuf J;                               // int32 skeleton rows (local), at koff
    DevBuf skel;                            // int64 skeleton points (cluster-tree order), at koff
    DevBuf rowmap;                          // int64 row of the level's sample block behind each skeleton, at koff
    DevBuf B;                               // (k_a x k_b) per inner node, at boff
    // ULV factors
    std::vector<char> pass;                 // 1: rank == size, nothing eliminated at this node
    std::vector<int64_t> foff;              // prefix sums of msz*msz over eliminated nodes (0 for pass nodes)
    DevBuf Mup, Mdown;                      // dense operators of the up / down sweep
    std::vector<int64_t> kkoff;             // prefix sums of rk*rk
    DevBuf RT, RTi;                         // R^T and R^-T per node (k x k), R = reduced basis handed to the parent
    DevBuf QT;                              // Q^T per eliminating node (m x m, at foff): depends on U only, kept across betas
    DevBuf OffD;                            // R_a B R_b^T per inner node (k_a x k_b, at boff): likewise
    // solve plumbing
    double *bvec = nullptr, *ce = nullptr, *xvec = nullptr;   // level vectors inside hss_ctx::vpool (single-column
                                            // layout): input (sum msz), eliminated part (sum msz-rk), output (sum msz)
    DevBuf up_items, down_items, work;      // SolveItem tables and the (node, row block) work list
    int nwork = 0;
    DevBuf work_wide;                       // the same for four interleaved right-hand sides (16-row blocks)
    int nwork_wide = 0;
    int rows_per_wave = 2;                  // launch shape of the level's solve kernel: a workgroup takes
                                            // 4 * rows_per_wave rows of one node
    bool vec = false;                       // 16-byte loads allowed (all sizes even)
    bool skip = false;                      // leaf level where no node eliminates anything: the level above reads
                                            // and writes the leaf vectors directly and no kernel is launched
    // mat-vec plumbing
    DevBuf UT;                              // U^T (rk x msz) per node at uoff, nodes with rk < msz only
    DevBuf BT;                              // B^T (k_b x k_a) per inner node at boff
    bool mv_vec = false;                    // 16-byte loads allowed in this level's mat-vec tables
    DevBuf xt, g;                           // (sum rk) each
    DevBuf mv_up, mv_dn_u, mv_dn_b, mv_leaf_d;   // GemvItem tables (mv_dn_b: B and B^T products of every pair)
    int n_dn_b = 0;
};

// FP32 copies of the generators and the item tables of the mat-vec on them (matvec32.hip): filled for the
// definiteness guard's run.  The pool stays allocated between compressions and only grows (freeing tens of
// gigabytes right before the factorization allocates its own made those allocations take seconds).
struct Matvec32 {
    struct Lev {
        float *U = nullptr, *UT = nullptr, *B = nullptr, *BT = nullptr;   // copies of the level's U, U^T and of the
                                            // parent level's B, B^T, inside `pool`
        const GemvItem32 *up = nullptr, *dn_u = nullptr, *dn_b = nullptr;   // item tables, in the context's upload arena
        int n_dn_b = 0;
        bool vec4 = false;                  // 16-byte loads allowed (sizes and ranks multiples of 4)
    };
    std::vector<Lev> lev;
    DevBuf pool;                            // all FP32 copies in one allocation, kept until the context is destroyed
    float* D = nullptr;
    const GemvItem32* leaf_d = nullptr;
    bool leaves4 = false, ready = false;
};

struct hss_ctx {
    BlockCache cache;                       // device blocks between their uses (see common.h); every call on the
                                            // context opens a CacheScope on it
    hipStream_t stream = nullptr;
    hipStream_t gstream = nullptr;          // the library's own stream for graph capture and replay (default priority)
    hipEvent_t gevent = nullptr;            // orders gstream after / before the caller's stream
    // options
    int64_t opt_s = 128, opt_p = -1, opt_max_rank = 0, opt_seed = 0, opt_guard = 1;   // opt_p < 0: s/2
    int64_t opt_sampling = 0;               // 0: random sample K Omega; 1: columns of approximate nearest neighbours
    int64_t opt_ann_k = 64, opt_ann_cell = 512, opt_ann_trees = 3;
    int64_t opt_cluster = 0, opt_cluster_iters = 2;   // cluster tree: 0 coordinate bisection, 1 two-means bisection
    int64_t opt_cache_basis = 1;            // keep the beta-independent parts of the factorization between factorizations
    int64_t opt_graph = 0;                  // replay the ADMM iterations from a HIP graph (measured slower: off)
    int64_t opt_merge_top = 1;              // merge the top levels of the solve into one dense operator
    int64_t opt_adapt_start = 0, opt_adapt_step = 128;   // adaptive sample width: first width (0 = off), increment
    double  opt_abs_tol = 1e-8;
    // problem
    bool compressed = false, factored = false;
    bool basis_cached = false;              // QT, RT, RTi, OffD of every level hold for the current compression
    int64_t n = 0, n_pad = 0;
    int r = 0, r_pad = 0, leaf = 0, L = 0, s = 0, s_pad = 0, kcap = 0;   // leaf: the largest leaf size (tree_depth)
    double h = 0.0, tol = 0.0, delta = 0.0, beta = -1.0;
    int warnings = 0;
    int width_used = 0;                     // sample columns the decompositions ended up using
    int64_t nodes_redone = 0;               // node decompositions repeated after widening the sample
    DevBuf Fp, nu, yp, perm;                // Fp: the points in cluster-tree order, centred (minus `centre`), zero padded
    DevBuf centre;                          // r feature means of the training points (subtracted from test points too)
    DevBuf Dleaf;                           // leaf diagonal blocks D_t (m_t x m_t row-major), leaf t at doff[t]
    std::vector<int64_t> doff;              // prefix sums of m_t^2 over the leaves            [2^L + 1]
    bool leaves_even = false;               // every leaf size is even: 16-byte loads allowed on the D_t
    DevBuf nbr_idx, nbr_dist;               // neighbour lists (n x ann_k, cluster-tree order), neighbour-based sampling
    int ann_k = 0;
    std::vector<int64_t> perm_host;
    std::vector<Level> lev;                 // 0 .. L
    DevBuf rootinv;                         // inverse of the root block (root_m x root_m)
    DevBuf vpool;                           // all level vectors of the solve, MAX_NRHS x their single-column length:
                                            // with nrhs interleaved right-hand sides a vector at pool + o lives at
                                            // pool + o * nrhs
    int root_m = 0;
    // Top of the tree merged into one dense operator: levels 0 .. top_l are replaced by x = topT b on the vectors
    // of level top_l (topT = inverse of the reduced matrix there, top_m x top_m); top_l = 0 with topT unset means
    // the plain root solve through rootinv.
    int top_l = 0, top_m = 0;
    DevBuf topT;
    double *top_in = nullptr, *top_out = nullptr;   // single-column pool pointers of the operator's input / output
    DevBuf flags;                           // int[4] device flags (bit 0: tiny pivot)
    DescArena arena;
    // fixed vectors (cluster-tree order)
    DevBuf mv_x, mv_y;                      // mat-vec in / out
    Matvec32 mv32;
    DevBuf v_x, v_z, v_mu, v_t, v_w, v_e, v_u;   // ADMM
    DevBuf partial, scal;                   // reduction partials (4*VEC_BLOCKS), device scalars (16)
    // stats
    double sample_flops = 0.0, t_tree = 0.0, t_sample = 0.0, t_levels = 0.0, t_guard = 0.0, t_factor = 0.0;
    double t_sample_kernel = 0.0;           // HIP-event time of the sampling kernel alone
    int64_t generator_bytes = 0, factor_bytes = 0, factor_bytes_compact = 0;
};

int build_cluster_tree(hipStream_t st, const double* F_dev, int64_t n, int r, int leaf, int64_t* perm_dev, int* bad_dev);
int build_cluster_tree_2means(hipStream_t st, const double* F_dev, int64_t n, int r, int leaf, int iters,
                              int64_t* perm_dev, int* bad_dev);

// noalloc.hip: device address of the library's fixed scratch array on the current device
int noalloc_scratch_for_current_device(double** out);
// ann.hip
int ann_search(hss_ctx* c, const double* F, int k, int cell, int trees, uint64_t seed);   // F: the caller's n x r points
struct AnnWork {    // work buffers of ann_select_columns, reused across the levels of one compression
    DevBuf rn, keys_a, keys_b, tmp, seg_lo, seg_hi, ncd, span;
};
int ann_select_columns(hss_ctx* c, AnnWork& wk, const int64_t* rowpoint, const std::vector<int32_t>& rownode_host,
                       int64_t rows, int N, int level, int s, int64_t* cols_dev, std::vector<int32_t>& ncols_host);
double ann_direction_component(uint64_t seed, int tree, int level, int64_t node, int f);
// hss.hip
int hss_compress_impl(hss_ctx* c, const double* F, const double* y, int64_t n, int r, double h, int leaf, double tol,
                      const double* Omega, int s_in);
int hss_import_impl(hss_ctx* c, const double* F, const double* y, int64_t n, int r, double h, int leaf,
                    const int64_t* perm_h, const int32_t* sizes, const int32_t* ranks, const double* D, const double* U,
                    const int32_t* J, const double* B, double delta);
int hss_matvec_perm(hss_ctx* c);           // mv_y = K~' mv_x  (cluster-tree order, shift included)
// matvec32.hip
int build_matvec32(hss_ctx* c);
void release_matvec32(hss_ctx* c);
int hss_matvec_perm32(hss_ctx* c);
// ulv.hip
int ulv_factor_impl(hss_ctx* c, double beta);
int ulv_solve_perm(hss_ctx* c, const double* b_perm, double* x_perm);   // cluster-tree order; may alias
// nrhs in {1, 2, 4} interleaved right-hand sides, in place in the leaf-level vectors: input in
// solve_rhs(c), result in solve_sol(c) (entry i of column j at [i * nrhs + j])
int ulv_solve_inplace(hss_ctx* c, int nrhs);
inline double* solve_rhs(hss_ctx* c) { return c->lev[c->L].bvec; }   // pool offset 0
inline double* solve_sol(hss_ctx* c, int nrhs) {
    return c->vpool.as<double>() + (c->lev[c->L].xvec - c->vpool.as<double>()) * nrhs;
}
constexpr int MAX_NRHS = 4;
