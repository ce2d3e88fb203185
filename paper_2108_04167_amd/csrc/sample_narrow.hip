// Narrow products with the Gaussian kernel matrix never stored:  S (rows x 16) = K(rows, cols) * V  for at most 16
// columns of V -- the label assignment (Algorithm 3, last line: one column, y .* z) and the probes of the achieved-
// error estimate (the tolerance of Sec. 3.2 / eq. (9)).  Same three steps per block of 32 column points as the wide
// sampling kernel (Gram tile on the matrix cores, exp on the vector ALUs into LDS, contraction on the matrix cores),
// but a 16-column result gives the contraction only 32 matrix instructions per block, so they are split over all 8
// wavefronts by row tile and by half of the block's 8 k-steps, and the two halves are added at the end; with a
// 128-column launch every wavefront would issue those 32 itself for 16 columns of which one is used.
// Few rows (a small test set) would leave most of the chip idle: the column blocks are then split over grid.y,
// every split writes its own partial result, and a second kernel adds the partials in a fixed order.
#include "common.h"
#include <algorithm>

namespace {

constexpr int NB = 32;          // column points per block
constexpr int BM = 64;          // rows per workgroup

// e^x for x <= 0: x = (64 m + j) ln2/64 + r, |r| <= ln2/128, e^x = 2^m 2^(j/64) (1 + r + r^2/2 + ... + r^5/120),
// 2^(j/64) from a table in LDS; underflows to 0 through the exponent scaling
__device__ __forceinline__ double exp_nonpos(double x, const double* __restrict__ tab) {
    const double kf = __builtin_rint(x * 92.332482616893656877);
    const int ki = (int)kf;
    double r = __builtin_fma(kf, -1.08304246932675596327e-02, x);
    r = __builtin_fma(kf, -2.98158582698529328128e-12, r);
    const double T = tab[ki & 63];
    double q = __builtin_fma(r, 1.0 / 120.0, 1.0 / 24.0);
    q = __builtin_fma(q, r, 1.0 / 6.0);
    q = __builtin_fma(q, r, 0.5);
    q = __builtin_fma(q, r, 1.0);
    return __builtin_amdgcn_ldexp(__builtin_fma(T, q * r, T), ki >> 6);
}

// NK4: k-steps of the Gram tile (4 features each); the feature dimension is padded to RP = 4 * NK4.
// grid.x: blocks of 64 rows; grid.y: splits of the column blocks, split y takes blocks [y * per_split, ...).
// P: gridDim.y x nr_pad x 16 partial results.
template <int NK4>
__global__ __launch_bounds__(512) void narrow_kernel(const double* __restrict__ Fr, const double* __restrict__ nur,
                                                      const double* __restrict__ Fp, const double* __restrict__ nu,
                                                      const double* __restrict__ V, double* __restrict__ P, int nr_pad,
                                                      int nblocks, int per_split, double inv2h2) {
    constexpr int RP = 4 * NK4;
    constexpr int LDF = RP + 1;
    constexpr int LDK = BM + 1;
    constexpr int TILE = NB * RP;
    constexpr int MAXF = (TILE + 511) / 512;
    extern __shared__ double smem[];
    double* Fi_s = smem;                           // BM x LDF
    double* Fj_s = Fi_s + BM * LDF;                // 2 x NB x LDF
    double* nui_s = Fj_s + 2 * NB * LDF;           // BM      -nu_i / (2h^2)
    double* nuj_s = nui_s + BM;                    // 2 x NB  -nu_j / (2h^2)
    double* tab_s = nuj_s + 2 * NB;                // 64      2^(j/64)
    double* K_s = tab_s + 64;                      // 2 x NB x LDK, j-major

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int lr = lane & 15, lk = lane >> 4;
    const int row0 = blockIdx.x * BM;
    const int jb0 = blockIdx.y * per_split;
    const int jb1 = jb0 + per_split < nblocks ? jb0 + per_split : nblocks;      // the host makes jb0 < jb1
    const double invh2 = 2.0 * inv2h2;

    if (tid < 64) tab_s[tid] = exp2((double)tid * (1.0 / 64.0));
    for (int idx = tid; idx < BM * RP; idx += 512) {
        const int rr = idx / RP, cc = idx - rr * RP;
        Fi_s[rr * LDF + cc] = Fr[(size_t)row0 * RP + idx];
    }
    if (tid < BM) nui_s[tid] = -nur[row0 + tid] * inv2h2;
    for (int b = 0; b < 2; ++b) {
        const int jb = jb0 + b < jb1 ? jb0 + b : jb1 - 1;
        for (int idx = tid; idx < TILE; idx += 512) {
            const int rr = idx / RP, cc = idx - rr * RP;
            Fj_s[(b * NB + rr) * LDF + cc] = Fp[(size_t)jb * TILE + idx];
        }
        if (tid < NB) nuj_s[b * NB + tid] = -nu[jb * NB + tid] * inv2h2;
    }
    __syncthreads();

    // K tile of a block: 4 x 2 tiles of 16 x 16, wavefront w computes tile (w >> 1, w & 1)
    const int rt = wave >> 1, ct2 = wave & 1;
    auto gram_exp = [&](int buf) {
        const double* ap = Fi_s + (rt * 16 + lr) * LDF + lk;
        const double* bp = Fj_s + (buf * NB + ct2 * 16 + lr) * LDF + lk;
        v4d g = (v4d){0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int q = 0; q < NK4; ++q) g = __builtin_amdgcn_mfma_f64_16x16x4f64(ap[4 * q], bp[4 * q], g, 0, 0, 0);
        // accumulator register v of lane (lk, lr) is G[4 v + lk][lr]
        const double nj = nuj_s[buf * NB + ct2 * 16 + lr];
        double* kp = K_s + (buf * NB + ct2 * 16 + lr) * LDK + rt * 16 + lk;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            double x = __builtin_fma(g[v], invh2, nui_s[rt * 16 + 4 * v + lk] + nj);
            x = x < 0.0 ? x : 0.0;
            kp[4 * v] = exp_nonpos(x, tab_s);
        }
    };
    gram_exp(0);
    __syncthreads();

    // contraction: wavefront w adds k-steps 4 (w & 1) .. 4 (w & 1) + 3 of every block into row tile w >> 1
    const int kh = wave & 1;
    v4d acc = (v4d){0.0, 0.0, 0.0, 0.0};
    double fj[MAXF];
    double nuj_next = 0.0;
    for (int jb = jb0; jb < jb1; ++jb) {
        const int cur = (jb - jb0) & 1, nxt = cur ^ 1;
        const int jb2 = jb + 2 < jb1 ? jb + 2 : jb1 - 1;
        const double* fsrc = Fp + (size_t)jb2 * TILE + tid;
#pragma unroll
        for (int u = 0; u < MAXF; ++u)
            if ((u + 1) * 512 <= TILE || tid + u * 512 < TILE) fj[u] = fsrc[u * 512];
        if (tid < NB) nuj_next = -nu[jb2 * NB + tid] * inv2h2;
        const double* vp = V + ((size_t)jb * NB + kh * 16 + lk) * 16 + lr;
        double b[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) b[q] = vp[q * 64];
        if (jb + 1 < jb1) gram_exp(nxt);                       // the next block's K tile, from the tile staged last time
        const double* kt = K_s + (cur * NB + kh * 16 + lk) * LDK + rt * 16 + lr;
#pragma unroll
        for (int q = 0; q < 4; ++q) acc = __builtin_amdgcn_mfma_f64_16x16x4f64(kt[q * 4 * LDK], b[q], acc, 0, 0, 0);
#pragma unroll
        for (int u = 0; u < MAXF; ++u) {
            const int idx = tid + u * 512;
            if ((u + 1) * 512 <= TILE || idx < TILE) {
                const int rr = idx / RP, cc = idx - rr * RP;
                Fj_s[(cur * NB + rr) * LDF + cc] = fj[u];
            }
        }
        if (tid < NB) nuj_s[cur * NB + tid] = nuj_next;
        __syncthreads();
    }
    // add the two k-halves of every row tile (through the K tile's LDS, free after the last barrier) and store:
    // accumulator register v of lane (lk, lr) is S[row0 + rt*16 + 4 v + lk][lr]
    double* red = K_s;
    if (kh == 1) {
#pragma unroll
        for (int v = 0; v < 4; ++v) red[(rt * 4 + v) * 64 + lane] = acc[v];
    }
    __syncthreads();
    if (kh == 0) {
        double* out = P + ((size_t)blockIdx.y * nr_pad + row0 + rt * 16 + lk) * 16 + lr;
#pragma unroll
        for (int v = 0; v < 4; ++v) out[(size_t)4 * v * 16] = acc[v] + red[(rt * 4 + v) * 64 + lane];
    }
}

// S[i] = sum over the splits, in split order, of P[split][i]
__global__ __launch_bounds__(256) void narrow_reduce_kernel(const double* __restrict__ P, int splits, int64_t count,
                                                             double* __restrict__ S) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= count) return;
    double s = 0.0;
    for (int p = 0; p < splits; ++p) s += P[(size_t)p * count + i];
    S[i] = s;
}

size_t narrow_smem(int r_pad) {
    const int ldf = r_pad + 1;
    return sizeof(double) * ((size_t)BM * ldf + 2 * NB * ldf + BM + 2 * NB + 64 + 2 * NB * (BM + 1));
}

template <int NK4>
int narrow_go(hipStream_t st, const double* Fr, const double* nur, int nr_pad, const double* Fp, const double* nu,
              const double* V, double* P, int nblocks, int splits, int per_split, double inv2h2) {
    const size_t smem = narrow_smem(4 * NK4);
    auto kern = narrow_kernel<NK4>;
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    hipLaunchKernelGGL(kern, dim3((unsigned)(nr_pad / BM), (unsigned)splits), dim3(512), smem, st, Fr, nur, Fp, nu, V, P,
                       nr_pad, nblocks, per_split, inv2h2);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}

}  // namespace

// S (nr_pad x 16) = K(rows, cols) V with rows = the points (Fr, nur), cols = the points (Fp, nu); V is n_pad x 16
// (unused columns zero).  Both point sets are padded (rows to a multiple of 256, features to r_pad, a multiple of
// 28; above 112 the product goes through sample_wide_launch).  `work` is grown to hold the partial results of the
// column splits.
int sample_narrow_launch(hipStream_t st, const double* Fr, const double* nur, int64_t nr_pad, const double* Fp,
                         const double* nu, int64_t n_pad, const double* V, double* S, int r_pad, double h, DevBuf& work) {
    if (r_pad > 112) return sample_wide_launch(st, Fr, nur, nr_pad, Fp, nu, n_pad, V, S, r_pad, 16, 16, h);
    if (n_pad % 256 || nr_pad % 256 || n_pad < 256 || nr_pad < 256 || r_pad % 28 || r_pad < 28 || r_pad > 112 ||
        nr_pad >= (int64_t(1) << 31) || n_pad >= (int64_t(1) << 31))
        return HSS_EUNSUPPORTED;
    if (narrow_smem(r_pad) > size_t(150) * 1024) return HSS_EUNSUPPORTED;
    const double inv2h2 = 1.0 / (2.0 * h * h);
    const int nblocks = (int)(n_pad / NB);
    const int64_t row_blocks = nr_pad / BM;
    // enough workgroups for two per compute unit; every split takes at least 8 column blocks
    int splits = 1;
    if (row_blocks < 512) splits = (int)std::min<int64_t>((512 + row_blocks - 1) / row_blocks, 64);
    splits = std::max(1, std::min(splits, nblocks / 8));
    int per_split = (nblocks + splits - 1) / splits;
    splits = (nblocks + per_split - 1) / per_split;           // no empty split
    double* P = S;
    if (splits > 1) {
        HSS_TRY(work.reserve(sizeof(double) * (size_t)splits * nr_pad * 16));
        P = work.as<double>();
    }
    int rc;
    switch (r_pad / 28) {
        case 1: rc = narrow_go<7>(st, Fr, nur, (int)nr_pad, Fp, nu, V, P, nblocks, splits, per_split, inv2h2); break;
        case 2: rc = narrow_go<14>(st, Fr, nur, (int)nr_pad, Fp, nu, V, P, nblocks, splits, per_split, inv2h2); break;
        case 3: rc = narrow_go<21>(st, Fr, nur, (int)nr_pad, Fp, nu, V, P, nblocks, splits, per_split, inv2h2); break;
        case 4: rc = narrow_go<28>(st, Fr, nur, (int)nr_pad, Fp, nu, V, P, nblocks, splits, per_split, inv2h2); break;
        default: return HSS_EUNSUPPORTED;
    }
    HSS_TRY(rc);
    if (splits > 1) {
        const int64_t count = nr_pad * 16;
        hipLaunchKernelGGL(narrow_reduce_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st, P, splits, count, S);
        HIP_TRY(hipGetLastError());
    }
    return HSS_OK;
}
