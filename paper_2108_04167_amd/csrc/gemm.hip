// Batched ragged FP64 GEMM on the gfx950 matrix cores (v_mfma_f64_16x16x4_f64).
//
// One workgroup computes a T x T tile of C for one batch item, T = 64 (4 wavefronts, each a 32 x 32 sub-tile of
// 2 x 2 MFMA tiles) or T = 128 (8 wavefronts, each a 64 x 32 sub-tile of 4 x 2 MFMA tiles) when the batch has
// items of at least 128 x 128: the larger tile halves the operand traffic per flop, which is what bounds the small
// one on large items.  K is walked in steps of 16 through LDS; the tile for step t+1 is fetched from HBM into
// registers while step t is being multiplied.  Operand tiles are stored k-major in LDS so that the MFMA operand
// fetch (lane = 16*k + row) reads 16 consecutive doubles per k.  Both tile sizes add the k-steps of an output
// element in the same order, so they give the same bits.
//
// MFMA f64 16x16x4 lane layout (checked on the device by the mfma layout probe test):
//   A operand: lane l holds A[l % 16][l / 16];  B operand: lane l holds B[l / 16][l % 16];
//   accumulator register v of lane l holds D[4 * v + l / 16][l % 16].
#include "common.h"

namespace {

constexpr int BK = 16;

// Fetch 4 elements of a (T x 16) operand tile into registers (T * 4 threads).
// KCONTIG: element (mn, k) lives at X[(mn0 + mn) * ld + k0 + k]; else at X[(k0 + k) * ld + mn0 + mn].
template <bool KCONTIG, int T>
__device__ __forceinline__ void tile_fetch(const double* __restrict__ X, int ld, int mn0, int MN, int k0, int K,
                                           int tid, double (&r)[4]) {
    if (KCONTIG) {
        int mn = mn0 + (tid >> 2);
        int k = k0 + ((tid & 3) << 2);
        const double* p = X + (size_t)mn * ld + k;
        bool okr = mn < MN;
#pragma unroll
        for (int u = 0; u < 4; ++u) r[u] = (okr && k + u < K) ? p[u] : 0.0;
    } else {
        int k = k0 + tid / (T / 4);
        int mn = mn0 + ((tid % (T / 4)) << 2);
        const double* p = X + (size_t)k * ld + mn;
        bool okk = k < K;
#pragma unroll
        for (int u = 0; u < 4; ++u) r[u] = (okk && mn + u < MN) ? p[u] : 0.0;
    }
}

template <bool KCONTIG, int T>
__device__ __forceinline__ void tile_store(double* __restrict__ Xs, int tid, const double (&r)[4]) {
    constexpr int LD = T + 4;   // + 4 keeps the four k rows of a fetch on distinct banks
    if (KCONTIG) {
        int mn = tid >> 2;
        int k = (tid & 3) << 2;
#pragma unroll
        for (int u = 0; u < 4; ++u) Xs[(k + u) * LD + mn] = r[u];
    } else {
        int k = tid / (T / 4);
        int mn = (tid % (T / 4)) << 2;
#pragma unroll
        for (int u = 0; u < 4; ++u) Xs[k * LD + mn + u] = r[u];
    }
}

// T = 64: 4 wavefronts in 2 x 2, sub-tile 32 x 32 (IM = 2).  T = 128: 8 wavefronts in 2 x 4, sub-tile 64 x 32 (IM = 4).
template <bool TA, bool TB, int T>
__global__ __launch_bounds__(T * 4) void bgemm_kernel(const GemmItem* __restrict__ items, int tilesN, double alpha,
                                                      double beta) {
    constexpr int LD = T + 4;
    constexpr int IM = T / 32;            // MFMA tiles per wavefront along M
    constexpr int WN = T / 32;            // wavefronts along N
    const GemmItem it = items[blockIdx.x];
    const int tm = blockIdx.y / tilesN, tn = blockIdx.y % tilesN;
    const int m0 = tm * T, n0 = tn * T;
    if (m0 >= it.M || n0 >= it.N) return;

    __shared__ double As[BK * LD];
    __shared__ double Bs[BK * LD];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int lr = lane & 15, lk = lane >> 4;

    v4d acc[IM][2];
#pragma unroll
    for (int i = 0; i < IM; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = (v4d){0.0, 0.0, 0.0, 0.0};

    double ra[4], rb[4];
    const int K = it.K;
    if (K > 0) {
        // op(A)(m,k): TA ? A[k*lda+m] : A[m*lda+k]   -> k contiguous when !TA
        // op(B)(k,n): TB ? B[n*ldb+k] : B[k*ldb+n]   -> k contiguous when TB
        tile_fetch<!TA, T>(it.A, it.lda, m0, it.M, 0, K, tid, ra);
        tile_fetch<TB, T>(it.B, it.ldb, n0, it.N, 0, K, tid, rb);
    }
    for (int k0 = 0; k0 < K; k0 += BK) {
        tile_store<!TA, T>(As, tid, ra);
        tile_store<TB, T>(Bs, tid, rb);
        __syncthreads();
        if (k0 + BK < K) {
            tile_fetch<!TA, T>(it.A, it.lda, m0, it.M, k0 + BK, K, tid, ra);
            tile_fetch<TB, T>(it.B, it.ldb, n0, it.N, k0 + BK, K, tid, rb);
        }
#pragma unroll
        for (int kk = 0; kk < BK / 4; ++kk) {
            const double* ap = As + (kk * 4 + lk) * LD + wm * (16 * IM) + lr;
            const double* bp = Bs + (kk * 4 + lk) * LD + wn * 32 + lr;
            double a[IM];
#pragma unroll
            for (int i = 0; i < IM; ++i) a[i] = ap[16 * i];
            const double b0 = bp[0], b1 = bp[16];
#pragma unroll
            for (int i = 0; i < IM; ++i) {
                acc[i][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[i], b0, acc[i][0], 0, 0, 0);
                acc[i][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[i], b1, acc[i][1], 0, 0, 0);
            }
        }
        __syncthreads();
    }

#pragma unroll
    for (int i = 0; i < IM; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                int row = m0 + wm * (16 * IM) + i * 16 + 4 * v + lk;
                int col = n0 + wn * 32 + j * 16 + lr;
                if (row < it.M && col < it.N) {
                    double* c = it.C + (size_t)row * it.ldc + col;
                    double val = alpha * acc[i][j][v];
                    if (beta != 0.0) val += beta * (*c);
                    *c = val;
                }
            }
}

template <int T>
int bgemm_go(hipStream_t st, const GemmItem* items_dev, int nitems, int maxM, int maxN, bool transA, bool transB,
             double alpha, double beta) {
    int tilesM = (maxM + T - 1) / T, tilesN = (maxN + T - 1) / T;
    if ((int64_t)tilesM * tilesN > 65535) return HSS_EUNSUPPORTED;
    dim3 grid((unsigned)nitems, (unsigned)(tilesM * tilesN));
    if (!transA && !transB)
        hipLaunchKernelGGL((bgemm_kernel<false, false, T>), grid, dim3(T * 4), 0, st, items_dev, tilesN, alpha, beta);
    else if (!transA && transB)
        hipLaunchKernelGGL((bgemm_kernel<false, true, T>), grid, dim3(T * 4), 0, st, items_dev, tilesN, alpha, beta);
    else if (transA && !transB)
        hipLaunchKernelGGL((bgemm_kernel<true, false, T>), grid, dim3(T * 4), 0, st, items_dev, tilesN, alpha, beta);
    else
        hipLaunchKernelGGL((bgemm_kernel<true, true, T>), grid, dim3(T * 4), 0, st, items_dev, tilesN, alpha, beta);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}

}  // namespace

int bgemm(hipStream_t st, const GemmItem* items_dev, int nitems, int maxM, int maxN, bool transA, bool transB,
          double alpha, double beta) {
    if (nitems <= 0 || maxM <= 0 || maxN <= 0) return HSS_OK;
    if (maxM >= 128 && maxN >= 128) return bgemm_go<128>(st, items_dev, nitems, maxM, maxN, transA, transB, alpha, beta);
    return bgemm_go<64>(st, items_dev, nitems, maxM, maxN, transA, transB, alpha, beta);
}
