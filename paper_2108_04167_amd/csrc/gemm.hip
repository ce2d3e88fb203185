// Batched ragged FP64 GEMM on the gfx950 matrix cores (v_mfma_f64_16x16x4_f64).
//
// One workgroup of 4 wavefronts computes a 64 x 64 tile of C for one batch item; each wavefront
// owns a 32 x 32 sub-tile (2 x 2 MFMA tiles, 16 accumulator doubles per lane).  K is walked in
// steps of 16 through LDS; the tile for step t+1 is fetched from HBM into registers while step t
// is being multiplied.  Operand tiles are stored k-major in LDS so that the MFMA operand fetch
// (lane = 16*k + row) reads 16 consecutive doubles per k.
//
// MFMA f64 16x16x4 lane layout (checked on the device by the mfma layout probe test):
//   A operand: lane l holds A[l % 16][l / 16];  B operand: lane l holds B[l / 16][l % 16];
//   accumulator register v of lane l holds D[4 * v + l / 16][l % 16].
#include "common.h"

namespace {

constexpr int BM = 64, BN = 64, BK = 16;
constexpr int LD = 68;   // LDS leading dimension (doubles): 64 + 4 keeps the four k rows of a fetch on distinct banks

// Fetch 4 elements of a (64 x 16) operand tile into registers.
// KCONTIG: element (mn, k) lives at X[(mn0 + mn) * ld + k0 + k]; else at X[(k0 + k) * ld + mn0 + mn].
template <bool KCONTIG>
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
        int k = k0 + (tid >> 4);
        int mn = mn0 + ((tid & 15) << 2);
        const double* p = X + (size_t)k * ld + mn;
        bool okk = k < K;
#pragma unroll
        for (int u = 0; u < 4; ++u) r[u] = (okk && mn + u < MN) ? p[u] : 0.0;
    }
}

template <bool KCONTIG>
__device__ __forceinline__ void tile_store(double* __restrict__ Xs, int tid, const double (&r)[4]) {
    if (KCONTIG) {
        int mn = tid >> 2;
        int k = (tid & 3) << 2;
#pragma unroll
        for (int u = 0; u < 4; ++u) Xs[(k + u) * LD + mn] = r[u];
    } else {
        int k = tid >> 4;
        int mn = (tid & 15) << 2;
#pragma unroll
        for (int u = 0; u < 4; ++u) Xs[k * LD + mn + u] = r[u];
    }
}

template <bool TA, bool TB>
__global__ __launch_bounds__(256) void bgemm_kernel(const GemmItem* __restrict__ items, int tilesN, double alpha,
                                                    double beta) {
    const GemmItem it = items[blockIdx.x];
    const int tm = blockIdx.y / tilesN, tn = blockIdx.y % tilesN;
    const int m0 = tm * BM, n0 = tn * BN;
    if (m0 >= it.M || n0 >= it.N) return;

    __shared__ double As[BK * LD];
    __shared__ double Bs[BK * LD];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int lr = lane & 15, lk = lane >> 4;

    v4d acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = (v4d){0.0, 0.0, 0.0, 0.0};

    double ra[4], rb[4];
    const int K = it.K;
    if (K > 0) {
        // op(A)(m,k): TA ? A[k*lda+m] : A[m*lda+k]   -> k contiguous when !TA
        // op(B)(k,n): TB ? B[n*ldb+k] : B[k*ldb+n]   -> k contiguous when TB
        tile_fetch<!TA>(it.A, it.lda, m0, it.M, 0, K, tid, ra);
        tile_fetch<TB>(it.B, it.ldb, n0, it.N, 0, K, tid, rb);
    }
    for (int k0 = 0; k0 < K; k0 += BK) {
        tile_store<!TA>(As, tid, ra);
        tile_store<TB>(Bs, tid, rb);
        __syncthreads();
        if (k0 + BK < K) {
            tile_fetch<!TA>(it.A, it.lda, m0, it.M, k0 + BK, K, tid, ra);
            tile_fetch<TB>(it.B, it.ldb, n0, it.N, k0 + BK, K, tid, rb);
        }
#pragma unroll
        for (int kk = 0; kk < BK / 4; ++kk) {
            const double* ap = As + (kk * 4 + lk) * LD + wm * 32 + lr;
            const double* bp = Bs + (kk * 4 + lk) * LD + wn * 32 + lr;
            double a0 = ap[0], a1 = ap[16];
            double b0 = bp[0], b1 = bp[16];
            acc[0][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b1, acc[1][1], 0, 0, 0);
        }
        __syncthreads();
    }

#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                int row = m0 + wm * 32 + i * 16 + 4 * v + lk;
                int col = n0 + wn * 32 + j * 16 + lr;
                if (row < it.M && col < it.N) {
                    double* c = it.C + (size_t)row * it.ldc + col;
                    double val = alpha * acc[i][j][v];
                    if (beta != 0.0) val += beta * (*c);
                    *c = val;
                }
            }
}

}  // namespace

int bgemm(hipStream_t st, const GemmItem* items_dev, int nitems, int maxM, int maxN, bool transA, bool transB,
          double alpha, double beta) {
    if (nitems <= 0 || maxM <= 0 || maxN <= 0) return HSS_OK;
    int tilesM = (maxM + BM - 1) / BM, tilesN = (maxN + BN - 1) / BN;
    if ((int64_t)tilesM * tilesN > 65535) return HSS_EUNSUPPORTED;
    dim3 grid((unsigned)nitems, (unsigned)(tilesM * tilesN));
    if (!transA && !transB)
        hipLaunchKernelGGL((bgemm_kernel<false, false>), grid, dim3(256), 0, st, items_dev, tilesN, alpha, beta);
    else if (!transA && transB)
        hipLaunchKernelGGL((bgemm_kernel<false, true>), grid, dim3(256), 0, st, items_dev, tilesN, alpha, beta);
    else if (transA && !transB)
        hipLaunchKernelGGL((bgemm_kernel<true, false>), grid, dim3(256), 0, st, items_dev, tilesN, alpha, beta);
    else
        hipLaunchKernelGGL((bgemm_kernel<true, true>), grid, dim3(256), 0, st, items_dev, tilesN, alpha, beta);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}
