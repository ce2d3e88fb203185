// Randomized range sampling  S = K(Fp, Fp) * Omega  with the Gaussian kernel never stored
// (randomized sampling with oversampling, end of Sec. 3.2; kernel definition in Sec. 1.1).
//
//   K_ij = exp(-(nu_i + nu_j - 2 f_i . f_j) / (2 h^2)),   nu_i = ||f_i||^2
//
// One workgroup (8 wavefronts, WR x WC) owns a (64*WR) x (16*CT*WC) block of S and walks over all
// column blocks j of K, 32 points at a time:
//   1. Gram tile  G = F_i F_j^T               on the matrix cores (operands from LDS),
//   2. K tile     exp(-max(nu_i+nu_j-2G,0)/(2h^2))   on the vector ALUs, written to LDS,
//   3. S block   += K tile * Omega_j          on the matrix cores; every wavefront keeps a 64 x (16*CT)
//      accumulator block (128 VGPRs at CT = 4) and streams its own columns of Omega straight from
//      HBM/L2 into registers one j-block ahead of use (each Omega element is used by exactly
//      WR wavefronts of the workgroup, so LDS staging would not add reuse).
// The K tile and the F_j tile are double buffered in LDS: one barrier per j-block, placed before the last
// contraction k-step of the block (whose operands are in registers by then), so that no wavefront leaves the
// barrier with nothing but LDS reads to wait for.
#include "common.h"

namespace {

constexpr int BN = 32;          // points per j-block

// Constants of e^x on the vector ALUs, read through scalar loads so that they live in scalar registers
// (literal operands would be re-materialised into vector registers inside the loop).
//   [0] 64/ln2, [1] -(ln2/64) high part, [2] -(ln2/64) low part, [3..6] 1/120, 1/24, 1/6, 1/2
__constant__ double EXPC[8] = {
    92.332482616893656877, -1.08304246932675596327e-02, -2.98158582698529328128e-12,
    1.0 / 120.0, 1.0 / 24.0, 1.0 / 6.0, 0.5, 0.0};

// e^x for x <= 0 to within two ulp: x = (64 m + j) ln2/64 + r with |r| <= ln2/128,
// e^x = 2^m * T[j] * (1 + r (1 + r/2 + r^2/6 + r^3/24 + r^4/120)), T[j] = 2^(j/64) from an LDS table
// (remainder r^6/720 < 4e-17); underflows to 0 through the exponent scaling.
// a * b + c with the addend held in scalar registers (the compiler would otherwise copy the constant
// into vector registers to use the two-address form).
__device__ __forceinline__ double fma_vvs(double a, double b, double c_uniform) {
    double d;
    asm("v_fma_f64 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "s"(c_uniform));
    return d;
}

__device__ __forceinline__ double exp_nonpos(double x, const double (&c)[8], const double* __restrict__ tab) {
    const double kf = __builtin_rint(x * c[0]);
    const int ki = (int)kf;
    double r = __builtin_fma(kf, c[1], x);
    r = __builtin_fma(kf, c[2], r);
    const double T = tab[ki & 63];
    double q = fma_vvs(r, c[7], c[4]);      // c[7] = 1/120 kept in a vector register by the caller
    q = fma_vvs(q, r, c[5]);
    q = fma_vvs(q, r, c[6]);
    q = __builtin_fma(q, r, 1.0);
    return __builtin_amdgcn_ldexp(__builtin_fma(T, q * r, T), ki >> 6);
}

// One workgroup of 8 wavefronts (WR x WC); every wavefront owns a 64 x (16*CT) block of S.
// GP: Gram k-steps issued per contraction k-step; the feature dimension is padded to r_pad = 28 * GP.
template <int WR, int WC, int CT, int GP>
__global__ __launch_bounds__(512) void sample_kernel(const double* __restrict__ Fr, const double* __restrict__ nur,
                                                      const double* __restrict__ Fp, const double* __restrict__ nu,
                                                      const double* __restrict__ Om, double* __restrict__ S,
                                                      int n_pad, int s_pad, double inv2h2) {
    // rows of S: the points (Fr, nur), one workgroup per BMR of them; columns of K: the points (Fp, nu), n_pad of
    // them.  The two sets are the same for the compression sample and differ for the label assignment.
    // s_pad is the leading dimension of Om and S; the grid's y extent fixes how many of their columns (from the
    // pointers on) this launch computes, so a launch can fill a column window of wider arrays.
    static_assert(WR * WC == 8, "8 wavefronts");
    constexpr int BMR = 64 * WR;           // rows of S per workgroup
    constexpr int LDK = BMR + 1;           // leading dimension of the K tile (j-major); odd: the exp results of 16 lanes
                                           // (consecutive j, stride LDK) then fall into 16 distinct bank pairs
    constexpr int NK4 = 7 * GP;            // Gram k-steps
    constexpr int RP = 4 * NK4;            // padded feature count
    constexpr int LDF = RP + 1;
    constexpr int TILE = BN * RP;          // doubles in one F_j tile (contiguous in Fp)
    constexpr int MAXF = (TILE + 511) / 512;
    extern __shared__ double smem[];
    double* Fi_s = smem;                           // BMR x LDF
    double* Fj_s = Fi_s + BMR * LDF;               // 2 x BN x LDF
    double* nui_s = Fj_s + 2 * BN * LDF;           // BMR        holds -nu_i / (2h^2)
    double* nuj_s = nui_s + BMR;                   // 2 x BN     holds -nu_j / (2h^2)
    double* tab_s = nuj_s + 2 * BN;                // 64         2^(j/64)
    double* K_s = tab_s + 64;                      // 2 x BN x LDK

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int lr = lane & 15, lk = lane >> 4;
    const int wr = wave / WC, wc = wave % WC;
    const int row0 = blockIdx.x * BMR;
    const int col0 = (blockIdx.y * WC + wc) * (16 * CT);
    const int NJ = n_pad / BN;
    const double invh2 = 2.0 * inv2h2;

    double ec[8];
#pragma unroll
    for (int i = 0; i < 7; ++i) ec[i] = EXPC[i];
    {   // 1/120 as a vector-register operand (an instruction reads at most one scalar-register constant)
        double c3v;
        asm volatile("v_mov_b64 %0, %1" : "=v"(c3v) : "s"(EXPC[3]));
        ec[7] = c3v;
    }

    // ---- prologue: exp table, F_i tile, nu_i, F_j tiles 0 and 1 ----
    if (tid < 64) tab_s[tid] = exp2((double)tid * (1.0 / 64.0));
    for (int idx = tid; idx < BMR * RP; idx += 512) {
        int rr = idx / RP, cc = idx - rr * RP;
        Fi_s[rr * LDF + cc] = Fr[(size_t)row0 * RP + idx];
    }
    for (int idx = tid; idx < BMR; idx += 512) nui_s[idx] = -nur[row0 + idx] * inv2h2;
    for (int b = 0; b < 2; ++b) {
        int jb = b < NJ ? b : NJ - 1;
        for (int idx = tid; idx < TILE; idx += 512) {
            int rr = idx / RP, cc = idx - rr * RP;
            Fj_s[(b * BN + rr) * LDF + cc] = Fp[(size_t)jb * TILE + idx];
        }
        if (tid < BN) nuj_s[b * BN + tid] = -nu[jb * BN + tid] * inv2h2;
    }
    __syncthreads();

    // The K tile of a column block has (4*WR) x 2 MFMA tiles; wavefront w computes tiles w*WR .. w*WR+WR-1:
    // Gram accumulators g[u] (register v of lane (lk, lr) is G[4*v + lk][lr]), then
    // K = exp(min(0, G/h^2 - nu_i/(2h^2) - nu_j/(2h^2))) written j-major into LDS.
    auto gram_steps = [&](v4d (&g)[WR], const double* Fj, int q0, int q1) {   // k-steps q0 .. q1-1 (static)
#pragma unroll
        for (int u = 0; u < WR; ++u) {
            const int t = wave * WR + u;
            const double* ap = Fi_s + ((t >> 1) * 16 + lr) * LDF + lk;
            const double* bp = Fj + ((t & 1) * 16 + lr) * LDF + lk;
#pragma unroll
            for (int q = q0; q < q1; ++q) g[u] = __builtin_amdgcn_mfma_f64_16x16x4f64(ap[4 * q], bp[4 * q], g[u], 0, 0, 0);
        }
    };
    auto exp_store = [&](const v4d (&g)[WR], int buf, int v) {   // accumulator register v of every tile
#pragma unroll
        for (int u = 0; u < WR; ++u) {
            const int t = wave * WR + u;
            const int rt = t >> 1, ct2 = t & 1;
            const double nj = nuj_s[buf * BN + ct2 * 16 + lr];
            double* kp = K_s + buf * BN * LDK + (ct2 * 16 + lr) * LDK + rt * 16 + lk;
            // (rounding can leave x a few ulp above 0 on the diagonal; e^x is then 1 to rounding)
            const double x = __builtin_fma(g[u][v], invh2, nui_s[rt * 16 + 4 * v + lk] + nj);
            kp[4 * v] = exp_nonpos(x, ec, tab_s);
        }
    };

    v4d acc[4][CT];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < CT; ++j) acc[i][j] = (v4d){0.0, 0.0, 0.0, 0.0};

    // Omega register ring, RING k-steps deep: slot ks%RING holds Omega[jb*32 + ks*4 + lk][col0 + CT*lr + ct];
    // a slot is refilled for the k-step RING ahead right after it has been consumed.
    constexpr int RING = (CT == 4) ? 2 : 4;
    double om[RING][CT];
    const size_t step_elems = (size_t)4 * s_pad;
    auto load_omega = [&](const double* q, int slot) {
        if constexpr (CT == 4) {
            double2 q0 = reinterpret_cast<const double2*>(q)[0], q1 = reinterpret_cast<const double2*>(q)[1];
            om[slot][0] = q0.x; om[slot][1] = q0.y; om[slot][2] = q1.x; om[slot][3] = q1.y;
        } else if constexpr (CT == 2) {
            double2 q0 = reinterpret_cast<const double2*>(q)[0];
            om[slot][0] = q0.x; om[slot][1] = q0.y;
        } else {
            om[slot][0] = q[0];
        }
    };
    const double* op = Om + (size_t)lk * s_pad + col0 + CT * lr;   // this lane's element of k-step 0 of block 0
#pragma unroll
    for (int ks = 0; ks < RING; ++ks) load_omega(op + ks * step_elems, ks);
    {
        v4d g0[WR];
#pragma unroll
        for (int u = 0; u < WR; ++u) g0[u] = (v4d){0.0, 0.0, 0.0, 0.0};
        gram_steps(g0, Fj_s, 0, NK4);
#pragma unroll
        for (int v = 0; v < 4; ++v) exp_store(g0, 0, v);
    }
    __syncthreads();

    double fj[MAXF];
    double nuj_raw = 0.0;
    // K-tile operands of the next contraction k-step, fetched from LDS one step ahead and carried over the
    // barrier: the barrier sits between k-steps 6 and 7, so every wavefront leaves it with sixteen MFMAs whose
    // operands are already in registers, and fetches the first operands of the next tile behind them
    double an[4];
    {
        const double* Kt0 = K_s + wr * 64 + lr + lk * LDK;
        an[0] = Kt0[0]; an[1] = Kt0[16]; an[2] = Kt0[32]; an[3] = Kt0[48];
    }
    for (int jb = 0; jb < NJ; ++jb) {
        const int cur = jb & 1, nxt = cur ^ 1;
        // stage F_j tile jb+2 in registers (stored to LDS before this iteration's barrier)
        const int jb2 = jb + 2 < NJ ? jb + 2 : NJ - 1;
        const double* fsrc = Fp + (size_t)jb2 * TILE + tid;
#pragma unroll
        for (int u = 0; u < MAXF; ++u)
            if ((u + 1) * 512 <= TILE || tid + u * 512 < TILE) fj[u] = fsrc[u * 512];
        nuj_raw = nu[jb2 * BN + (tid & (BN - 1))];

        // Contraction with K tile jb.  The Gram tile of K tile jb+1 is spread over k-steps 0-2 and its
        // exponentials over steps 3-6 (one accumulator register each), so vector-ALU work and Gram MFMAs sit
        // between the contraction MFMAs.  (After the last column block the extra tile is computed from the
        // clamped F_j tile and never used.)
        const double* Kt = K_s + cur * BN * LDK + wr * 64 + lr + lk * LDK;
        const double* Ktn = K_s + nxt * BN * LDK + wr * 64 + lr + lk * LDK;
        const double* Fjn = Fj_s + nxt * BN * LDF;
        // Omega: block jb+1 is clamped to the last block (loads past it are never consumed)
        const size_t wrap = (jb + 1 < NJ) ? 0 : (size_t)BN * s_pad;
        v4d g[WR];
#pragma unroll
        for (int u = 0; u < WR; ++u) g[u] = (v4d){0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            if (ks == 7) {
                // publish F_j tile jb+2 into the buffer tile jb used; every read of K tile jb has been issued
                // (the operands of k-step 7 are in registers) and K tile jb+1 is complete
#pragma unroll
                for (int u = 0; u < MAXF; ++u) {
                    const int idx = tid + u * 512;
                    if ((u + 1) * 512 <= TILE || idx < TILE) {
                        const int rr = idx / RP, cc = idx - rr * RP;
                        Fj_s[(cur * BN + rr) * LDF + cc] = fj[u];
                    }
                }
                if (tid < BN) nuj_s[cur * BN + tid] = -nuj_raw * inv2h2;
                __syncthreads();
            }
            const double a0 = an[0], a1 = an[1], a2 = an[2], a3 = an[3];
            {
                const double* kp = ks < 7 ? Kt + (ks + 1) * 4 * LDK : Ktn;
                an[0] = kp[0]; an[1] = kp[16]; an[2] = kp[32]; an[3] = kp[48];
            }
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                double b = om[ks % RING][ct];
                acc[0][ct] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b, acc[0][ct], 0, 0, 0);
                acc[1][ct] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b, acc[1][ct], 0, 0, 0);
                acc[2][ct] = __builtin_amdgcn_mfma_f64_16x16x4f64(a2, b, acc[2][ct], 0, 0, 0);
                acc[3][ct] = __builtin_amdgcn_mfma_f64_16x16x4f64(a3, b, acc[3][ct], 0, 0, 0);
            }
            if (ks + RING < 8) load_omega(op + (ks + RING) * step_elems, ks % RING);
            else load_omega(op + (ks + RING) * step_elems - wrap, ks % RING);
            if (ks < 3) gram_steps(g, Fjn, (NK4 * ks) / 3, (NK4 * (ks + 1)) / 3);
            else if (ks < 7) exp_store(g, nxt, ks - 3);
        }
        op += (size_t)BN * s_pad;
    }

    // acc[rt][ct][v]  ->  S[row0 + wr*64 + rt*16 + 4*v + lk][col0 + CT*lr + ct]
#pragma unroll
    for (int rt = 0; rt < 4; ++rt)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            size_t row = (size_t)row0 + wr * 64 + rt * 16 + 4 * v + lk;
            double* q = S + row * s_pad + col0 + CT * lr;
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) q[ct] = acc[rt][ct][v];
        }
}

template <int WR>
size_t sample_smem(int r_pad) {
    int ldf = r_pad + 1;
    int bmr = 64 * WR;
    return sizeof(double) * ((size_t)bmr * ldf + 2 * BN * ldf + bmr + 2 * BN + 64 + 2 * BN * (bmr + 1));
}

template <int WR, int WC, int CT, int GP>
int sample_go_g(hipStream_t st, const double* Fr, const double* nur, int64_t nr_pad, const double* Fp, const double* nu,
                const double* Om, double* S, int64_t n_pad, int width, int s_pad, double inv2h2) {
    size_t smem = sample_smem<WR>(28 * GP);
    auto kern = sample_kernel<WR, WC, CT, GP>;
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)smem));
    dim3 grid((unsigned)(nr_pad / (64 * WR)), (unsigned)(width / (16 * CT * WC)));
    hipLaunchKernelGGL(kern, grid, dim3(512), smem, st, Fr, nur, Fp, nu, Om, S, (int)n_pad, s_pad, inv2h2);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}

template <int WR, int WC, int CT>
int sample_go(hipStream_t st, const double* Fr, const double* nur, int64_t nr_pad, const double* Fp, const double* nu,
              const double* Om, double* S, int64_t n_pad, int r_pad, int width, int s_pad, double inv2h2) {
    switch (r_pad / 28) {
        case 1: return sample_go_g<WR, WC, CT, 1>(st, Fr, nur, nr_pad, Fp, nu, Om, S, n_pad, width, s_pad, inv2h2);
        case 2: return sample_go_g<WR, WC, CT, 2>(st, Fr, nur, nr_pad, Fp, nu, Om, S, n_pad, width, s_pad, inv2h2);
        case 3: return sample_go_g<WR, WC, CT, 3>(st, Fr, nur, nr_pad, Fp, nu, Om, S, n_pad, width, s_pad, inv2h2);
        case 4: return sample_go_g<WR, WC, CT, 4>(st, Fr, nur, nr_pad, Fp, nu, Om, S, n_pad, width, s_pad, inv2h2);
        default: return HSS_EUNSUPPORTED;
    }
}

__global__ void row_norms_kernel(const double* __restrict__ Fp, double* __restrict__ nu, int64_t n_pad, int r_pad) {
    // one wavefront per point: lanes stride over the features, then a shuffle reduction
    int64_t row = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    int lane = threadIdx.x & 63;
    if (row >= n_pad) return;
    double acc = 0.0;
    for (int c = lane; c < r_pad; c += 64) {
        double v = Fp[row * r_pad + c];
        acc += v * v;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (lane == 0) nu[row] = acc;
}

__global__ void gather_pad_rows_kernel(const double* __restrict__ F, const int64_t* __restrict__ perm,
                                       double* __restrict__ Fp, int64_t n, int64_t n_pad, int r, int r_pad) {
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n_pad * r_pad) return;
    int64_t row = idx / r_pad;
    int c = (int)(idx - row * r_pad);
    double v = 0.0;
    if (row < n && c < r) {
        int64_t src = perm ? perm[row] : row;
        v = F[src * r + c];
    }
    Fp[idx] = v;
}

// Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3", SC'11),
// written from the published round function and constants.
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                              uint32_t k1, uint32_t (&out)[4]) {
    const uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)M0 * c0, p1 = (uint64_t)M1 * c2;
        uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        uint32_t n0 = hi1 ^ c1 ^ k0, n1 = lo1, n2 = hi0 ^ c3 ^ k1, n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += W0; k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Element (row, col) of Omega: counter = (row_lo, row_hi, col/2, 0), key = seed; one Philox block gives
// two 53-bit uniforms -> one Box-Muller pair; column parity picks cos or sin.
__global__ void omega_fill_kernel(double* __restrict__ Om, int64_t n, int64_t n_pad, int s, int s_pad, uint64_t seed) {
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // one thread per column pair
    int half = s_pad >> 1;
    if (idx >= n_pad * half) return;
    int64_t row = idx / half;
    int cp = (int)(idx - row * half);
    double v0 = 0.0, v1 = 0.0;
    if (row < n && 2 * cp < s) {
        uint32_t o[4];
        philox4x32_10((uint32_t)row, (uint32_t)(row >> 32), (uint32_t)cp, 0u, (uint32_t)seed, (uint32_t)(seed >> 32), o);
        uint64_t a = ((uint64_t)o[0] << 32 | o[1]) >> 11, b = ((uint64_t)o[2] << 32 | o[3]) >> 11;
        double u1 = ((double)a + 0.5) * (1.0 / 9007199254740992.0);   // (0,1)
        double u2 = ((double)b + 0.5) * (1.0 / 9007199254740992.0);
        double rad = sqrt(-2.0 * log(u1));
        double sn, cs;
        sincospi(2.0 * u2, &sn, &cs);
        v0 = rad * cs;
        v1 = (2 * cp + 1 < s) ? rad * sn : 0.0;
    }
    Om[row * s_pad + 2 * cp] = v0;
    Om[row * s_pad + 2 * cp + 1] = v1;
}

}  // namespace

// S (nr_pad x width) = K(rows, cols) Om with rows = the points (Fr, nur), cols = the points (Fp, nu); Om is
// n_pad x width.  Both arrays have leading dimension ld >= width (a column window of wider arrays is a pointer
// offset).  Both point sets are padded (rows to a multiple of 256, features to r_pad).
int sample_launch_window(hipStream_t st, const double* Fr, const double* nur, int64_t nr_pad, const double* Fp,
                         const double* nu, int64_t n_pad, const double* Om, double* S, int r_pad, int width, int ld,
                         double h) {
    if (n_pad % 256 || nr_pad % 256 || r_pad % 28 || r_pad < 28 || r_pad > 112 || width % 128 || width < 128 ||
        ld < width || (ld & 1))
        return HSS_EUNSUPPORTED;
    if ((reinterpret_cast<uintptr_t>(Om) | reinterpret_cast<uintptr_t>(S)) & 15) return HSS_EUNSUPPORTED;
    const double inv2h2 = 1.0 / (2.0 * h * h);
    // Widest block of S per workgroup whose column span divides the width and whose LDS footprint fits:
    // 64 x 512, else 128 x 256 (64 x 256 when the feature tiles are too large), else 128 x 128 (64 x 128).
    const size_t lds_cap = 150 * 1024;
    const bool fit2 = sample_smem<2>(r_pad) <= lds_cap;
    if (sample_smem<1>(r_pad) > lds_cap) return HSS_EUNSUPPORTED;
    if (width % 512 == 0)
        return sample_go<1, 8, 4>(st, Fr, nur, nr_pad, Fp, nu, Om, S, n_pad, r_pad, width, ld, inv2h2);
    if (width % 256 == 0)
        return fit2 ? sample_go<2, 4, 4>(st, Fr, nur, nr_pad, Fp, nu, Om, S, n_pad, r_pad, width, ld, inv2h2)
                    : sample_go<1, 8, 2>(st, Fr, nur, nr_pad, Fp, nu, Om, S, n_pad, r_pad, width, ld, inv2h2);
    return fit2 ? sample_go<2, 4, 2>(st, Fr, nur, nr_pad, Fp, nu, Om, S, n_pad, r_pad, width, ld, inv2h2)
                : sample_go<1, 8, 1>(st, Fr, nur, nr_pad, Fp, nu, Om, S, n_pad, r_pad, width, ld, inv2h2);
}

int sample_launch_rect(hipStream_t st, const double* Fr, const double* nur, int64_t nr_pad, const double* Fp,
                       const double* nu, int64_t n_pad, const double* Om, double* S, int r_pad, int s_pad, double h) {
    return sample_launch_window(st, Fr, nur, nr_pad, Fp, nu, n_pad, Om, S, r_pad, s_pad, s_pad, h);
}

int sample_launch(hipStream_t st, const double* Fp, const double* nu, const double* Om, double* S, int64_t n_pad,
                  int r_pad, int s_pad, double h) {
    return sample_launch_window(st, Fp, nu, n_pad, Fp, nu, n_pad, Om, S, r_pad, s_pad, s_pad, h);
}

int row_norms_launch(hipStream_t st, const double* Fp, double* nu, int64_t n_pad, int r_pad) {
    unsigned blocks = (unsigned)((n_pad + 3) / 4);
    hipLaunchKernelGGL(row_norms_kernel, dim3(blocks), dim3(256), 0, st, Fp, nu, n_pad, r_pad);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}

int gather_pad_rows_launch(hipStream_t st, const double* F, const int64_t* perm, double* Fp, int64_t n, int64_t n_pad,
                           int r, int r_pad) {
    int64_t total = n_pad * r_pad;
    hipLaunchKernelGGL(gather_pad_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, F, perm, Fp, n,
                       n_pad, r, r_pad);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}

int omega_fill_launch(hipStream_t st, double* Om, int64_t n, int64_t n_pad, int s, int s_pad, uint64_t seed) {
    int64_t total = n_pad * (s_pad / 2);
    hipLaunchKernelGGL(omega_fill_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, Om, n, n_pad, s, s_pad,
                       seed);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
}
