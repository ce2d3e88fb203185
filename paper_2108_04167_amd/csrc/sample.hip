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
// The K tile and the F_j tile are double buffered in LDS: one barrier per j-block.
#include "common.h"

namespace {

constexpr int BN = 32;          // points per j-block
constexpr int MAXF = 8;         // F_j tile elements staged per thread (32 * r_pad <= 8 * 512)

template <int WR, int WC, int CT>
__global__ __launch_bounds__(512) void sample_kernel(const double* __restrict__ Fp, const double* __restrict__ nu,
                                                      const double* __restrict__ Om, double* __restrict__ S,
                                                      int n_pad, int r_pad, int s_pad, double inv2h2) {
    static_assert(WR * WC == 8, "8 wavefronts");
    constexpr int BMR = 64 * WR;           // rows of S per workgroup
    constexpr int LDK = BMR + 16;          // leading dimension of the K tile (j-major)
    extern __shared__ double smem[];
    const int ldf = r_pad + 1;
    double* Fi_s = smem;                           // BMR x ldf
    double* Fj_s = Fi_s + BMR * ldf;               // 2 x BN x ldf
    double* nui_s = Fj_s + 2 * BN * ldf;           // BMR
    double* nuj_s = nui_s + BMR;                   // 2 x BN
    double* K_s = nuj_s + 2 * BN;                  // 2 x BN x LDK

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int lr = lane & 15, lk = lane >> 4;
    const int wr = wave / WC, wc = wave % WC;
    const int row0 = blockIdx.x * BMR;
    const int col0 = (blockIdx.y * WC + wc) * (16 * CT);
    const int NJ = n_pad / BN;
    const int tile_elems = BN * r_pad;

    // ---- prologue: F_i tile, nu_i, F_j tiles 0 and 1 ----
    for (int idx = tid; idx < BMR * r_pad; idx += 512) {
        int rr = idx / r_pad, cc = idx - rr * r_pad;
        Fi_s[rr * ldf + cc] = Fp[(size_t)row0 * r_pad + idx];
    }
    for (int idx = tid; idx < BMR; idx += 512) nui_s[idx] = nu[row0 + idx];
    for (int b = 0; b < 2; ++b) {
        int jb = b < NJ ? b : NJ - 1;
        for (int idx = tid; idx < tile_elems; idx += 512) {
            int rr = idx / r_pad, cc = idx - rr * r_pad;
            Fj_s[(b * BN + rr) * ldf + cc] = Fp[(size_t)jb * tile_elems + idx];
        }
        if (tid < BN) nuj_s[b * BN + tid] = nu[jb * BN + tid];
    }
    __syncthreads();

    // Gram + exp of one K tile (block jb, LDS buffer buf).  The tile has (4*WR) x 2 MFMA tiles;
    // wavefront w computes tiles w*WR .. w*WR+WR-1.
    auto make_ktile = [&](int buf) {
        const double* Fj = Fj_s + buf * BN * ldf;
        const double* nj = nuj_s + buf * BN;
        double* Kt = K_s + buf * BN * LDK;
#pragma unroll
        for (int u = 0; u < WR; ++u) {
            int t = wave * WR + u;
            int rt = t >> 1, ct = t & 1;
            v4d g = (v4d){0.0, 0.0, 0.0, 0.0};
            const double* ap = Fi_s + (rt * 16 + lr) * ldf + lk;
            const double* bp = Fj + (ct * 16 + lr) * ldf + lk;
            for (int ks = 0; ks < r_pad; ks += 4) g = __builtin_amdgcn_mfma_f64_16x16x4f64(ap[ks], bp[ks], g, 0, 0, 0);
            double nuj = nj[ct * 16 + lr];
            // accumulator register v of lane (lk, lr) is G[4*v + lk][lr]
            double* kp = Kt + (ct * 16 + lr) * LDK + rt * 16 + lk;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                double d2 = nui_s[rt * 16 + 4 * v + lk] + nuj - 2.0 * g[v];
                d2 = d2 > 0.0 ? d2 : 0.0;
                kp[4 * v] = exp(-d2 * inv2h2);
            }
        }
    };

    v4d acc[4][CT];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < CT; ++j) acc[i][j] = (v4d){0.0, 0.0, 0.0, 0.0};

    // Omega register ring, four k-steps deep: slot ks%4 holds Omega[jb*32 + ks*4 + lk][col0 + CT*lr + ct];
    // a slot is refilled for the k-step four ahead right after it has been consumed.
    double om[4][CT];
    auto load_omega = [&](const double* op, int kstep, int ks) {
        const double* q = op + (size_t)kstep * 4 * s_pad;
        if constexpr (CT == 4) {
            double2 q0 = reinterpret_cast<const double2*>(q)[0], q1 = reinterpret_cast<const double2*>(q)[1];
            om[ks][0] = q0.x; om[ks][1] = q0.y; om[ks][2] = q1.x; om[ks][3] = q1.y;
        } else if constexpr (CT == 2) {
            double2 q0 = reinterpret_cast<const double2*>(q)[0];
            om[ks][0] = q0.x; om[ks][1] = q0.y;
        } else {
            om[ks][0] = q[0];
        }
    };
    {
        const double* op = Om + (size_t)lk * s_pad + col0 + CT * lr;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) load_omega(op, ks, ks);
    }
    make_ktile(0);
    __syncthreads();

    double fj[MAXF];
    double nuj_next = 0.0;
    for (int jb = 0; jb < NJ; ++jb) {
        const int cur = jb & 1, nxt = cur ^ 1;
        // stage F_j tile jb+2 in registers (stored to LDS at the end of this iteration)
        const int jb2 = jb + 2 < NJ ? jb + 2 : NJ - 1;
#pragma unroll
        for (int u = 0; u < MAXF; ++u) {
            int idx = tid + u * 512;
            fj[u] = idx < tile_elems ? Fp[(size_t)jb2 * tile_elems + idx] : 0.0;
        }
        if (tid < BN) nuj_next = nu[jb2 * BN + tid];

        if (jb + 1 < NJ) make_ktile(nxt);

        // contraction with K tile jb
        const double* Kt = K_s + cur * BN * LDK + wr * 64 + lr;
        const int jbn = jb + 1 < NJ ? jb + 1 : jb;
        const double* op_cur = Om + ((size_t)jb * BN + lk) * s_pad + col0 + CT * lr;
        const double* op_nxt = Om + ((size_t)jbn * BN + lk) * s_pad + col0 + CT * lr;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const double* kp = Kt + (ks * 4 + lk) * LDK;
            double a0 = kp[0], a1 = kp[16], a2 = kp[32], a3 = kp[48];
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                double b = om[ks & 3][ct];
                acc[0][ct] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b, acc[0][ct], 0, 0, 0);
                acc[1][ct] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b, acc[1][ct], 0, 0, 0);
                acc[2][ct] = __builtin_amdgcn_mfma_f64_16x16x4f64(a2, b, acc[2][ct], 0, 0, 0);
                acc[3][ct] = __builtin_amdgcn_mfma_f64_16x16x4f64(a3, b, acc[3][ct], 0, 0, 0);
            }
            if (ks < 4) load_omega(op_cur, ks + 4, ks);
            else load_omega(op_nxt, ks - 4, ks - 4);
        }

        // publish F_j tile jb+2 into the buffer tile jb used
#pragma unroll
        for (int u = 0; u < MAXF; ++u) {
            int idx = tid + u * 512;
            if (idx < tile_elems) {
                int rr = idx / r_pad, cc = idx - rr * r_pad;
                Fj_s[(cur * BN + rr) * ldf + cc] = fj[u];
            }
        }
        if (tid < BN) nuj_s[cur * BN + tid] = nuj_next;
        __syncthreads();
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
    return sizeof(double) * ((size_t)bmr * ldf + 2 * BN * ldf + bmr + 2 * BN + 2 * BN * (bmr + 16));
}

template <int WR, int WC, int CT>
int sample_go(hipStream_t st, const double* Fp, const double* nu, const double* Om, double* S, int64_t n_pad,
              int r_pad, int s_pad, double inv2h2) {
    size_t smem = sample_smem<WR>(r_pad);
    auto kern = sample_kernel<WR, WC, CT>;
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)smem));
    dim3 grid((unsigned)(n_pad / (64 * WR)), (unsigned)(s_pad / (16 * CT * WC)));
    hipLaunchKernelGGL(kern, grid, dim3(512), smem, st, Fp, nu, Om, S, (int)n_pad, r_pad, s_pad, inv2h2);
    HIP_TRY(hipGetLastError());
    return HSS_OK;
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

int sample_launch(hipStream_t st, const double* Fp, const double* nu, const double* Om, double* S, int64_t n_pad,
                  int r_pad, int s_pad, double h) {
    if (n_pad % 256 || r_pad % 4 || r_pad < 4 || r_pad > 96 || s_pad % 128 || s_pad < 128) return HSS_EUNSUPPORTED;
    const double inv2h2 = 1.0 / (2.0 * h * h);
    // Widest block of S per workgroup whose column span divides s_pad and whose LDS footprint fits:
    // 64 x 512, else 128 x 256 (64 x 256 when the feature tiles are too large), else 128 x 128 (64 x 128).
    const size_t lds_cap = 150 * 1024;
    const bool fit2 = sample_smem<2>(r_pad) <= lds_cap;
    if (sample_smem<1>(r_pad) > lds_cap) return HSS_EUNSUPPORTED;
    if (s_pad % 512 == 0) return sample_go<1, 8, 4>(st, Fp, nu, Om, S, n_pad, r_pad, s_pad, inv2h2);
    if (s_pad % 256 == 0)
        return fit2 ? sample_go<2, 4, 4>(st, Fp, nu, Om, S, n_pad, r_pad, s_pad, inv2h2)
                    : sample_go<1, 8, 2>(st, Fp, nu, Om, S, n_pad, r_pad, s_pad, inv2h2);
    return fit2 ? sample_go<2, 4, 2>(st, Fp, nu, Om, S, n_pad, r_pad, s_pad, inv2h2)
                : sample_go<1, 8, 1>(st, Fp, nu, Om, S, n_pad, r_pad, s_pad, inv2h2);
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
