// Stand-alone driver of the C ABI (no Python): runs compress, factor, a few solves and a short ADMM run
// on seeded synthetic points.  It exists so that hardware-counter collection (rocprofv3 --pmc) can wrap
// a plain executable; the measured kernels and launch shapes are those of the library.
//
//   hss_bench_native n r s leaf h maxit [nsolve [key=value ...]]
//
// key=value pairs after nsolve are passed to hss_set_i64 before the compression (e.g. sampling=1 clustering=1
// adaptive_start=128), so that the same driver exercises every option of the library (it is also what the host
// sanitizer build of the library is run through).
//
// After the library calls it runs the library's hss_stream_copy three times on 2^27 doubles (1 GiB read,
// 1 GiB written per launch): the reference that converts the memory counters' raw readings into bytes.
// All device code lives in the library: the executable itself carries no kernel.
#include <hip/hip_runtime.h>

#include <chrono>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/hss_svm.h"


static uint64_t splitmix(uint64_t& s) {
    s += 0x9E3779B97F4A7C15ull;
    uint64_t z = s;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
static double uni(uint64_t& s) { return ((double)(splitmix(s) >> 11) + 0.5) / 9007199254740992.0; }
static double now() {
    return std::chrono::duration<double>(std::chrono::steady_clock::now().time_since_epoch()).count();
}
#define CHECK(x)                                                              \
    do {                                                                      \
        int rc_ = (x);                                                        \
        if (rc_ < 0) {                                                        \
            fprintf(stderr, "%s failed: %s (%d)\n", #x, hss_strerror(rc_), rc_); \
            return 1;                                                         \
        }                                                                     \
    } while (0)

int main(int argc, char** argv) {
    if (argc < 7) {
        fprintf(stderr, "usage: %s n r s leaf h maxit [nsolve]\n", argv[0]);
        return 2;
    }
    const int64_t n = atoll(argv[1]);
    const int r = atoi(argv[2]), s = atoi(argv[3]), leaf = atoi(argv[4]);
    const double h = atof(argv[5]);
    const int maxit = atoi(argv[6]);
    const int nsolve = argc > 7 ? atoi(argv[7]) : 5;
    std::vector<double> F((size_t)n * r), y(n);
    uint64_t sd = 2108;
    for (int64_t i = 0; i < n; ++i) {
        for (int f = 0; f < r; ++f) {
            double u1 = uni(sd), u2 = uni(sd);
            F[(size_t)i * r + f] = std::sqrt(-2.0 * std::log(u1)) * std::cos(6.283185307179586 * u2);
        }
        double sc = F[(size_t)i * r] + (r > 2 ? F[(size_t)i * r + 1] * F[(size_t)i * r + 2] : 0.0);
        y[i] = sc >= 0.0 ? 1.0 : -1.0;
    }
    double *dF, *dy, *dx;
    if (hipMalloc(&dF, sizeof(double) * n * r) != hipSuccess || hipMalloc(&dy, sizeof(double) * n) != hipSuccess ||
        hipMalloc(&dx, sizeof(double) * n) != hipSuccess)
        return 1;
    hipMemcpy(dF, F.data(), sizeof(double) * n * r, hipMemcpyHostToDevice);
    hipMemcpy(dy, y.data(), sizeof(double) * n, hipMemcpyHostToDevice);
    hipMemcpy(dx, y.data(), sizeof(double) * n, hipMemcpyHostToDevice);
    hss_ctx* ctx = nullptr;
    CHECK(hss_create(&ctx, nullptr));
    CHECK(hss_set_i64(ctx, "sample_width", s));
    for (int a = 8; a < argc; ++a) {
        const char* eq = strchr(argv[a], '=');
        if (!eq) {
            fprintf(stderr, "expected key=value, got %s\n", argv[a]);
            return 2;
        }
        const std::string key(argv[a], eq - argv[a]);
        CHECK(hss_set_i64(ctx, key.c_str(), atoll(eq + 1)));
    }
    double t0 = now();
    CHECK(hss_compress(ctx, dF, dy, n, r, h, leaf, 1e-3));
    hipDeviceSynchronize();
    double t1 = now();
    CHECK(hss_ulv_factor(ctx, 1.0));
    hipDeviceSynchronize();
    double t2 = now();
    for (int i = 0; i < nsolve; ++i) CHECK(hss_ulv_solve(ctx, dx, 1));
    hipDeviceSynchronize();
    double t3 = now();
    double bias = 0.0;
    int64_t nm = 0;
    CHECK(admm_svm_train(ctx, 1.0, 1.0, maxit, nullptr, nullptr, nullptr, &bias, &nm));
    double t4 = now();
    {   // the C-sweep in lockstep at another beta (re-factorization with the cached bases) and the label loop
        const double Cs[3] = {0.1, 1.0, 10.0};
        double b3[3];
        int64_t m3[3];
        double *dz = nullptr, *ddec = nullptr;
        if (hipMalloc(&dz, sizeof(double) * n * 3) != hipSuccess || hipMalloc(&ddec, sizeof(double) * 256) != hipSuccess) return 1;
        CHECK(admm_svm_train_multi(ctx, Cs, 3, 2.0, maxit, nullptr, dz, nullptr, b3, m3));
        CHECK(svm_decision(ctx, dF, n < 256 ? n : 256, dz + n, b3[1], ddec));
        double err = 0.0;
        CHECK(hss_error_estimate(ctx, 4, 7, &err));
        hipFree(dz);
        hipFree(ddec);
    }
    hss_stats_t st;
    CHECK(hss_stats(ctx, &st));
    printf("n %lld r %d s %d leaf %d: compress %.4f s (sampling kernel %.4f s, %.2f TFLOP/s), factor %.4f s, "
           "solve %.3f ms (%.1f GB/s), admm %d it %.4f s, bias %.6g, margin %lld, delta %.4g\n",
           (long long)n, r, s, leaf, t1 - t0, st.t_sample_kernel, st.sample_flops / st.t_sample_kernel / 1e12, t2 - t1,
           (t3 - t2) / nsolve * 1e3, st.factor_bytes / ((t3 - t2) / nsolve) / 1e9, maxit, t4 - t3, bias, (long long)nm,
           st.delta);
    {
        const size_t nd = (size_t)1 << 27;
        double *a = nullptr, *b = nullptr;
        if (hipMalloc(&a, nd * sizeof(double)) != hipSuccess || hipMalloc(&b, nd * sizeof(double)) != hipSuccess) return 1;
        hipMemset(a, 0, nd * sizeof(double));
        hipMemset(b, 0, nd * sizeof(double));
        hipDeviceSynchronize();
        double tc = now();
        for (int i = 0; i < 3; ++i) CHECK(hss_stream_copy(ctx, a, b, (int64_t)nd));
        if (hipDeviceSynchronize() != hipSuccess) return 1;
        printf("stream_copy_kernel: %.1f GB/s (read + write, 3 launches of 2 x 1 GiB)\n",
               3.0 * 2.0 * nd * sizeof(double) / (now() - tc) / 1e9);
        hipFree(a);
        hipFree(b);
    }
    hss_destroy(ctx);
    hipFree(dF);
    hipFree(dy);
    hipFree(dx);
    fflush(stdout);
    return 0;
}
