/* Entry points of libhsssvm_hooks.so: building blocks of libhsssvm driven one at a time by the GPU unit
 * tests (tests/test_gpu_blocks.py and friends).  Not part of the product; the shipped libhsssvm.so does not
 * export them.  "dev" / "host" say where a pointer lives; `stream` is a hipStream_t (0 = null stream).
 * Every call returns 0 or a negative HSS_E* code and synchronises the stream before returning. */
#ifndef HSS_TEST_HOOKS_H
#define HSS_TEST_HOOKS_H
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif
int hsx_probe_mfma(const double* a_dev, const double* b_dev, double* d_dev);
int hsx_bgemm(void* stream, int nitems, const int32_t* dims_host, const int64_t* offs_host, double* base_dev, int transA,
              int transB, double alpha, double beta);
int hsx_inverse(void* stream, int nmat, const int32_t* n_host, const int64_t* offs_host, double* base_dev,
                int32_t* flags_out_host);
int hsx_chol(void* stream, int nmat, const int32_t* n_host, const int64_t* offs_host, double* base_dev);
int hsx_row_id(void* stream, const double* A_dev, int32_t ld, int32_t nnodes, const int64_t* moff_host, int32_t kcap,
               double rel, double abs_tol, int32_t gram, int32_t* ranks_host, int32_t* J_host, double* U_dev);
int hsx_row_id_blocks(void* stream, const double* A_dev, int32_t ld, int32_t nnodes, const int64_t* moff_host, int32_t kcap,
                      double rel, double abs_tol, int32_t gram, int32_t rows_per_block, int32_t* ranks_host,
                      int32_t* J_host, double* U_dev);
int hsx_omega(void* stream, double* Om_dev, int64_t n, int32_t s, uint64_t seed);
#ifdef __cplusplus
}
#endif
#endif
