/*
 * gcoo_baseline.h - C ABI of libgcoo_baseline.so: context for benchmarks, not part of the GCOO path.
 *
 * A plain CSR row-split SpMM (one wave per row and 256 columns, no staging, no reuse of B across
 * rows), the kind of routine Section 4 of the paper compares GCOOSpDM against.  The sweeps of the
 * benchmark time it next to the GCOO path; nothing in libgcoo.so uses it.
 */
#ifndef GCOO_BASELINE_H
#define GCOO_BASELINE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * C = A x B for a CSR matrix A (m x k) on the device; B (k x N) and C (m x N) row-major with leading
 * dimensions ldb, ldc >= N.  All pointers are device pointers; C is fully overwritten.  Asynchronous
 * on `stream` (a hipStream_t passed as void*).  Returns 0, -1 for invalid arguments, -4 if the launch failed.
 */
int gcoo_csr_spmm_baseline(int64_t m, int64_t k, const int32_t* row_ptr_dev, const int32_t* col_idx_dev,
                           const float* vals_dev, const float* B_dev, int64_t ldb, int64_t N,
                           float* C_dev, int64_t ldc, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* GCOO_BASELINE_H */
