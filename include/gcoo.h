/*
 * gcoo.h - C ABI of the grouped-COO (GCOO) sparse x dense multiplication library for
 * AMD Instinct MI355X (gfx950).
 *
 * The library computes C = A x B in fp32 (Equation 1 of the paper, Section 2), with
 * A (m x k, sparse) held on the device in the GCOO layout of Section 3.1 and B (k x N), C (m x N)
 * dense and row-major.  All compute runs in HIP kernels on the device that is current when a
 * function is called; there is no CPU path.
 *
 * Layout conventions.  A is cut into g = (m + p - 1) / p groups of p consecutive rows
 * (Algorithm 1 derives the group count from the height of A; the last group holds
 * m - (g-1)p rows).  Each group is a COO list ordered by column, then row, then position in
 * the input; the lists are concatenated into values[nnz] (fp32), rows[nnz], cols[nnz] (int32,
 * 0-based, absolute coordinates).  gIdxes[q] is the position of the first entry of group q,
 * with one extra entry gIdxes[g] = nnz; nnzPerGroup[q] is the number of entries of group q.
 *
 * Memory ownership.  The library never allocates or frees device memory.  The caller
 * allocates one device buffer of gcoo_device_bytes() bytes (256-byte aligned), hands it to a
 * gcoo_from_* call and keeps it alive, unmodified, until gcoo_free() of the handle and until
 * every gcoo_spdm() launched on it has finished.  The handle itself is a small host object owned
 * by the library.
 *
 * Streams.  `stream` arguments are hipStream_t values passed as void* (NULL = the default
 * stream).  Kernels are launched on that stream and the call returns without waiting, except
 * where a function says that it synchronises.
 *
 * Errors.  Every function returning int returns GCOO_OK (0) or a negative gcoo_status.  On error
 * no handle is produced and C is not written by the failing call.  No C++ exception crosses
 * this boundary.
 *
 * Threads.  A handle is complete when its gcoo_from_* call returns and is never modified afterwards:
 * gcoo_spdm*, gcoo_info and gcoo_export* only read it, so any number of host threads may use one
 * handle at once, on any streams (each caller orders its own streams behind the conversion).
 * Distinct handles are independent.  gcoo_free() must not run while another call still uses the
 * handle.  gcoo_set_share_policy() is process-wide; it may be called from any thread at any time, and a
 * conversion uses, for all of its work, the value it finds when it starts.
 */
#ifndef GCOO_H
#define GCOO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum gcoo_status {
    GCOO_OK = 0,
    GCOO_EINVAL = -1,   /* null pointer, negative size, p outside [1, GCOO_MAX_P], ld < N, misaligned buffer,
                           nnz or a dimension above INT32_MAX, unknown variant */
    GCOO_EBOUNDS = -2,  /* host-side validation: row_ptr not non-decreasing from 0, or a column outside [0, k) */
    GCOO_ENOMEM = -3,   /* dev_buf smaller than gcoo_device_bytes() for this input */
    GCOO_EHIP = -4,     /* a HIP runtime call failed; gcoo_last_hip_error() holds its text */
    GCOO_ELIMIT = -5    /* gcoo_from_csr_device_static(): more stored entries than its fixed scratch serves */
} gcoo_status;

/* Largest supported group height p (rows per group). */
#define GCOO_MAX_P 256

/* Opaque host-side handle of one converted matrix. */
typedef struct gcoo_matrix gcoo_matrix;

/*
 * Group height to use when the caller has no better idea (the paper leaves p to a tuner, Section 5).
 * 32 is the tallest group the widest instance of the register kernel holds (32 rows x 4 columns
 * per lane); on MI355X it was the fastest of {4, 8, 16, 32, 64} for that kernel for uniform random
 * matrices of density 0.001 .. 0.5, for a power-law row-length matrix and for a diagonal one.
 * Where gcoo_spdm() will run the workgroup-shared kernel (GCOO_VARIANT_SHARE: N a multiple of 4,
 * density at most 6 %, and at least 1.5 % from 3500 columns on, 0.8 % from 5500, 0.35 % from 7000; never while
 * the policy is GCOO_SHARE_NEVER), a height between
 * 24 and 48 is returned that makes the workgroups of that kernel (one per 8p rows x 256 columns of C)
 * fill whole rounds over the 256 compute units: the p that minimises
 * ceil(workgroups / 256) x (p + 24).
 * 38, the tallest group the register kernel holds with four columns per lane (its second
 * accumulator layout), is returned between 6 % and 12 % density from 5000 columns on (N a multiple
 * of 4): there most groups touch most columns and fewer, taller groups fetch fewer rows of B.
 * A caller that multiplies the same matrix many times can do better by timing a few values (the
 * Python binding has gcoo_tune_p for that).  Pure host arithmetic; 0 for invalid arguments.
 */
int32_t gcoo_default_p(int64_t m, int64_t k, int64_t nnz, int64_t N);

/*
 * Device bytes a gcoo_from_csr() / gcoo_from_dense() call needs in dev_buf for an m x k matrix
 * with nnz stored entries and group height p: the five arrays of Section 3.1 (Table 1:
 * 3*nnz + 2*g elements, plus one sentinel), the kernel-private schedules derived from them (the run
 * schedule of the register kernel, at most 3*nnz + 2048*g + 128 words; where gcoo_set_share_policy()
 * asks for it the share schedule of the workgroup-shared kernel) and the scratch space the
 * conversion kernels use; for p > 64 also a second copy of the matrix regrouped at 32 rows with its
 * schedules, which is what the fast kernels multiply with (they hold at most 64 rows of partial sums).
 * Returns 0 for invalid arguments.  Pure host arithmetic.
 */
size_t gcoo_device_bytes(int64_t m, int64_t k, int64_t nnz, int32_t p);

/*
 * Section 3.1 / Algorithm 1 for a CSR input: convert an m x k CSR matrix to GCOO on the device.
 *   row_ptr[m+1]  0-based, non-decreasing, row_ptr[0] = 0, nnz = row_ptr[m]
 *   col_idx[nnz]  each in [0, k); columns of a row may be unsorted and may repeat
 *   vals[nnz]     fp32; every stored entry is kept, explicit zeros included (nnz is preserved)
 *   src_on_device 0: the three arrays are host pointers (validated, then copied to the device);
 *                 1: device pointers (not validated; row_ptr[m] is read back, which synchronises
 *                    `stream`)
 *   p             rows per group, 1..GCOO_MAX_P
 *   dev_buf       caller-owned device memory, 256-byte aligned, >= gcoo_device_bytes(m,k,nnz,p)
 * The conversion kernels (group index from row_ptr, then a stable per-group radix sort on the
 * column) run on `stream`.  With host input the call returns after the input has been copied
 * (the copies synchronise); the kernels may still be running.  *out receives the handle.
 * Degenerate shapes (m = 0, nnz = 0) succeed.
 */
int gcoo_from_csr(int64_t m, int64_t k,
                  const int32_t* row_ptr, const int32_t* col_idx, const float* vals,
                  int src_on_device, int32_t p,
                  void* dev_buf, size_t dev_buf_bytes, void* stream,
                  gcoo_matrix** out);

/*
 * gcoo_from_csr() for a CSR matrix that is already on the device, by a caller who knows nnz (the
 * one who sized dev_buf with it).  Nothing is read back: the call only launches kernels on `stream`
 * and returns.  row_ptr_dev[m] must equal nnz; if it does not, the result is unspecified but every
 * kernel stays inside the arrays (offsets are clamped to nnz).  Columns are not validated for
 * device input, but a column outside [0, k) is stored clamped into that range, so that no
 * kernel reads outside B; gcoo_export() reports GCOO_EBOUNDS for such a matrix.
 */
int gcoo_from_csr_device(int64_t m, int64_t k, int64_t nnz,
                         const int32_t* row_ptr_dev, const int32_t* col_idx_dev, const float* vals_dev,
                         int32_t p, void* dev_buf, size_t dev_buf_bytes, void* stream,
                         gcoo_matrix** out);

/*
 * gcoo_from_csr_device() for callers that may not allocate device memory beyond what they hand over as
 * output - code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  out_buf
 * (256-byte aligned, >= gcoo_static_handle_bytes(m, k, nnz, p)) receives only what the handle keeps:
 * the five arrays, the statistics and the schedules.  What the conversion needs beyond that (the second
 * buffer of the radix sort, 12 bytes per stored entry, and a counter) is a fixed array inside the
 * library, 24 MiB + 256 bytes per device, held until the process ends; hence the limit
 *   nnz <= GCOO_STATIC_MAX_NNZ, else GCOO_ELIMIT (gcoo_static_handle_bytes() then returns 0).
 * The call allocates and frees no device memory and copies nothing back; it launches the same
 * kernels as gcoo_from_csr_device() and produces the same arrays, schedules and products.
 * Every call on a device uses that device's one array: two such conversions that overlap in time on
 * one GPU (other streams, other threads) race on it and give unspecified arrays; a second call
 * may start once the kernels of the first have finished.
 */
#define GCOO_STATIC_MAX_NNZ 2097152
size_t gcoo_static_handle_bytes(int64_t m, int64_t k, int64_t nnz, int32_t p);
int gcoo_from_csr_device_static(int64_t m, int64_t k, int64_t nnz,
                                const int32_t* row_ptr_dev, const int32_t* col_idx_dev, const float* vals_dev,
                                int32_t p, void* out_buf, size_t out_buf_bytes, void* stream,
                                gcoo_matrix** out);

/*
 * Algorithm 1, step 1: count the entries of a dense device matrix A_dev (m x k, row-major,
 * leading dimension lda >= k) that are not equal to zero.  Writes the count to *nnz (host).
 * Synchronises `stream`.  Used to size dev_buf before gcoo_from_dense().
 */
int gcoo_dense_nnz(int64_t m, int64_t k, const float* A_dev, int64_t lda, void* stream, int64_t* nnz);

/*
 * Algorithm 1 (both steps) for a dense device matrix: count per group, prefix sum, then fill
 * values/rows/cols.  An entry is stored when it is != 0.0f (so +0 and -0 are dropped, NaN is
 * kept).  Synchronises `stream` once, between the two steps, to learn nnz and check that
 * dev_buf is large enough (GCOO_ENOMEM otherwise).
 */
int gcoo_from_dense(int64_t m, int64_t k, const float* A_dev, int64_t lda, int32_t p,
                    void* dev_buf, size_t dev_buf_bytes, void* stream,
                    gcoo_matrix** out);

/*
 * Algorithm 2 (GCOOSpDM): C = A x B, alpha = 1, beta = 0; every element of C (m x N) is
 * overwritten, rows of empty groups with +0.
 *   B_dev  k x N row-major device matrix, leading dimension ldb >= N
 *   C_dev  m x N row-major device matrix, leading dimension ldc >= N; must not overlap B_dev
 * Entries that A does not store are skipped, never multiplied (a non-finite value in a row of B
 * that no stored entry touches does not reach C).  The summation order inside one element of C
 * is fixed by the matrix, p and the kernel variant, never by timing: results are the same bits
 * from run to run.
 * Asynchronous on `stream`: the call launches kernels and returns, it never waits for the device,
 * copies nothing back and allocates nothing, so it may be recorded into a stream capture.
 * N = 0 or m = 0 is a no-op success.  The handle is only read.
 */
int gcoo_spdm(const gcoo_matrix* A, const float* B_dev, int64_t ldb, int64_t N,
              float* C_dev, int64_t ldc, void* stream);

/*
 * gcoo_spdm() with the kernel chosen by the caller instead of the built-in heuristic
 * (Section 5 of the paper leaves the choice of launch parameters to a tuner).
 *   variant  GCOO_VARIANT_AUTO, or one of the GCOO_VARIANT_* below.  A variant that does not
 *            support this matrix/shape returns GCOO_EINVAL.
 */
#define GCOO_VARIANT_AUTO 0
#define GCOO_VARIANT_LDS  1  /* partial sums in LDS, reads the five arrays directly; any p, any alignment */
/* partial sums in VGPRs, reads the run schedule built at conversion; needs N >= 4 (p <= 38 and p > 64:
 * four columns per lane) or N >= 2 (39 <= p <= 64: two), else GCOO_EINVAL.  A matrix of groups taller than
 * 64 rows is multiplied through a second, kernel-private copy regrouped at 32 rows that the conversion keeps
 * behind the five arrays (gcoo_device_bytes() counts it); GCOO_VARIANT_SHARE works on that copy too.  Any N, ldb, ldc and base
 * addresses: where N is not a multiple of the columns per lane, the lane at the end of a row computes the
 * last columns of the row instead of reaching beyond N, and rows aligned to 4 bytes only are read and
 * written with unaligned 16-byte accesses (a few per cent slower than aligned ones).  No access leaves
 * the first N columns of a row.  Groups with very many entries are shared by the waves of a workgroup
 * except for 33 <= p <= 38 */
#define GCOO_VARIANT_REG  2
/* the eight groups of a workgroup (a super-group, up to 8 x 48 rows of A) fetch each row of B that
 * any of them needs once into LDS, and every multiply-add takes its B values from there; reads the
 * share schedule built at conversion (see gcoo_set_share_policy()); needs p <= 48, B, C, ldb, ldc, N
 * multiples of 4 elements (16-byte aligned rows) and k * ldb * 4 < 2^32, else GCOO_EINVAL.
 * gcoo_spdm() picks it where the matrix has that schedule by the automatic rule, the operands
 * qualify and C has at least 192 blocks of (8p rows) x 256 columns - below 9000 columns of A also
 * only if those blocks fill their rounds over the 256 compute units to 80 % */
#define GCOO_VARIANT_SHARE 3
int gcoo_spdm_variant(const gcoo_matrix* A, const float* B_dev, int64_t ldb, int64_t N,
                      float* C_dev, int64_t ldc, void* stream, int variant);

/* Variant gcoo_spdm() would pick for this matrix and these operand shapes (one of GCOO_VARIANT_* > 0). */
int gcoo_spdm_pick(const gcoo_matrix* A, const float* B_dev, int64_t ldb, int64_t N,
                   const float* C_dev, int64_t ldc);

/* Release the host handle.  The device buffer stays the caller's.  NULL is accepted. */
int gcoo_free(gcoo_matrix* A);

/* Shape of a handle: any output pointer may be NULL. */
int gcoo_info(const gcoo_matrix* A, int64_t* m, int64_t* k, int64_t* nnz, int32_t* p, int64_t* g);

/*
 * Copy the five arrays of Section 3.1 to HOST buffers: values[nnz], rows[nnz], cols[nnz],
 * gIdxes[g+1] (widened to int64), nnzPerGroup[g].  Any pointer may be NULL to skip that array.
 * Waits for the conversion kernels on `stream` first (synchronises).  GCOO_EBOUNDS (after the
 * copies) if the conversion met a column outside [0, k) in a device CSR input and clamped it.
 */
int gcoo_export(const gcoo_matrix* A, float* values, int32_t* rows, int32_t* cols,
                int64_t* gIdxes, int32_t* nnzPerGroup, void* stream);

/*
 * When conversions build the share schedule (process-wide setting, not thread-safe; takes effect
 * for matrices converted afterwards).
 * GCOO_SHARE_AUTO: only for matrices on which gcoo_spdm() then picks GCOO_VARIANT_SHARE when B is
 *   wide enough: p <= 48, density at most 6 %, and at least 1.5 % from 3500 columns on, 0.8 % from 5500, 0.35 % from
 *   7000 (at most 262144 columns);
 * GCOO_SHARE_ALWAYS: whenever that kernel could run (p <= 48, at most 262144 columns, nnz > 0);
 *   gcoo_spdm() keeps its usual choice and GCOO_VARIANT_SHARE must be asked for;
 * GCOO_SHARE_NEVER: never.
 */
#define GCOO_SHARE_AUTO   0
#define GCOO_SHARE_ALWAYS 1
#define GCOO_SHARE_NEVER  2
int gcoo_set_share_policy(int policy);

/*
 * Introspection for tests: copies the share schedule (the kernel-private re-listing that the
 * workgroup-shared SpDM kernel reads) to HOST buffers, any of which may be NULL.
 * *hdr_words and *block_count receive the sizes of `hdr` (32-bit words) and `blocks` (blocks of 64 words);
 * call once with the arrays NULL to learn them.  sbase has 8 * ceil(g / 8) entries, ucount ceil(g / 8),
 * ucols nnz (the distinct columns of super-group Q start at index gIdxes[8Q]).  Synchronises `stream`.
 * GCOO_EINVAL if A is NULL or has no share schedule.
 */
int gcoo_export_share(const gcoo_matrix* A, uint32_t* hdr, uint32_t* blocks, int32_t* sbase, int32_t* ucount, int32_t* ucols,
                      int64_t* hdr_words, int64_t* block_count, void* stream);

/* Static text for a status code. */
const char* gcoo_strerror(int status);

/* Text of the last HIP error seen by the calling thread inside this library ("" if none). */
const char* gcoo_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* GCOO_H */
