/*
 * CPU oracle for the grouped-COO (GCOO) sparse x dense product.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * GPU library must compute.  It is used by the tests, by the smoke check and by
 * the benchmark's reported CPU baseline; the GPU library never links, loads or
 * calls it, and it shares no source, header, table or helper with that library.
 *
 * Conventions (the readings of the paper taken here are listed with each
 * function): A is m x k, B is k x N row-major with leading dimension ldb,
 * C is m x N row-major.  Indices are 0-based int32, values fp32, sums fp64.
 * A "group" is a band of p consecutive rows of A (Algorithm 1 derives the
 * number of groups from the height of A; Algorithm 2 uses blockIdx.x*p as the
 * first row of C written by a block).  Inside a group, entries are ordered by
 * column, then row, then position in the input: that is the order in which
 * Algorithm 2's search for "the next entry with the same col" finds the entries
 * that share a column next to each other.
 *
 * Every function is pinned by tests/test_oracle_*.py against values printed in
 * the paper (Section 2.3 and Section 3.1 examples), closed forms (group count,
 * footprint), library formats (CSR for p = 1, CSC for p >= m) and brute force.
 * No function here is "parity unpinned".
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Section 3.1: number of groups g = floor((n + p - 1) / p). */
int64_t oracle_group_count(int64_t n, int64_t p)
{
    return (n + p - 1) / p;
}

/* Section 3.1: every group has p lines except the last, which has n - (g-1)p. */
int64_t oracle_last_group_width(int64_t n, int64_t p)
{
    int64_t g = oracle_group_count(n, p);
    return g == 0 ? 0 : n - (g - 1) * p;
}

/* Table 1: GCOO stores 3*nnz + 2*g elements. */
int64_t oracle_gcoo_footprint_elems(int64_t n, int64_t p, int64_t nnz)
{
    return 3 * nnz + 2 * oracle_group_count(n, p);
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Section 2.3: COO of a row-major dense matrix.  Entries are listed in the
 * order a row-major scan meets them; an entry is stored when it is not equal
 * to zero.  Returns nnz; arrays may be NULL to count only.
 */
int64_t oracle_coo_from_dense(int64_t m, int64_t k, const float *A, int64_t lda,
                              float *values, int32_t *rows, int32_t *cols)
{
    int64_t n = 0;
    for (int64_t i = 0; i < m; ++i)
        for (int64_t j = 0; j < k; ++j) {
            float a = A[i * lda + j];
            if (a != 0.0f) {
                if (values) { values[n] = a; rows[n] = (int32_t)i; cols[n] = (int32_t)j; }
                ++n;
            }
        }
    return n;
}

/* One stored entry with everything its place in GCOO depends on. */
typedef struct {
    int64_t group;
    int32_t col;
    int32_t row;
    int64_t pos;   /* position in the input, so that equal (group,col,row) keep input order */
    float   val;
} entry_t;

static int entry_cmp(const void *pa, const void *pb)
{
    const entry_t *a = (const entry_t *)pa, *b = (const entry_t *)pb;
    if (a->group != b->group) return a->group < b->group ? -1 : 1;
    if (a->col != b->col) return a->col < b->col ? -1 : 1;
    if (a->row != b->row) return a->row < b->row ? -1 : 1;
    if (a->pos != b->pos) return a->pos < b->pos ? -1 : 1;
    return 0;
}

/*
 * Section 3.1 (format) applied to a CSR input.  Every stored entry is kept
 * (explicit zeros and repeated coordinates included), so nnz is preserved.
 * Output: values/rows/cols of length nnz, the concatenation of the groups'
 * COO lists; gIdxes[g+1] with gIdxes[q] = first position of group q and
 * gIdxes[g] = nnz; nnzPerGroup[g].  The first g entries of gIdxes are the
 * paper's array; the extra last one is a sentinel.
 * Returns 0, or -1 on malformed input.
 */
int oracle_gcoo_from_csr(int64_t m, int64_t k, const int32_t *row_ptr, const int32_t *col_idx,
                         const float *vals, int32_t p,
                         float *values, int32_t *rows, int32_t *cols,
                         int32_t *gIdxes, int32_t *nnzPerGroup)
{
    if (m < 0 || k < 0 || p < 1) return -1;
    int64_t nnz = m > 0 ? row_ptr[m] : 0;
    int64_t g = oracle_group_count(m, p);
    entry_t *e = (entry_t *)malloc((size_t)(nnz > 0 ? nnz : 1) * sizeof(entry_t));
    if (!e) return -1;
    for (int64_t i = 0; i < m; ++i)
        for (int64_t q = row_ptr[i]; q < row_ptr[i + 1]; ++q) {
            if (col_idx[q] < 0 || col_idx[q] >= k) { free(e); return -1; }
            e[q].group = i / p;
            e[q].col = col_idx[q];
            e[q].row = (int32_t)i;
            e[q].pos = q;
            e[q].val = vals[q];
        }
    qsort(e, (size_t)nnz, sizeof(entry_t), entry_cmp);   /* the key is a total order */
    for (int64_t q = 0; q < g; ++q) nnzPerGroup[q] = 0;
    for (int64_t q = 0; q < nnz; ++q) {
        values[q] = e[q].val;
        rows[q] = e[q].row;
        cols[q] = e[q].col;
        nnzPerGroup[e[q].group] += 1;
    }
    int64_t run = 0;
    for (int64_t q = 0; q < g; ++q) { gIdxes[q] = (int32_t)run; run += nnzPerGroup[q]; }
    gIdxes[g] = (int32_t)run;
    free(e);
    return 0;
}

/*
 * Algorithm 1, step 1 (count): scan the dense matrix and produce nnz,
 * nnzPerGroup and gIdxes.  An entry counts when it is not equal to zero.
 * Returns nnz.
 */
int64_t oracle_gcoo_count_dense(int64_t m, int64_t k, const float *A, int64_t lda, int32_t p,
                                int32_t *gIdxes, int32_t *nnzPerGroup)
{
    int64_t g = oracle_group_count(m, p);
    for (int64_t q = 0; q < g; ++q) nnzPerGroup[q] = 0;
    for (int64_t i = 0; i < m; ++i)
        for (int64_t j = 0; j < k; ++j)
            if (A[i * lda + j] != 0.0f) nnzPerGroup[i / p] += 1;
    int64_t run = 0;
    for (int64_t q = 0; q < g; ++q) { gIdxes[q] = (int32_t)run; run += nnzPerGroup[q]; }
    gIdxes[g] = (int32_t)run;
    return run;
}

/*
 * Algorithm 1, step 2 (fill): scan the dense matrix again and write each
 * nonzero with its coordinates to its slot.  Within a group the scan goes
 * column by column and, inside a column, down the rows of the band, which
 * yields the (col, row) order directly.
 */
void oracle_gcoo_fill_dense(int64_t m, int64_t k, const float *A, int64_t lda, int32_t p,
                            const int32_t *gIdxes,
                            float *values, int32_t *rows, int32_t *cols)
{
    int64_t g = oracle_group_count(m, p);
    for (int64_t q = 0; q < g; ++q) {
        int64_t at = gIdxes[q];
        int64_t r0 = q * p, r1 = r0 + p < m ? r0 + p : m;
        for (int64_t j = 0; j < k; ++j)
            for (int64_t i = r0; i < r1; ++i) {
                float a = A[i * lda + j];
                if (a != 0.0f) { values[at] = a; rows[at] = (int32_t)i; cols[at] = (int32_t)j; ++at; }
            }
    }
}

/*
 * Equation 1 restricted to the stored entries of a CSR matrix:
 *   C64(i,j) = sum over stored entries e of row i of  (double)val(e) * (double)B(col(e), j)
 *   D64(i,j) = sum over the same entries of |val(e)| * |B(col(e), j)|
 * Entries that are not stored contribute nothing (Section 1: a zero entry
 * times any number adds nothing and is skipped).  D64 is the scale against
 * which the fp32 result is judged; it may be NULL.
 * Rows [r0, r1) only are computed and written to C64/D64 rows 0..r1-r0-1
 * (leading dimension N), so that a sample of rows can be checked at full size.
 */
void oracle_spdm_csr(int64_t k, int64_t N, const int32_t *row_ptr, const int32_t *col_idx,
                     const float *vals, const float *B, int64_t ldb,
                     int64_t r0, int64_t r1, double *C64, double *D64)
{
    (void)k;
#pragma omp parallel for schedule(dynamic, 8)
    for (int64_t i = r0; i < r1; ++i) {
        double *c = C64 + (i - r0) * N;
        double *d = D64 ? D64 + (i - r0) * N : NULL;
        for (int64_t j = 0; j < N; ++j) c[j] = 0.0;
        if (d) for (int64_t j = 0; j < N; ++j) d[j] = 0.0;
        for (int64_t q = row_ptr[i]; q < row_ptr[i + 1]; ++q) {
            double a = (double)vals[q];
            const float *b = B + (int64_t)col_idx[q] * ldb;
            for (int64_t j = 0; j < N; ++j) c[j] += a * (double)b[j];
            if (d) for (int64_t j = 0; j < N; ++j) d[j] += fabs(a) * fabs((double)b[j]);
        }
    }
}

/*
 * The same sum, enumerated from GCOO arrays instead of CSR: for every stored
 * triple (row, col, val), C64(row, :) += val * B(col, :).  Serial.  It ties
 * the GCOO arrays to the product: a conversion that loses, repeats or
 * misplaces an entry changes this result.
 */
void oracle_spdm_gcoo(int64_t m, int64_t N, int64_t nnz,
                      const float *values, const int32_t *rows, const int32_t *cols,
                      const float *B, int64_t ldb, double *C64)
{
    for (int64_t i = 0; i < m * N; ++i) C64[i] = 0.0;
    for (int64_t q = 0; q < nnz; ++q) {
        double a = (double)values[q];
        const float *b = B + (int64_t)cols[q] * ldb;
        double *c = C64 + (int64_t)rows[q] * N;
        for (int64_t j = 0; j < N; ++j) c[j] += a * (double)b[j];
    }
}

/* Equation 1 as printed: C(i,j) = sum_{l=0}^{k-1} A(i,l) * B(l,j), dense, fp64 sums. */
void oracle_dense_gemm(int64_t m, int64_t k, int64_t N, const float *A, int64_t lda,
                       const float *B, int64_t ldb, double *C64)
{
    for (int64_t i = 0; i < m; ++i)
        for (int64_t j = 0; j < N; ++j) {
            double s = 0.0;
            for (int64_t l = 0; l < k; ++l) s += (double)A[i * lda + l] * (double)B[l * ldb + j];
            C64[i * N + j] = s;
        }
}

/*
 * Section 3.3 (reuse of the fetched B value): a "run" is a maximal stretch of
 * consecutive entries of one group that share a column.  Returns the number of
 * runs over all groups; nnz / runs is the mean run length.
 */
int64_t oracle_count_runs(int64_t g, const int32_t *gIdxes, const int32_t *cols)
{
    int64_t runs = 0;
    for (int64_t q = 0; q < g; ++q)
        for (int64_t e = gIdxes[q]; e < gIdxes[q + 1]; ++e)
            if (e == gIdxes[q] || cols[e] != cols[e - 1]) ++runs;
    return runs;
}

/*
 * Worst elementwise deviation of an fp32 result from C64 in units of D64:
 *   max over (i,j) of |C(i,j) - C64(i,j)| / D64(i,j).
 * Where D64 is zero the fp32 value has to be exactly zero; such a violation,
 * and any NaN in C, are counted in *bad.  Returns the maximum over the
 * elements with D64 > 0.
 */
double oracle_max_scaled_error(int64_t rows, int64_t N, const float *C, int64_t ldc,
                               const double *C64, const double *D64, int64_t *bad)
{
    double worst = 0.0;
    int64_t nb = 0;
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t j = 0; j < N; ++j) {
            double c = (double)C[i * ldc + j], r = C64[i * N + j], d = D64[i * N + j];
            if (c != c) { ++nb; continue; }
            if (d == 0.0) { if (c != 0.0) ++nb; continue; }
            double e = fabs(c - r) / d;
            if (e > worst) worst = e;
        }
    if (bad) *bad = nb;
    return worst;
}
