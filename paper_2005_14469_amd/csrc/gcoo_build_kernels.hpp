// Conversion kernels: CSR or dense device matrix -> GCOO arrays (Section 3.1, Algorithm 1).
//
// All kernels are deterministic: the slot of every entry is computed from counts and
// wave-wide ballots, never from the arrival order of atomics, so the arrays come out
// bit-identical from run to run (and equal to the definition: per group, ordered by
// column, then row, then input position).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gcoo {

constexpr int kWave = 64;

// ---------------------------------------------------------------------------------------------
// Algorithm 1, step 1 for a CSR input.  CSR is row-major, so the entries of group q are the
// contiguous CSR range [row_ptr[q*p], row_ptr[min((q+1)*p, m)]): the count and the prefix sum
// are two reads of row_ptr.  One thread per group; thread g also writes the sentinel.
// ---------------------------------------------------------------------------------------------
__global__ void group_index_from_row_ptr(const int32_t* __restrict__ row_ptr, int64_t m, int32_t p, int64_t g,
                                         int32_t* __restrict__ gIdxes, int32_t* __restrict__ nnzPerGroup)
{
    int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q > g) return;
    int64_t r0 = q * p;
    if (r0 > m) r0 = m;
    int32_t b = row_ptr[r0];
    gIdxes[q] = b;
    if (q < g) {
        int64_t r1 = r0 + p;
        if (r1 > m) r1 = m;
        nnzPerGroup[q] = row_ptr[r1] - b;
    }
}

__device__ __forceinline__ uint64_t lanemask_lt()
{
    return (1ull << (threadIdx.x & 63)) - 1ull;   // one wave per workgroup in the kernels below
}

// Lanes of the wave whose 8-bit digit equals this lane's, among the lanes in `active`.
__device__ __forceinline__ uint64_t match_digit(uint32_t d, bool is_active)
{
    uint64_t mask = __ballot(is_active);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
        bool bit = (d >> b) & 1u;
        uint64_t bb = __ballot(is_active && bit);
        mask &= bit ? bb : ~bb;
    }
    return mask;
}

// ---------------------------------------------------------------------------------------------
// Algorithm 1, step 2 for a CSR input: one pass of a stable least-significant-digit radix sort
// of every group's entries on an 8-bit digit of the column index.  One workgroup of kSortWaves
// waves per group.
//
// The CSR order of a group's entries is (row, input position); sorting that stably by column
// gives (column, row, input position).  Each pass is a counting sort.  The group's entries are
// cut into kSortWaves contiguous parts, one per wave.  Every wave counts the digits of its part
// (LDS, a histogram of its own); from those counts each (wave, digit) gets the slot where the
// wave's first entry with that digit goes: digit base + what earlier waves hold of the digit.
// Then every wave walks its part 64 entries at a time, in order, and gives each entry
// slot = that running base + number of earlier entries of the 64 with the same digit (ballots).
// Nothing depends on timing: counts are sums, ranks come from ballots.
//
// FIRST: the source is the CSR input itself (row of an entry = search in row_ptr); otherwise the
// source is the (cols, rows, values) triple written by the previous pass.
// ---------------------------------------------------------------------------------------------
constexpr int kSortWaves = 16;

template <bool FIRST>
__global__ __launch_bounds__(kSortWaves * kWave) void sort_groups_by_col_digit(
    const int32_t* __restrict__ gIdxes, const int32_t* __restrict__ row_ptr, int64_t m, int32_t p,
    const int32_t* __restrict__ src_cols, const int32_t* __restrict__ src_rows, const float* __restrict__ src_vals,
    int32_t* __restrict__ dst_cols, int32_t* __restrict__ dst_rows, float* __restrict__ dst_vals, int shift)
{
    __shared__ int32_t slot_of[kSortWaves][256];      // counts, then running slots, per wave and digit
    __shared__ int32_t total[256];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int64_t q = blockIdx.x;
    const int32_t beg = gIdxes[q], end = gIdxes[q + 1];
    if (beg >= end) return;
    // part of wave wv: whole 64-entry tiles
    const int32_t tiles = (end - beg + kWave - 1) / kWave;
    const int32_t tiles_per = (tiles + kSortWaves - 1) / kSortWaves;
    const int32_t pb = beg + wv * tiles_per * kWave;
    const int32_t pe = (pb + tiles_per * kWave < end) ? pb + tiles_per * kWave : end;

    for (int i = tid; i < kSortWaves * 256; i += kSortWaves * kWave) (&slot_of[0][0])[i] = 0;
    __syncthreads();
    for (int32_t e = pb + lane; e < pe; e += kWave)
        atomicAdd(&slot_of[wv][((uint32_t)src_cols[e] >> shift) & 255u], 1);   // counts only: order-free
    __syncthreads();
    if (tid < 256) {
        int32_t run = 0;
        for (int w = 0; w < kSortWaves; ++w) {
            const int32_t c = slot_of[w][tid];
            slot_of[w][tid] = run;
            run += c;
        }
        total[tid] = run;
    }
    __syncthreads();
    if (wv == 0) {
        // exclusive scan of the 256 digit totals: lane owns digits 4*lane .. 4*lane+3
        const int32_t c0 = total[4 * lane], c1 = total[4 * lane + 1], c2 = total[4 * lane + 2], c3 = total[4 * lane + 3];
        const int32_t sum = c0 + c1 + c2 + c3;
        int32_t incl = sum;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            const int32_t t = __shfl_up(incl, d, kWave);
            if (lane >= d) incl += t;
        }
        const int32_t ex = incl - sum;
        total[4 * lane] = ex;
        total[4 * lane + 1] = ex + c0;
        total[4 * lane + 2] = ex + c0 + c1;
        total[4 * lane + 3] = ex + c0 + c1 + c2;
    }
    __syncthreads();
    for (int i = tid; i < kSortWaves * 256; i += kSortWaves * kWave) (&slot_of[0][0])[i] += total[i & 255];
    __syncthreads();

    // From here on the waves do not meet again: a wave's LDS operations execute in order, and the
    // volatile accesses keep the compiler from reordering the read of a slot and its update.
    volatile int32_t* my_slot = slot_of[wv];
    const int64_t r_lo = q * p;
    const int64_t r_hi = (r_lo + p < m) ? r_lo + p : m;
    const uint64_t lt = lanemask_lt();
    for (int32_t t0 = pb; t0 < pe; t0 += kWave) {
        const int32_t e = t0 + lane;
        const bool act = e < pe;
        int32_t col = 0, row = 0;
        float val = 0.0f;
        if (act) {
            col = src_cols[e];
            val = src_vals[e];
            if (FIRST) {
                // row r with row_ptr[r] <= e < row_ptr[r+1]; empty rows are skipped by the upper bound
                int64_t lo = r_lo, hi = r_hi;          // answer in [lo, hi)
                while (hi - lo > 1) {
                    const int64_t mid = (lo + hi) >> 1;
                    if (row_ptr[mid] <= e) lo = mid; else hi = mid;
                }
                row = (int32_t)lo;
            } else {
                row = src_rows[e];
            }
        }
        const uint32_t d = ((uint32_t)col >> shift) & 255u;
        const uint64_t same = match_digit(d, act);
        const int32_t before = __popcll(same & lt);
        int32_t slot = 0;
        if (act) slot = my_slot[d];
        __builtin_amdgcn_wave_barrier();
        if (act && before == 0) my_slot[d] = slot + __popcll(same);   // first lane of each digit advances it
        __builtin_amdgcn_wave_barrier();
        if (act) {
            const int32_t at = beg + slot + before;
            dst_cols[at] = col;
            dst_rows[at] = row;
            dst_vals[at] = val;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Algorithm 1, step 1 for a dense input: entries != 0 per group.  One workgroup per group;
// threads stride over the band row by row (coalesced), block-reduce, one write.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void count_dense_per_group(const float* __restrict__ A, int64_t lda, int64_t m, int64_t k,
                                                              int32_t p, int32_t* __restrict__ nnzPerGroup)
{
    __shared__ int32_t part[4];
    const int64_t q = blockIdx.x;
    const int64_t r0 = q * p, r1 = (r0 + p < m) ? r0 + p : m;
    int32_t n = 0;
    for (int64_t r = r0; r < r1; ++r) {
        const float* a = A + r * lda;
        for (int64_t j = threadIdx.x; j < k; j += 256) n += (a[j] != 0.0f) ? 1 : 0;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) n += __shfl_down(n, d, kWave);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = n;
    __syncthreads();
    if (threadIdx.x == 0) nnzPerGroup[q] = part[0] + part[1] + part[2] + part[3];
}

// Exclusive prefix sum of nnzPerGroup[g] into gIdxes[g+1] (sentinel = total).  One workgroup;
// g is small (m / p), so a serial carry over 256-wide tiles is enough.
__global__ __launch_bounds__(256) void scan_group_counts(const int32_t* __restrict__ nnzPerGroup, int64_t g,
                                                          int32_t* __restrict__ gIdxes, unsigned long long* __restrict__ total)
{
    __shared__ int64_t wsum[4];
    __shared__ int64_t carry_s;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    for (int64_t t0 = 0; t0 < g; t0 += 256) {
        const int64_t i = t0 + threadIdx.x;
        const int64_t v = (i < g) ? nnzPerGroup[i] : 0;
        int64_t incl = v;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            int64_t t = __shfl_up(incl, d, kWave);
            if (lane >= d) incl += t;
        }
        if (lane == 63) wsum[w] = incl;
        __syncthreads();
        int64_t off = carry_s;
        for (int j = 0; j < w; ++j) off += wsum[j];
        if (i < g) gIdxes[i] = (int32_t)(off + incl - v);
        __syncthreads();
        if (threadIdx.x == 255) carry_s = off + incl;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        // totals above INT32_MAX are reported through *total and rejected by the host
        gIdxes[g] = (int32_t)(carry_s > 0x7fffffffLL ? 0x7fffffffLL : carry_s);
        *total = (unsigned long long)carry_s;
    }
}

// ---------------------------------------------------------------------------------------------
// Algorithm 1, step 2 for a dense input.  One wave per group.  The band (pb rows x k columns)
// is walked in column-major order, 64 elements at a time: element index t -> column t / pb,
// band row t % pb.  A ballot of "!= 0" gives each nonzero its rank among the 64, a running
// count carries over, and the entry is written straight to its final slot: the output is in
// (column, row) order with no sort.  Reads of one 64-chunk touch pb rows x (64/pb) columns;
// consecutive chunks reuse the same cache lines.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kWave) void fill_from_dense(const float* __restrict__ A, int64_t lda, int64_t m, int64_t k,
                                                         int32_t p, const int32_t* __restrict__ gIdxes,
                                                         float* __restrict__ values, int32_t* __restrict__ rows,
                                                         int32_t* __restrict__ cols)
{
    const int lane = threadIdx.x;
    const int64_t q = blockIdx.x;
    const int64_t r0 = q * p;
    const int64_t pb = (r0 + p < m) ? p : (m - r0);       // rows in this band
    const int64_t total = pb * k;
    int64_t at = gIdxes[q];
    const uint64_t lt = lanemask_lt();
    for (int64_t t0 = 0; t0 < total; t0 += kWave) {
        const int64_t t = t0 + lane;
        float a = 0.0f;
        int64_t c = 0, r = 0;
        if (t < total) {
            c = t / pb;
            r = r0 + (t - c * pb);
            a = A[r * lda + c];
        }
        const bool nz = (t < total) && (a != 0.0f);
        const uint64_t bal = __ballot(nz);
        if (nz) {
            const int64_t slot = at + __popcll(bal & lt);
            values[slot] = a;
            rows[slot] = (int32_t)r;
            cols[slot] = (int32_t)c;
        }
        at += __popcll(bal);
    }
}

// Total count of entries != 0 of a dense matrix (Algorithm 1, step 1, without the grouping).
__global__ __launch_bounds__(256) void count_dense_total(const float* __restrict__ A, int64_t lda, int64_t m, int64_t k,
                                                          unsigned long long* __restrict__ total)
{
    unsigned long long n = 0;
    for (int64_t r = blockIdx.x; r < m; r += gridDim.x) {
        const float* a = A + r * lda;
        for (int64_t j = threadIdx.x; j < k; j += 256) n += (a[j] != 0.0f) ? 1u : 0u;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) n += __shfl_down(n, d, kWave);
    if ((threadIdx.x & 63) == 0 && n) atomicAdd(total, n);   // integer sum: order-free
}

}  // namespace gcoo
