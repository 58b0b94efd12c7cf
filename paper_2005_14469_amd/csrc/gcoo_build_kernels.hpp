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

// What the host wants to know about a CSR input before it sizes anything: out[0] = nnz = row_ptr[m],
// out[1] = entries of the largest group.  The work of one workgroup of 256 threads.
__device__ __forceinline__ void group_stats_block(const int32_t* __restrict__ row_ptr, int64_t m, int32_t p, int64_t g,
                                                  unsigned long long* __restrict__ out)
{
    __shared__ int32_t part[4];
    int32_t mx = 0;
    for (int64_t q = threadIdx.x; q < g; q += 256) {
        const int64_t r0 = q * p, r1 = (r0 + p < m) ? r0 + p : m;
        const int32_t n = row_ptr[r1] - row_ptr[r0];
        mx = n > mx ? n : mx;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const int32_t o = __shfl_down(mx, d, kWave);
        mx = o > mx ? o : mx;
    }
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 1; i < 4; ++i) mx = part[i] > mx ? part[i] : mx;
        const int32_t last = row_ptr[m];
        out[0] = last < 0 ? ~0ull : (unsigned long long)last;
        out[1] = (unsigned long long)mx;
    }
}

__global__ __launch_bounds__(256) void group_stats_from_row_ptr(const int32_t* __restrict__ row_ptr, int64_t m, int32_t p, int64_t g,
                                                                 unsigned long long* __restrict__ out)
{
    group_stats_block(row_ptr, m, p, g, out);
}

// ---------------------------------------------------------------------------------------------
// Algorithm 1, step 1 for a CSR input.  CSR is row-major, so the entries of group q are the
// contiguous CSR range [row_ptr[q*p], row_ptr[min((q+1)*p, m)]): the count and the prefix sum
// are two reads of row_ptr.  One thread per group; thread g also writes the sentinel.
// 256 threads per workgroup, ceil((g+1)/256) workgroups; with `stats` given, one workgroup more,
// which computes the statistics above in the same launch.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void group_index_from_row_ptr(const int32_t* __restrict__ row_ptr, int64_t m, int32_t p, int64_t g,
                                                                 int32_t nnz, int32_t* __restrict__ gIdxes,
                                                                 int32_t* __restrict__ nnzPerGroup, unsigned long long* __restrict__ stats,
                                                                 uint32_t* __restrict__ bad_col)
{
    if (stats && blockIdx.x == gridDim.x - 1) {                   // the whole workgroup
        if (threadIdx.x == 0) *bad_col = 0u;                      // set by the sort that follows if it meets a column out of range
        group_stats_block(row_ptr, m, p, g, stats);
        return;
    }
    int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q > g) return;
    // Offsets are clamped to [0, nnz]: with a device input whose row_ptr does not match the nnz
    // the buffer was laid out for, every later kernel still stays inside the arrays.
    auto at = [&](int64_t r) { const int32_t v = row_ptr[r]; return v < 0 ? 0 : (v > nnz ? nnz : v); };
    int64_t r0 = q * p;
    if (r0 > m) r0 = m;
    const int32_t b = at(r0);
    gIdxes[q] = b;
    if (q < g) {
        int64_t r1 = r0 + p;
        if (r1 > m) r1 = m;
        const int32_t n = at(r1) - b;
        nnzPerGroup[q] = n < 0 ? 0 : n;
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
// FIRST: the source is the CSR input itself (row of an entry = search in row_ptr; columns are forced
// into [0, kcols) and *bad_col is set if one was outside); otherwise the source is the (cols, rows,
// values) triple written by the previous pass.
//
// nb > 0: the workgroup sorts one bucket of one group instead of a whole group.  The pass before
// it has sorted the group by the digit above (col >> 8, nb values); bucket b of group q is the
// stretch of the group with that digit equal to b, found by two binary searches, and it is sorted
// in place (inside its own stretch of the destination) by the low digit.  High digit first keeps
// the stores of both passes close together: consecutive entries of a CSR row fall into the same
// bucket in the first pass, and a bucket's stretch is a few kilobytes in the second, where the
// low digit first scatters every store of both passes over the whole group.
// ---------------------------------------------------------------------------------------------
constexpr int kSortWaves = 16;          // waves of the workgroup that sorts a whole group
constexpr int kSortBucketWaves = 4;     // and of the one that sorts one bucket of a group (about a thousand entries)

template <bool FIRST, int WAVES>
__global__ __launch_bounds__(WAVES * kWave) void sort_groups_by_col_digit(
    const int32_t* __restrict__ gIdxes, const int32_t* __restrict__ row_ptr, int64_t m, int32_t p,
    const int32_t* __restrict__ src_cols, const int32_t* __restrict__ src_rows, const float* __restrict__ src_vals,
    int32_t* __restrict__ dst_cols, int32_t* __restrict__ dst_rows, float* __restrict__ dst_vals, int shift, int32_t nb,
    int32_t kcols, uint32_t* __restrict__ bad_col)
{
    // FIRST: a column of the input outside [0, kcols) is stored clamped into that range and reported in
    // *bad_col, so that no later kernel forms an address outside B from it
    auto in_range = [&](int32_t c) { return FIRST ? (c < 0 ? 0 : (c >= kcols ? kcols - 1 : c)) : c; };
    __shared__ int32_t slot_of[WAVES][256];      // counts, then running slots, per wave and digit
    __shared__ int32_t total[256];
    __shared__ int32_t rp_s[FIRST ? 257 : 1];         // FIRST: row_ptr of the group's rows (at most 256 + 1), searched per entry
    __shared__ int32_t range_s[2];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int64_t q = nb > 0 ? blockIdx.x / nb : blockIdx.x;
    int32_t beg = gIdxes[q], end = gIdxes[q + 1];
    if (beg >= end) return;
    if (nb > 0) {
        // threads 0 and 1: first entry of the group whose high digit is >= b, and >= b + 1
        if (tid < 2) {
            const int32_t want = (int32_t)(blockIdx.x - q * nb) + tid;
            int32_t lo = beg, hi = end;
            while (lo < hi) {
                const int32_t mid = lo + (hi - lo) / 2;
                if ((src_cols[mid] >> 8) < want) lo = mid + 1; else hi = mid;
            }
            range_s[tid] = lo;
        }
        __syncthreads();
        beg = range_s[0];
        end = range_s[1];
        if (beg >= end) return;                      // the whole workgroup
    }
    if (FIRST) {
        const int64_t r_lo = q * p;
        const int64_t r_hi = (r_lo + p < m) ? r_lo + p : m;
        static_assert(!FIRST || WAVES * kWave >= 257, "one thread per row of the group, and one more");
        if (tid <= r_hi - r_lo) rp_s[tid] = row_ptr[r_lo + tid];     // the barriers below publish it
    }
    // part of wave wv: whole 64-entry tiles
    const int32_t tiles = (end - beg + kWave - 1) / kWave;
    const int32_t tiles_per = (tiles + WAVES - 1) / WAVES;
    const int32_t pb = beg + wv * tiles_per * kWave;
    const int32_t pe = (pb + tiles_per * kWave < end) ? pb + tiles_per * kWave : end;

    for (int i = tid; i < WAVES * 256; i += WAVES * kWave) (&slot_of[0][0])[i] = 0;
    __syncthreads();
    // (four loads in flight per lane: a wave's part is some thirty tiles, and one load at a time made the pass a chain
    // of memory latencies)
    for (int32_t e = pb + lane; e < pe; e += 4 * kWave) {
        int32_t c[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) c[u] = e + u * kWave < pe ? src_cols[e + u * kWave] : 0;
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (e + u * kWave < pe) atomicAdd(&slot_of[wv][((uint32_t)in_range(c[u]) >> shift) & 255u], 1);   // counts only: order-free
    }
    __syncthreads();
    if (tid < 256) {
        int32_t run = 0;
        for (int w = 0; w < WAVES; ++w) {
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
    for (int i = tid; i < WAVES * 256; i += WAVES * kWave) (&slot_of[0][0])[i] += total[i & 255];
    __syncthreads();

    // From here on the waves do not meet again: a wave's LDS operations execute in order, and the
    // volatile accesses keep the compiler from reordering the read of a slot and its update.
    volatile int32_t* my_slot = slot_of[wv];
    const int64_t r_lo = q * p;
    const int64_t r_hi = (r_lo + p < m) ? r_lo + p : m;
    const uint64_t lt = lanemask_lt();
    // the loads of the next tile are issued before this tile is ranked and stored
    int32_t col_next = 0, row_next = 0;
    float val_next = 0.0f;
    auto request = [&](int32_t t) {
        const int32_t e = t + lane;
        if (e < pe) {
            col_next = src_cols[e];
            val_next = src_vals[e];
            if (!FIRST) row_next = src_rows[e];
        }
    };
    request(pb);
    for (int32_t t0 = pb; t0 < pe; t0 += kWave) {
        const int32_t e = t0 + lane;
        const bool act = e < pe;
        int32_t col = col_next, row = row_next;
        float val = val_next;
        if (t0 + kWave < pe) request(t0 + kWave);
        if (act) {
            if (FIRST) {
                const int32_t c = in_range(col);
                if (c != col) { *bad_col = 1u; col = c; }
                // row r with row_ptr[r] <= e < row_ptr[r+1]; empty rows are skipped by the upper bound
                int32_t lo = 0, hi = (int32_t)(r_hi - r_lo);      // answer in [lo, hi), relative to the group's first row
                while (hi - lo > 1) {
                    const int32_t mid = (lo + hi) >> 1;
                    if (rp_s[mid] <= e) lo = mid; else hi = mid;
                }
                row = (int32_t)r_lo + lo;
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
// Algorithm 1 for a dense input.  The band of group q (pb rows x k columns) is cut into blocks of
// kDenseThreads*VW columns; workgroup (block, q) gives every thread VW adjacent columns, and the
// threads of a wave read 64*VW adjacent floats of a row at a time (coalesced), row after row.
//
// Step 1 (count_dense_blocks): entries != 0 per block.  scan_dense_blocks then turns the counts
// of a group into offsets (exclusive prefix sum over its blocks) and their sum into
// nnzPerGroup[q]; scan_group_counts makes gIdxes from that.
// ---------------------------------------------------------------------------------------------
constexpr int kDenseThreads = 256;

// VW adjacent floats of a row: one 16-byte load when VW = 4 (the launcher checks alignment).
template <int VW>
struct DenseVec { float x[VW]; };

template <int VW>
__device__ __forceinline__ DenseVec<VW> load_dense(const float* a)
{
    DenseVec<VW> v;
    if constexpr (VW == 4) {
        const float4 t = *reinterpret_cast<const float4*>(a);
        v.x[0] = t.x; v.x[1] = t.y; v.x[2] = t.z; v.x[3] = t.w;
    } else {
        v.x[0] = *a;
    }
    return v;
}

__device__ __forceinline__ int32_t block_sum_256(int32_t n, int32_t* part)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) n += __shfl_down(n, d, kWave);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = n;
    __syncthreads();
    return part[0] + part[1] + part[2] + part[3];
}

// Thread t of block b owns columns (b*kDenseThreads + t)*VW .. +VW-1 of the band (k % VW == 0 when VW > 1).
template <int VW>
__global__ __launch_bounds__(kDenseThreads) void count_dense_blocks(const float* __restrict__ A, int64_t lda, int64_t m, int64_t k,
                                                                     int32_t p, int64_t nblk, int32_t* __restrict__ blk_cnt)
{
    __shared__ int32_t part[4];
    const int64_t q = blockIdx.x / nblk, b = blockIdx.x - q * nblk;      // blockIdx.x = q*nblk + b
    const int64_t c = (b * kDenseThreads + threadIdx.x) * VW;
    const int64_t r0 = q * p, r1 = (r0 + p < m) ? r0 + p : m;
    int32_t n = 0;
    if (c < k) {
        const float* a = A + r0 * lda + c;
        for (int64_t r = r0; r < r1; ++r, a += lda) {
            const DenseVec<VW> v = load_dense<VW>(a);
#pragma unroll
            for (int u = 0; u < VW; ++u) n += (v.x[u] != 0.0f) ? 1 : 0;
        }
    }
    const int32_t tot = block_sum_256(n, part);
    if (threadIdx.x == 0) blk_cnt[blockIdx.x] = tot;
}

// One workgroup per group: blk[q][0..nblk) counts -> exclusive offsets in place, sum -> nnzPerGroup[q].
__global__ __launch_bounds__(256) void scan_dense_blocks(int32_t* __restrict__ blk, int64_t nblk, int32_t* __restrict__ nnzPerGroup)
{
    __shared__ int32_t wsum[4];
    __shared__ int32_t carry_s;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int32_t* b = blk + (int64_t)blockIdx.x * nblk;
    for (int64_t t0 = 0; t0 < nblk; t0 += 256) {
        const int64_t i = t0 + threadIdx.x;
        const int32_t v = (i < nblk) ? b[i] : 0;
        int32_t incl = v;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            const int32_t t = __shfl_up(incl, d, kWave);
            if (lane >= d) incl += t;
        }
        if (lane == 63) wsum[w] = incl;
        __syncthreads();
        int32_t off = carry_s;
        for (int j = 0; j < w; ++j) off += wsum[j];
        if (i < nblk) b[i] = off + incl - v;
        __syncthreads();
        if (threadIdx.x == 255) carry_s = off + incl;
        __syncthreads();
    }
    if (threadIdx.x == 0) nnzPerGroup[blockIdx.x] = carry_s;
}

// Exclusive prefix sum of nnzPerGroup[g] into gIdxes[g+1] (sentinel = total).  One workgroup;
// g is small (m / p), so a serial carry over 256-wide tiles is enough.  total[0] = nnz,
// total[1] = entries of the largest group.
__global__ __launch_bounds__(256) void scan_group_counts(const int32_t* __restrict__ nnzPerGroup, int64_t g,
                                                          int32_t* __restrict__ gIdxes, unsigned long long* __restrict__ total)
{
    __shared__ int64_t wsum[4];
    __shared__ int64_t carry_s;
    __shared__ int32_t wmax[4];
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int32_t mx = 0;
    for (int64_t t0 = 0; t0 < g; t0 += 256) {
        const int64_t i = t0 + threadIdx.x;
        const int64_t v = (i < g) ? nnzPerGroup[i] : 0;
        mx = (int32_t)v > mx ? (int32_t)v : mx;
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
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const int32_t o = __shfl_down(mx, d, kWave);
        mx = o > mx ? o : mx;
    }
    if (lane == 0) wmax[w] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
        // totals above INT32_MAX are reported through total[0] and rejected by the host
        gIdxes[g] = (int32_t)(carry_s > 0x7fffffffLL ? 0x7fffffffLL : carry_s);
        total[0] = (unsigned long long)carry_s;
        for (int i = 1; i < 4; ++i) mx = wmax[i] > mx ? wmax[i] : mx;
        total[1] = (unsigned long long)mx;
    }
}

// ---------------------------------------------------------------------------------------------
// Algorithm 1, step 2 for a dense input (fill_dense_blocks), same blocks as step 1.  Inside a
// group the entries are ordered by (column, row), so the entries of block b come right after
// those of blocks 0..b-1, column by column, and inside a column by row.  Thread c counts the
// entries of its column, a workgroup-wide exclusive prefix sum of those counts gives the first
// slot of every column, and the thread walks its column a second time (now from cache) and
// writes each entry to its final slot.  No sort, no atomics: the slot of an entry is a
// function of the matrix alone.
// ---------------------------------------------------------------------------------------------
template <int VW>
__global__ __launch_bounds__(kDenseThreads) void fill_dense_blocks(const float* __restrict__ A, int64_t lda, int64_t m, int64_t k,
                                                                    int32_t p, int64_t nblk, const int32_t* __restrict__ gIdxes,
                                                                    const int32_t* __restrict__ blk_off, float* __restrict__ values,
                                                                    int32_t* __restrict__ rows, int32_t* __restrict__ cols)
{
    __shared__ int32_t wsum[4];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t q = blockIdx.x / nblk, b = blockIdx.x - q * nblk;      // blockIdx.x = q*nblk + b
    const int64_t c = (b * kDenseThreads + threadIdx.x) * VW;
    const int64_t r0 = q * p, r1 = (r0 + p < m) ? r0 + p : m;
    const float* col0 = A + r0 * lda + c;
    int32_t n[VW];
#pragma unroll
    for (int u = 0; u < VW; ++u) n[u] = 0;
    if (c < k) {
        const float* a = col0;
        for (int64_t r = r0; r < r1; ++r, a += lda) {
            const DenseVec<VW> v = load_dense<VW>(a);
#pragma unroll
            for (int u = 0; u < VW; ++u) n[u] += (v.x[u] != 0.0f) ? 1 : 0;
        }
    }
    int32_t mine = 0;
#pragma unroll
    for (int u = 0; u < VW; ++u) mine += n[u];
    int32_t incl = mine;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const int32_t t = __shfl_up(incl, d, kWave);
        if (lane >= d) incl += t;
    }
    if (lane == 63) wsum[w] = incl;
    __syncthreads();
    int32_t first = gIdxes[q] + blk_off[blockIdx.x] + incl - mine;       // slot of the first entry of this thread's columns
    for (int j = 0; j < w; ++j) first += wsum[j];
    if (c < k && mine > 0) {
        int32_t at[VW];
#pragma unroll
        for (int u = 0; u < VW; ++u) { at[u] = first; first += n[u]; }
        const float* a = col0;
        for (int64_t r = r0; r < r1; ++r, a += lda) {
            const DenseVec<VW> v = load_dense<VW>(a);
#pragma unroll
            for (int u = 0; u < VW; ++u) {
                if (v.x[u] != 0.0f) {
                    values[at[u]] = v.x[u];
                    rows[at[u]] = (int32_t)r;
                    cols[at[u]] = (int32_t)(c + u);
                    ++at[u];
                }
            }
        }
    }
}

// Total count of entries != 0 of a dense matrix (Algorithm 1, step 1, without the grouping).
template <int VW>
__global__ __launch_bounds__(256) void count_dense_total(const float* __restrict__ A, int64_t lda, int64_t m, int64_t k,
                                                          unsigned long long* __restrict__ total)
{
    unsigned long long n = 0;
    for (int64_t r = blockIdx.x; r < m; r += gridDim.x) {
        const float* a = A + r * lda;
        for (int64_t j = (int64_t)threadIdx.x * VW; j < k; j += 256 * VW) {
            const DenseVec<VW> v = load_dense<VW>(a + j);
#pragma unroll
            for (int u = 0; u < VW; ++u) n += (v.x[u] != 0.0f) ? 1u : 0u;
        }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) n += __shfl_down(n, d, kWave);
    if ((threadIdx.x & 63) == 0 && n) atomicAdd(total, n);   // integer sum: order-free
}

}  // namespace gcoo
