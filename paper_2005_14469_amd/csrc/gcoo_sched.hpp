// The run schedule: a kernel-private re-listing of a GCOO matrix that makes the reuse loop of
// Algorithm 2 ("while the next entry has the same col, reuse the fetched B value") free of
// run-time branches.
//
// Inside a group, a run is a maximal stretch of entries with one column (they share one fetched
// segment of B).  Runs longer than kMaxRun are cut into pieces of kMaxRun.  The columns are cut
// into `nw` windows of `window_cols` columns; the pieces of one (group, window) are re-listed by
// length class L = 1..kMaxRun, in column order inside a class, packed into chunks of
// runs_per_chunk(L) pieces.  A chunk is chunk_dwords(L) 32-bit words:
//     col[J] | row[J*L] | value bits[J*L]        (J = runs_per_chunk(L); piece j owns entries j*L .. j*L+L-1)
// where row is the row inside the group.  The windows keep the waves that work on one column
// tile of B inside a band of B that fits the L2 of their XCD, whatever class they are in.
//
// A class is filled up with dummy pieces to a whole, even number of chunks (the kernel's loop
// takes them two at a time): a valid column and entries whose row is p, one past the rows of the
// group; the SpDM kernel keeps a partial sum for that row too and never stores it, so a dummy
// entry has no effect on C whatever B holds.
//
// A class with little work in a (group, window) is not worth a loop of its own (starting and
// draining the load pipeline costs a few memory latencies): when the pieces of class L > 1 hold
// fewer than kMinClassEntries entries, they are listed as L pieces of class 1 instead (the same
// column fetched L times in a row, which the vector cache absorbs).
//
// Group q owns the words [4*gIdxes[q] + kSchedPad*nw*q, ...) of the stream.  Real pieces take at
// most 3 words per entry (column of the piece, row, value).  Dummy pieces: class 1 adds at most
// 45 words per window; a class L > 1 exists only with kMinClassEntries entries or more and adds at
// most 49 words, less than one word per five entries.  So 4 words per entry plus kSchedPad words
// per window bound a group, and no prefix sum over groups is needed.
// hdr[(q*nw + w)*kMaxRun + L-1] = {first word of the class relative to the group's base, number of chunks}.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gcoo {

constexpr int kMaxRun = 8;

__host__ __device__ constexpr int runs_per_chunk(int L) { return L == 1 ? 8 : (L <= 3 ? 4 : (L <= 6 ? 2 : 1)); }
__host__ __device__ constexpr int chunk_dwords(int L) { return runs_per_chunk(L) * (1 + 2 * L); }

constexpr int kMinClassEntries = 256;

constexpr int kSchedPad = 48;            // words per (group, window) for the dummy pieces of class 1
constexpr int kMaxWindows = 32;

__host__ __device__ inline int64_t sched_group_base(int64_t first_entry, int64_t q, int32_t nw)
{
    return 4 * first_entry + (int64_t)kSchedPad * nw * q;
}
__host__ __device__ inline int64_t sched_words(int64_t nnz, int64_t g, int32_t nw)
{
    return 4 * nnz + (int64_t)kSchedPad * nw * g;
}

struct SchedClass {
    int32_t first_word;   // relative to the group's base
    int32_t chunks;
};

}  // namespace gcoo
