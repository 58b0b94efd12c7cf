// The run schedule: a kernel-private re-listing of a GCOO matrix that makes the reuse loop of
// Algorithm 2 ("while the next entry has the same col, reuse the fetched B value") free of
// run-time branches, and that the SpDM kernel can stream through LDS (the staging of a group's
// entries in shared memory of Algorithm 2).
//
// Runs and classes.  Inside a group, a run is a maximal stretch of entries with one column (they
// share one fetched segment of B).  Runs longer than kMaxRun are cut into pieces of kMaxRun.  The
// columns are cut into `nw` windows of `window_cols` columns; the pieces of one (group, window)
// are re-listed by length class L = 1..kMaxRun, in column order inside a class.  The windows keep
// the waves that work on one column tile of B inside a band of B that fits the L2 of their XCD,
// whatever class they are in.
//
// Chunks and bodies.  J = runs_per_chunk(L) pieces make a chunk; kBody = 4 chunks make a body,
// the unit of the kernel's loop (one turn multiplies four chunks while the B loads of the next
// three chunks are in flight).  A class segment is
//     pre-block | block 0 | block 1 | ... | block nb-1
// Block b (block_dwords(L) 32-bit words) holds what turn b needs:
//     col[4*J]         columns of chunks 4b+3 .. 4b+6 (the loads that turn b starts)
//     rowpack[4][RP]   rows inside the group, one byte each, of chunks 4b .. 4b+3 (RP = ceil(J*L/4) words per chunk)
//     val[4][VS]       value bits of chunks 4b .. 4b+3 (VS = J*L rounded up to a multiple of 4 words)
// and the pre-block (4*J words) holds {unused, columns of chunks 0, 1, 2}.  Piece j of a chunk
// owns entries j*L .. j*L+L-1 of the chunk.  Column slots of chunks that do not exist hold a
// valid column (the load happens and is ignored).
//
// Dummy pieces fill a class up to whole bodies: a valid column and entries whose row is p, one
// past the rows of the group; the SpDM kernel keeps a partial sum for that row too and never
// stores it, so a dummy entry has no effect on C whatever B holds.
//
// A class with little work in a (group, window) is not worth a loop of its own (starting and
// draining the load pipeline costs a few memory latencies): when the pieces of class L > 1 hold
// fewer than kMinClassEntries entries, they are listed as L pieces of class 1 instead (the same
// column fetched L times in a row, which the vector cache absorbs).
//
// Space.  Group q owns the words [3*gIdxes[q] + kSchedPad*nw*q, ...) of the stream.  A real entry
// costs at most block_dwords(1)/16 = 2.25 words.  Dummy pieces and the pre-block add at most one
// block plus one pre-block per class: 52 words for class 1; a class L > 1 exists only with
// kMinClassEntries entries or more and adds at most 92 words, under 0.4 words per entry.  So
// 3 words per entry plus kSchedPad words per (group, window) bound a group, and no prefix sum over
// groups is needed.  The kernel reads whole 512-byte lines, so the stream ends with that much slack.
// hdr[(q*nw + w)*kMaxRun + L-1] = {first word of the class segment relative to the group's base, nb}.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gcoo {

constexpr int kMaxRun = 8;
constexpr int kBody = 4;                 // chunks per loop turn of the SpDM kernel
constexpr int kMinClassEntries = 256;
constexpr int kSchedPad = 64;            // words per (group, window) for class 1's dummy pieces and pre-block
constexpr int kSchedSlack = 128;         // words after the last group (whole-line reads)
constexpr int kMaxWindows = 32;
// Tallest group the register kernel serves.  The layout itself (rows as bytes, row p included)
// and the one-column-per-lane instance reach p = 128, but that instance is not part of the build: see
// sched_width() in gcoo_api.hip.
constexpr int kSchedMaxP = 64;

__host__ __device__ constexpr int runs_per_chunk(int L) { return L <= 3 ? 4 : (L <= 6 ? 2 : 1); }
__host__ __device__ constexpr int rowpack_dwords(int L) { return (runs_per_chunk(L) * L + 3) / 4; }
__host__ __device__ constexpr int pre_dwords(int L) { return kBody * runs_per_chunk(L); }
// words of one chunk's values inside a block: J*L rounded up to whole 16-byte LDS reads
__host__ __device__ constexpr int val_stride(int L) { return (runs_per_chunk(L) * L + 3) / 4 * 4; }
__host__ __device__ constexpr int block_dwords(int L)
{
    return kBody * runs_per_chunk(L) + kBody * rowpack_dwords(L) + kBody * val_stride(L);
}
// word offsets inside a block
__host__ __device__ constexpr int blk_rowpack(int L, int c) { return kBody * runs_per_chunk(L) + c * rowpack_dwords(L); }
__host__ __device__ constexpr int blk_val(int L, int c)
{
    return kBody * runs_per_chunk(L) + kBody * rowpack_dwords(L) + c * val_stride(L);
}

__host__ __device__ inline int64_t sched_group_base(int64_t first_entry, int64_t q, int32_t nw)
{
    return 3 * first_entry + (int64_t)kSchedPad * nw * q;
}
__host__ __device__ inline int64_t sched_words(int64_t nnz, int64_t g, int32_t nw)
{
    return 3 * nnz + (int64_t)kSchedPad * nw * g + kSchedSlack;
}

struct SchedClass {
    int32_t first_word;   // of the pre-block, relative to the group's base
    int32_t bodies;       // nb
};

// When a launch has too few (group, tile) items to fill the machine, the longest group sets the run
// time: groups well above the mean load of a wave slot are then shared by the eight waves of a
// workgroup (spdm_sched_coop).  Sharing costs every wave a start-up per class and window, so it is
// only used when the largest group stands out (four times the mean group, a skewed matrix) or when
// plain waves would leave seven eighths of the machine idle.  Returns the entry count from which a
// group is treated that way, INT32_MAX for "none".  Evaluated on the device from the statistics the
// conversion left there (largest = entries of the largest group), so that a launch needs nothing
// from the host but the shape; the host evaluates only the part that does not need `largest`.
constexpr int64_t kHeavyWaveSlots = 2048;                  // 256 compute units x 8 resident waves of the register kernel
constexpr int64_t kHeavyMin = 1024;
constexpr int64_t kOrderMaxGroups = 2 * kHeavyWaveSlots;   // a launch of few items has at most that many groups
__host__ __device__ inline bool sched_heavy_possible(int64_t nnz, int64_t g, int64_t tiles)
{
    const int64_t items = g * tiles;
    return items > 0 && items <= 2 * kHeavyWaveSlots && nnz > 0;
}
__host__ __device__ inline int32_t sched_heavy_min(int64_t nnz, int64_t g, int64_t tiles, int64_t largest)
{
    if (!sched_heavy_possible(nnz, g, tiles)) return 0x7fffffff;
    const int64_t items = g * tiles;
    const int64_t mean_group = nnz / g;
    const bool skewed = largest >= 4 * mean_group;
    const bool empty = items * 8 <= kHeavyWaveSlots;       // plain waves would fill an eighth of the machine at most
    if (!skewed && !empty) return 0x7fffffff;
    // Split what carries more than one and a half times the mean load of a wave of this launch (a wave per item
    // while the items do not outnumber the wave slots, a slot's share of all entries beyond that): a workgroup of
    // eight waves for a group costs its compute unit the seven other groups that would run beside it, so a lower
    // bar loses more than it gains, and a higher one leaves single waves with the long groups.  On the power-law
    // workload (16384 rows, 512 columns of B) at 32 rows per group (1024 items) the bar is 2544 entries: 0.161 ms
    // against 0.185 at 1272 and 0.186 at 3392; at 16 rows per group (2048 items) it is 1272: 0.20 ms against 0.26 at 2544.
    const int64_t mean_per_slot = nnz * tiles / kHeavyWaveSlots;
    const int64_t mean_wave = mean_group > mean_per_slot ? mean_group : mean_per_slot;
    int64_t t = mean_wave + mean_wave / 2;
    if (t < kHeavyMin) t = kHeavyMin;
    return t >= 0x7fffffff ? 0x7fffffff : (int32_t)t;
}

}  // namespace gcoo
