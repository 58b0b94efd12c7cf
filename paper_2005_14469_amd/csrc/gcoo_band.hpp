// The band schedule: a second kernel-private re-listing of a GCOO matrix, for the SpDM kernel in
// which the W waves of a workgroup share the rows of B through LDS (gcoo_spdm_band_kernel.hpp).
//
// Why.  With one wave per group, every run of entries costs its wave a 1 KB segment of a B row
// through the vector cache, and that traffic (runs x 1 KB) is what bounds the register kernel once
// a matrix is sparse enough that few entries share a column inside a group (Section 3.3 counts
// exactly these fetches).  W consecutive groups (a super-group, W*p rows of A) ask for the same
// B rows far more often than one group does, so the workgroup fetches each needed row once into
// LDS and its waves read it from there.
//
// Two shapes.  W = 8 for groups of 17..32 rows (a wave keeps 33 x 4 partial sums per lane, two waves
// per SIMD); W = 16 for groups of at most 16 rows (17 x 4 partial sums, four waves per SIMD).  Both
// cover up to 256 rows of A per workgroup.  Below, R = 64 / W is the number of B rows a wave
// fetches per band, and a block is at most band_block_max(W) words.
//
// Bands.  ucols(Q) = the distinct columns that hold an entry of super-group Q, ascending.  Band b
// of Q = ucols[64b .. 64b+63]: the kBandRows rows of B that are in LDS together; a column's slot is
// its place in the band.  Rows of B that no entry of Q touches are never fetched.
//
// Streams.  Every (Q, wave w) has one stream of 32-bit words, also when group W*Q+w does not exist
// (the wave still fetches its share of every band):
//     pre-block | blocks of band 0 | blocks of band 1 | ...
// A band has one block per segment of the group's entries in it (a segment = the runs that start
// within band_seg(W) = 68 or 24 entries of its first entry, so at most 99 or 55 entries; a band
// without entries has one empty block).  A block is at most band_block_max(W) = 256 or 128 words:
// 12 header words, then chunks:
//     w0       n1 | n2 << 8 | n4 << 16 | n8 << 24      chunks of each type in this block
//     w1       bit 0: last block of its band; bits 1..2: piece slots in use in the last chunk of
//              type 1 (0 = all four, or no such chunk); bits 8..15: rows of the next band    (*)
//     w2       words from the start of this block to the first block of the next band  (*)
//     w3       words of this block
//     w4..w11  the B rows this wave fetches for the next band: slots t*W + w, t = 0..R-1 (0 if none
//              and for t >= R)  (*)
//     (*) in the first block of a band and in the pre-block (whose "next band" is band 0)
// Runs are cut into pieces of 8, 4, 2 and 1 entries (a run of 7 = 4 + 2 + 1); a chunk holds
//     type 1: 4 pieces of 1 entry   8 words:  2 offset words, 1 row word, 1 unused, 4 values
//     type 2: 4 pieces of 2        12 words:  2 offset words, 2 row words, 8 values
//     type 4: 2 pieces of 4        12 words:  1 offset word, 2 row words, 1 unused, 8 values
//     type 8: 1 piece  of 8        12 words:  1 offset word, 2 row words, 1 unused, 8 values
// Pieces of 4 and of 2 that would leave a chunk partly filled are halved and join the end of
// the list of the next smaller type, so that only the last chunk of type 1 can hold unused piece
// slots (at most three entries that multiply by zero).
// offset = slot * 1024 as 16-bit halves (the byte offset of the B row inside the LDS band),
// rows = row inside the group, one byte each, values = fp32 bits.  Unused piece slots of the last
// chunk of a type hold offset 0, row p (the sink row of the accumulators) and value 0.
//
// Space.  Records take at most 2 words per entry, a block adds at most 12 + 6 words (header, the
// unused piece slots of its last chunk of type 1), and a group has at most NB + 1 + nnz_g / seg
// blocks, so (2 + 18 / 24 <= 3)
//     3 * nnz_g + 56 * (ceil(k / 64) + 2)
// words bound a stream and no prefix sum over groups is needed: stream (Q, w) starts at word
// band_stream_base(gIdxes[min(q, g)], q, k) with q = W*Q + w.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gcoo {

constexpr int kBandRows = 64;            // rows of B per band
constexpr int kBandRunCap = 32;          // longest run (more entries of one column in a group, from repeated coordinates, form several runs)
constexpr int kBandHdr = 12;             // header words of a block
constexpr int kBandMaxP = 32;            // the kernel keeps 4 columns per lane
constexpr int64_t kBandMaxK = 262144;    // the column bitmap of a super-group is built in LDS

// groups per super-group = waves per workgroup, for groups of p rows
__host__ __device__ constexpr int band_waves(int p) { return p <= 16 ? 16 : 8; }
// runs that start within this many entries of a block's first entry share the block
__host__ __device__ constexpr int band_seg(int W) { return W == 8 ? 68 : 24; }
// words of the largest block: 12 + 8 * ceil((seg + 31) / 4)
__host__ __device__ constexpr int band_block_max(int W) { return W == 8 ? 256 : 128; }

__host__ __device__ constexpr int band_pieces_per_chunk(int t) { return t <= 2 ? 4 : (t == 4 ? 2 : 1); }
__host__ __device__ constexpr int band_chunk_words(int t) { return t == 1 ? 8 : 12; }
// words before the row bytes / before the values inside a chunk
__host__ __device__ constexpr int band_chunk_rows_at(int t) { return t <= 2 ? 2 : 1; }
__host__ __device__ constexpr int band_chunk_vals_at(int t) { return 4; }

__host__ __device__ inline int64_t band_stream_slack(int64_t k) { return 56 * ((k + 63) / 64 + 2) + 4; }
__host__ __device__ inline int64_t band_stream_base(int64_t first_entry, int64_t q, int64_t k)
{
    return (3 * first_entry + 3) / 4 * 4 + band_stream_slack(k) * q;
}
__host__ __device__ inline int64_t band_stream_words(int64_t nnz, int64_t g, int64_t k, int W)
{
    const int64_t nq = (g + W - 1) / W;
    return band_stream_base(nnz, nq * W, k) + 256;   // the kernel reads whole blocks: slack behind the last one
}

}  // namespace gcoo
