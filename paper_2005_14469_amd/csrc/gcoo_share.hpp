// The share schedule: the kernel-private re-listing of a GCOO matrix that the workgroup-shared SpDM
// kernel reads (gcoo_spdm_share_kernel.hpp).
//
// Why.  Algorithm 2 lets every thread block fetch the B value of each of its entries from global
// memory and counts on the caches for reuse between blocks (Section 3.3).  On this machine the
// vector-cache path delivers 64 bytes per clock and compute unit, LDS four times as much, so the
// rows of B that the groups of a workgroup need are fetched once into LDS and every multiply-add
// reads its B values from there.  The more rows of A share a fetched row, the fewer bytes cross
// the cache path: a workgroup therefore covers a super-group of kShareW = 8 consecutive groups of
// up to kShareMaxP = 48 rows (up to 384 rows of A), one wave per group.
//
// Bands.  ucols(Q) = the distinct columns that hold an entry of super-group Q, ascending (rows of
// B that no entry of Q touches are never fetched).  Band b of Q = ucols[48b .. 48b+47]: the rows
// of B that are in LDS together, a row's slot being its place in the band.  The entries of a
// group are in (column, row) order (Section 3.1), so the entries of one (group, band) are
// contiguous in the GCOO arrays.
//
// Blocks.  The entries of one (group, band) are re-listed in blocks of 16 records of 16 bytes:
//     record = { value (fp32 bits), row inside the group, byte offset of the B row inside the
//                band (slot * 1024), 0 }
// A maximal stretch of entries of one column (a run, cut into stretches of at most kShareRunCap)
// gives floor(len / 4) quads and len % 4 singles.
//   Q blocks (first): four quads each; records 4i .. 4i+3 are the four entries of quad i and all
//     carry the quad's offset, so the kernel reads the B row once per quad (the reuse of the
//     fetched value along a run, Algorithm 2).
//   S blocks (then): sixteen singles each; the kernel handles them four at a time, so the singles
//     of a band are padded to a multiple of four.
// Unused records (of a last Q block, of a last group of four singles, of the rest of a last S block)
// hold value 0, row kShareSink and offset 0: they add zero to a partial sum that is never stored.
//
// Streams.  The blocks of a group, band after band, form one contiguous stream of 256-byte blocks;
// sbase[q] is the index of its first block (the streams are placed by an atomic counter, so
// their order in memory is not fixed, only their content).  The kernel reads a stream strictly
// front to back, four blocks (1 KB) per load, up to eight blocks beyond its end: the array has that
// much slack.
//
// Headers.  Every stream has its own array of (quads, groups of four singles) pairs, one per band:
// hdr[2 * (8 * hbase(Q) + w * (hbase(Q+1) - hbase(Q)) + b) + {0, 1}] for wave w and band b, with
// hbase(Q) = gIdxes[8Q] / 48 + Q (a super-group has at most nnz_Q / 48 + 1 bands).  The kernel loads the
// pairs of 64 bands at a time, two such loads ahead: the array ends with that much slack.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gcoo {

constexpr int kShareW = 8;               // groups per super-group = waves per workgroup
constexpr int kShareMaxP = 48;           // tallest group: (48 + 1) x 4 partial sums per lane in v[60:255]
constexpr int kShareSink = kShareMaxP;   // row of the records that multiply by zero
constexpr int kShareBandRows = 48;       // rows of B per band
constexpr int kShareRunCap = 32;         // longest run (a multiple of 4; repeated coordinates can make longer ones)
constexpr int kShareBlockWords = 64;     // 16 records x 4 words
constexpr int kShareRingBlocks = 8;      // per wave in LDS: two pieces of four blocks
constexpr int kShareSlackBlocks = 16;    // read-ahead of the kernel behind the last stream
constexpr int64_t kShareMaxK = 262144;   // the column bitmap of a super-group is built in LDS

__host__ __device__ inline int64_t share_super_groups(int64_t g) { return (g + kShareW - 1) / kShareW; }
__host__ __device__ inline int64_t share_hdr_base(int64_t first_entry_of_Q, int64_t Q) { return first_entry_of_Q / kShareBandRows + Q; }
constexpr int kShareHdrSlackBands = 256;
// words of the header array
__host__ __device__ inline int64_t share_hdr_words(int64_t nnz, int64_t g)
{
    return (share_hdr_base(nnz, share_super_groups(g)) * kShareW + kShareHdrSlackBands) * 2;
}
// upper bound of the blocks of all streams: a (group, band) with n > 0 entries has at most
// ceil(n/16) + 1 <= n/16 + 2 blocks, and there are at most min(nnz, groups x bands) such pairs
__host__ __device__ inline int64_t share_stream_blocks(int64_t nnz, int64_t g, int64_t k)
{
    const int64_t pairs_by_shape = share_super_groups(g) * kShareW * ((k + kShareBandRows - 1) / kShareBandRows);
    const int64_t pairs = nnz < pairs_by_shape ? nnz : pairs_by_shape;
    return nnz / 16 + 2 * pairs + kShareSlackBlocks;
}

}  // namespace gcoo
