// Kernels that write the band schedule (layout in gcoo_band.hpp) from the finished GCOO arrays.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gcoo_band.hpp"

namespace gcoo {

constexpr int kBandBuildThreads = 1024;
constexpr int kBandBuildWaves = kBandBuildThreads / 64;

// Exclusive prefix sum over the kBandBuildThreads values `mine` (one per thread); returns this
// thread's offset and leaves the total in *total_s (shared).  `wsum` is shared scratch.
__device__ __forceinline__ int32_t band_block_scan(int32_t mine, int32_t* wsum, int32_t* total_s)
{
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    int32_t incl = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int32_t t = __shfl_up(incl, d, 64);
        if (lane >= d) incl += t;
    }
    if (lane == 63) wsum[wv] = incl;
    __syncthreads();
    int32_t off = incl - mine;
    for (int j = 0; j < wv; ++j) off += wsum[j];
    if (threadIdx.x == kBandBuildThreads - 1) *total_s = off + mine;
    __syncthreads();
    return off;
}

// ---------------------------------------------------------------------------------------------
// ucols(Q): one workgroup per super-group marks the columns of its entries in a bitmap in LDS
// (bit sets commute, so the order of the atomics is irrelevant), counts the bits in front of every
// bitmap word and lists the set bits in ascending order.  ucols(Q) is written to the slice of
// `ucols` that starts at the super-group's first entry (it cannot be longer than its entries).
// Dynamic LDS: 2 * ceil(k/32) words.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBandBuildThreads) void band_union(const int32_t* __restrict__ gIdxes, const int32_t* __restrict__ cols,
                                                               int64_t g, int64_t k, int32_t W,
                                                               int32_t* __restrict__ ucols, int32_t* __restrict__ ucount)
{
    extern __shared__ uint32_t band_lds[];
    __shared__ int32_t wsum[kBandBuildWaves];
    __shared__ int32_t total_s;
    const int32_t nbw = (int32_t)((k + 31) / 32);
    uint32_t* bits = band_lds;
    const int64_t Q = blockIdx.x;
    const int64_t q0 = Q * W, q1 = (q0 + W < g) ? q0 + W : g;
    const int32_t e0 = gIdxes[q0], e1 = gIdxes[q1];
    for (int32_t i = threadIdx.x; i < nbw; i += kBandBuildThreads) bits[i] = 0u;
    __syncthreads();
    for (int32_t e = e0 + (int32_t)threadIdx.x; e < e1; e += kBandBuildThreads) {
        const uint32_t c = (uint32_t)cols[e];
        atomicOr(&bits[c >> 5], 1u << (c & 31u));
    }
    __syncthreads();
    // thread t owns the words [t*per, (t+1)*per)
    const int32_t per = (nbw + kBandBuildThreads - 1) / kBandBuildThreads;
    const int32_t w0 = (int32_t)threadIdx.x * per, w1 = (w0 + per < nbw) ? w0 + per : nbw;
    int32_t mine = 0;
    for (int32_t w = w0; w < w1; ++w) mine += __popc(bits[w]);
    int32_t at = e0 + band_block_scan(mine, wsum, &total_s);
    for (int32_t w = w0; w < w1; ++w) {
        uint32_t b = bits[w];
        while (b) {
            const int bit = __ffs(b) - 1;
            b &= b - 1u;
            ucols[at++] = w * 32 + bit;
        }
    }
    if (threadIdx.x == 0) ucount[Q] = total_s;
}

// ---------------------------------------------------------------------------------------------
// Piece of a run of `len` entries that the entry at place x of the run belongs to: runs are cut
// into pieces of 8 from the front; the rest r < 8 is cut into 4, 2, 1 as the bits of r say.
// Returns the piece's length and writes the place of its first entry.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ int band_piece_of(int len, int x, int* piece_first)
{
    const int full = len & ~7;
    if (x < full) { *piece_first = x & ~7; return 8; }
    const int r = len - full;
    int at = full;
    if (r & 4) { if (x < at + 4) { *piece_first = at; return 4; } at += 4; }
    if (r & 2) { if (x < at + 2) { *piece_first = at; return 2; } at += 2; }
    *piece_first = at;
    return 1;
}

__device__ __forceinline__ int band_type_index(int t) { return t == 1 ? 0 : (t == 2 ? 1 : (t == 4 ? 2 : 3)); }
// a[k] for a run-time k without making `a` an array in memory
template <class X>
__device__ __forceinline__ X band_pick(const X (&a)[4], int k) { return k == 0 ? a[0] : (k == 1 ? a[1] : (k == 2 ? a[2] : a[3])); }

// One wave: the blocks of one (group, band).  Entries [s, e) of the group (columns ascending, all
// inside the band), band_cols = the band's columns (ncols of them).  With out == nullptr only
// the size is computed.  Returns the words of all blocks of the band (the same in every lane).
//   next_cols, next_ids   header fields of the band's first block
__device__ __forceinline__ int32_t band_blocks_of(const int32_t* __restrict__ rows, const int32_t* __restrict__ cols,
                                                  const float* __restrict__ values, int32_t s, int32_t e, int32_t row0, int32_t p,
                                                  const int32_t* __restrict__ band_cols, int32_t ncols, uint32_t* __restrict__ out,
                                                  int32_t next_cols, const int32_t* __restrict__ next_ids, int32_t total_words,
                                                  int32_t seg)
{
    const int lane = threadIdx.x & 63;
    int32_t words = 0;
    int32_t cur = s;
    bool first_block = true;
    // the band's columns, one per lane (ascending; lanes past the end hold a column no entry has):
    // the slot of an entry's column is then found with lane exchanges instead of reads of memory
    const int32_t band_col_of_lane = (out && lane < ncols) ? band_cols[lane] : INT32_MAX;
    do {
        // A run here is at most kBandRunCap entries of one column (an input that repeats a
        // coordinate can hold more: they form several runs).  The segment takes the runs that
        // start within seg = band_seg(W) entries of its first entry: at most seg + 31 entries, which
        // is also what the two tiles of 64 lanes below cover.
        int32_t seg_end = cur + seg;
        if (seg_end >= e) {
            seg_end = e;
        } else {
            const int32_t c = cols[seg_end];
            int32_t rs = seg_end;
            while (rs > cur && cols[rs - 1] == c) --rs;
            const int32_t cs = rs + (seg_end - rs) / kBandRunCap * kBandRunCap;   // start of the run that holds entry seg_end
            if (cs != seg_end) {
                int32_t stop = cs + kBandRunCap < e ? cs + kBandRunCap : e;
                while (seg_end < stop && cols[seg_end] == c) ++seg_end;
            }
        }
        const bool last_block = seg_end >= e;

        // per entry (two tiles of 64 lanes): type of its piece, head or not
        int type[2] = {0, 0}, in_piece[2] = {0, 0};
        int32_t head[2] = {0, 0};                         // entry index of the piece's first entry, relative to cur
        int32_t col_of[2] = {0, 0};
        uint64_t heads[2][4];
        const bool two_tiles = seg_end - cur > 64;        // the same in every lane: the second tile is skipped as a whole
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int32_t i = cur + t * 64 + lane;
            if ((t == 0 || two_tiles) && i < seg_end) {
                // the entry's column and its two neighbours in one go (three independent reads); the
                // loops read on only inside runs of three and more
                const int32_t c = cols[i];
                const int32_t before = i > cur ? cols[i - 1] : -1;
                const int32_t after = i + 1 < seg_end ? cols[i + 1] : -1;
                col_of[t] = c;
                int32_t rs = i, re = i + 1;
                if (before == c) {
                    --rs;
                    while (rs > cur && cols[rs - 1] == c) --rs;
                }
                rs += (i - rs) / kBandRunCap * kBandRunCap;
                if (after == c && re < rs + kBandRunCap) {
                    ++re;
                    while (re < seg_end && re < rs + kBandRunCap && cols[re] == c) ++re;
                }
                int pf;
                type[t] = band_piece_of(re - rs, i - rs, &pf);
                head[t] = rs + pf - cur;
                in_piece[t] = i - rs - pf;
            }
#pragma unroll
            for (int ti = 0; ti < 4; ++ti) heads[t][ti] = (t == 0 || two_tiles) ? __ballot(type[t] == (1 << ti) && in_piece[t] == 0) : 0ull;
        }
        // Pieces per type as cut from the runs (nat), then after the pieces of 4 and of 2 that
        // would leave a chunk partly filled have been halved into the next smaller type (cnt).
        int32_t nat[4], cnt[4], nch[4], off[4];
#pragma unroll
        for (int ti = 0; ti < 4; ++ti) nat[ti] = __popcll(heads[0][ti]) + __popcll(heads[1][ti]);
        cnt[3] = nat[3];
        cnt[2] = nat[2] & ~1;                                  // whole chunks of two 4s
        const int32_t twos = nat[1] + 2 * (nat[2] - cnt[2]);
        cnt[1] = twos & ~3;                                    // whole chunks of four 2s
        cnt[0] = nat[0] + 2 * (twos - cnt[1]);
        int32_t size = kBandHdr;
#pragma unroll
        for (int ti = 0; ti < 4; ++ti) {
            const int J = band_pieces_per_chunk(1 << ti);
            nch[ti] = (cnt[ti] + J - 1) / J;
            off[ti] = size;
            size += nch[ti] * band_chunk_words(1 << ti);
        }
        if (out) {
            uint32_t* blk = out + words;
            // header
            if (lane == 0) {
                blk[0] = (uint32_t)nch[0] | (uint32_t)nch[1] << 8 | (uint32_t)nch[2] << 16 | (uint32_t)nch[3] << 24;
                blk[1] = (last_block ? 1u : 0u) | (uint32_t)(cnt[0] & 3) << 1 | (first_block ? (uint32_t)next_cols << 8 : 0u);
                blk[2] = first_block ? (uint32_t)total_words : 0u;
                blk[3] = (uint32_t)size;
            }
            if (lane < 8) blk[4 + lane] = first_block ? (uint32_t)next_ids[lane] : 0u;
            // the words of a chunk that hold neither offsets, rows nor values
            for (int32_t i = lane; i < nch[0]; i += 64) blk[off[0] + i * 8 + 3] = 0u;
            for (int32_t i = lane; i < nch[2]; i += 64) blk[off[2] + i * 12 + 3] = 0u;
            for (int32_t i = lane; i < nch[3]; i += 64) blk[off[3] + i * 12 + 3] = 0u;
            // entries
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int32_t i = cur + t * 64 + lane;
                // slot of the entry's column inside the band = how many of the band's columns are smaller:
                // a lower bound over the 64 lanes, six exchanges, every lane takes part
                int32_t slot = 0;
                if (t == 0 || two_tiles) {
#pragma unroll
                    for (int step = 32; step >= 1; step >>= 1) {
                        const int32_t probe = __shfl(band_col_of_lane, slot + step - 1, 64);
                        if (probe < col_of[t]) slot += step;
                    }
                }
                if (i < seg_end) {
                    int T = type[t], u = in_piece[t];
                    const int nti = band_type_index(T);
                    const int32_t h = head[t];
                    int32_t rank;                                 // of the piece among the pieces of its type, in entry order
                    const uint64_t heads0 = band_pick(heads[0], nti), heads1 = band_pick(heads[1], nti);
                    if (h < 64) rank = __popcll(heads0 & ((1ull << h) - 1ull));
                    else rank = __popcll(heads0) + __popcll(heads1 & ((1ull << (h - 64)) - 1ull));
                    if (T == 4 && rank >= cnt[2]) {               // halved: two 2s behind the 2s cut from the runs
                        rank = nat[1] + 2 * (rank - cnt[2]) + (u >> 1);
                        u &= 1;
                        T = 2;
                    }
                    if (T == 2 && rank >= cnt[1]) {               // halved: two 1s behind the 1s cut from the runs
                        rank = nat[0] + 2 * (rank - cnt[1]) + u;
                        u = 0;
                        T = 1;
                    }
                    const int ti = band_type_index(T), J = band_pieces_per_chunk(T);
                    uint32_t* ch = blk + band_pick(off, ti) + (rank / J) * band_chunk_words(T);
                    const int j = rank % J;
                    reinterpret_cast<uint8_t*>(ch + band_chunk_rows_at(T))[j * T + u] = (uint8_t)(rows[i] - row0);
                    ch[band_chunk_vals_at(T) + j * T + u] = __float_as_uint(values[i]);
                    if (u == 0) reinterpret_cast<uint16_t*>(ch)[j] = (uint16_t)(slot * 1024);
                }
            }
            // unused piece slots of the last chunk of every type
#pragma unroll
            for (int ti = 0; ti < 4; ++ti) {
                const int T = 1 << ti, J = band_pieces_per_chunk(T);
                const int32_t slots = nch[ti] * J - cnt[ti];          // < J
                if (lane < slots * T) {
                    const int32_t rank = cnt[ti] + lane / T;
                    uint32_t* ch = blk + off[ti] + (rank / J) * band_chunk_words(T);
                    const int j = rank % J, u = lane % T;
                    reinterpret_cast<uint8_t*>(ch + band_chunk_rows_at(T))[j * T + u] = (uint8_t)p;
                    ch[band_chunk_vals_at(T) + j * T + u] = 0u;
                    if (u == 0) reinterpret_cast<uint16_t*>(ch)[j] = 0;
                }
                // the halves / bytes of the offset and row words that no piece slot owns
                if (lane == 0 && nch[ti] > 0) {
                    if (T == 8) {
                        for (int32_t c2 = 0; c2 < nch[ti]; ++c2) reinterpret_cast<uint16_t*>(blk + off[ti] + c2 * 12)[1] = 0;
                    }
                }
            }
        }
        words += size;
        cur = seg_end;
        first_block = false;
    } while (cur < e);
    return words;
}

// ---------------------------------------------------------------------------------------------
// One workgroup per stream (Q, w).  The entries of group q = W*Q + w are in column order, so band
// b of the group is the entry range [bstart[b], bstart[b+1]).  Pass 1: every wave sizes bands
// (wave v takes b = v, v + 16, ...); prefix sum over the bands; pass 2: the same waves write the
// blocks.  Dynamic LDS: 2 * (NBmax + 1) words with NBmax = ceil(k / 64).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBandBuildThreads, 8) void band_fill(const int32_t* __restrict__ gIdxes, const int32_t* __restrict__ rows,
                                                              const int32_t* __restrict__ cols, const float* __restrict__ values,
                                                              int32_t p, int64_t g, int64_t k, int32_t W,
                                                              const int32_t* __restrict__ ucols, const int32_t* __restrict__ ucount,
                                                              uint32_t* __restrict__ stream)
{
    extern __shared__ uint32_t band_lds[];
    __shared__ int32_t wsum[kBandBuildWaves];
    __shared__ int32_t total_s;
    __shared__ int32_t carry_s;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int64_t q = blockIdx.x, Q = q / W;
    const int w = (int)(q - Q * W);
    const int64_t q0 = Q * W;
    const int32_t R = kBandRows / W, seg = band_seg(W);
    const int32_t nU = ucount[Q];
    const int32_t NB = (nU + kBandRows - 1) / kBandRows;
    const int32_t* uc = ucols + gIdxes[q0];
    const int32_t beg = gIdxes[q < g ? q : g], end = gIdxes[q < g ? q + 1 : g];
    const int32_t row0 = (int32_t)(q * p);
    uint32_t* out = stream + band_stream_base(beg, q, k);
    int32_t* bstart = reinterpret_cast<int32_t*>(band_lds);          // [NB + 1]
    int32_t* boff = bstart + ((k + 63) / 64 + 1);                     // [NB + 1] sizes, then offsets

    for (int32_t b = threadIdx.x; b <= NB; b += kBandBuildThreads) {
        int32_t lo = beg, hi = end;
        if (b < NB) {
            const int32_t c = uc[b * kBandRows];
            while (lo < hi) {
                const int32_t mid = lo + (hi - lo) / 2;
                if (cols[mid] < c) lo = mid + 1; else hi = mid;
            }
        } else {
            lo = end;
        }
        bstart[b] = lo;
    }
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();

    auto band_ids = [&](int32_t b, int32_t* ncols_out, int32_t* ids) {
        // rows of B that wave w fetches for band b: slots t*W + w, t < R
        int32_t n = nU - b * kBandRows;
        n = n < 0 ? 0 : (n > kBandRows ? kBandRows : n);
        *ncols_out = n;
        if (lane < 8) {
            const int32_t slot = lane * W + w;
            ids[0] = (lane < R && slot < n) ? uc[b * kBandRows + slot] : 0;
        }
    };

    // pass 1: sizes
    for (int32_t b = wv; b < NB; b += kBandBuildWaves) {
        const int32_t nc = (nU - b * kBandRows < kBandRows) ? nU - b * kBandRows : kBandRows;
        const int32_t sz = band_blocks_of(rows, cols, values, bstart[b], bstart[b + 1], row0, p, uc + b * kBandRows, nc, nullptr, 0,
                                          nullptr, 0, seg);
        if (lane == 0) boff[b] = sz;
    }
    __syncthreads();
    // exclusive prefix sum of the sizes, kBandBuildThreads bands at a time; the pre-block comes first
    for (int32_t t0 = 0; t0 < NB; t0 += kBandBuildThreads) {
        const int32_t b = t0 + (int32_t)threadIdx.x;
        const int32_t mine = b < NB ? boff[b] : 0;
        const int32_t off = band_block_scan(mine, wsum, &total_s);
        if (b < NB) boff[b] = kBandHdr + carry_s + off;
        __syncthreads();
        if (threadIdx.x == 0) carry_s += total_s;
        __syncthreads();
    }
    if (threadIdx.x == 0) boff[NB] = kBandHdr + carry_s;
    __syncthreads();

    // the pre-block: what to fetch for band 0
    if (wv == 0) {
        int32_t nc, id = 0;
        band_ids(0, &nc, &id);
        if (lane == 0) { out[0] = 0u; out[1] = 1u | (uint32_t)nc << 8; out[2] = (uint32_t)kBandHdr; out[3] = (uint32_t)kBandHdr; }
        if (lane < 8) out[4 + lane] = (uint32_t)id;
    }
    // pass 2: blocks.  The ids of the next band go through LDS-free registers: lanes 0..7 hold them.
    __shared__ int32_t ids_s[kBandBuildWaves][8];
    for (int32_t b = wv; b < NB; b += kBandBuildWaves) {
        int32_t nc_next, id = 0;
        band_ids(b + 1, &nc_next, &id);
        if (lane < 8) ids_s[wv][lane] = id;
        __builtin_amdgcn_wave_barrier();
        const int32_t nc = (nU - b * kBandRows < kBandRows) ? nU - b * kBandRows : kBandRows;
        band_blocks_of(rows, cols, values, bstart[b], bstart[b + 1], row0, p, uc + b * kBandRows, nc, out + boff[b], nc_next,
                       ids_s[wv], boff[b + 1] - boff[b], seg);
        __builtin_amdgcn_wave_barrier();
    }
}

}  // namespace gcoo
