// Kernels that write the share schedule (layout in gcoo_share.hpp) from the finished GCOO arrays: the
// distinct columns of every super-group (share_union), then headers and records (share_fill).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gcoo_share.hpp"

namespace gcoo {

constexpr int kShareBuildThreads = 1024;
constexpr int kShareBuildWaves = kShareBuildThreads / 64;


// Exclusive prefix sum over the kShareBuildThreads values `mine` (one per thread); returns this
// thread's offset and leaves the total in *total_s (shared).  `wsum` is shared scratch.
__device__ __forceinline__ int32_t share_block_scan(int32_t mine, int32_t* wsum, int32_t* total_s)
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
    if (threadIdx.x == kShareBuildThreads - 1) *total_s = off + mine;
    __syncthreads();
    return off;
}

// ---------------------------------------------------------------------------------------------
// ucols(Q): one workgroup per super-group marks the columns of its entries in a bitmap in LDS
// (bit sets commute, so the order of the atomics is irrelevant), counts the bits in front of every
// bitmap word and lists the set bits in ascending order.  ucols(Q) is written to the slice of
// `ucols` that starts at the super-group's first entry (it cannot be longer than its entries).
// Dynamic LDS: ceil(k/32) words.
// ---------------------------------------------------------------------------------------------
// Marks the columns of the entries [e0, e1) in the bitmap `bits` (LDS, nbw words, cleared here).
__device__ __forceinline__ void share_mark(const int32_t* __restrict__ cols, int32_t e0, int32_t e1, uint32_t* bits, int32_t nbw)
{
    for (int32_t i = threadIdx.x; i < nbw; i += kShareBuildThreads) bits[i] = 0u;
    __syncthreads();
    // A thread takes eight consecutive entries at a time and collects the bits of one bitmap word in a register
    // while the word stays the same (the columns of a group ascend, so it mostly does): one atomic per word
    // and thread instead of one per entry, and the lanes of a wave, 8 entries apart, rarely meet in a word.
    // (One atomic per entry cost 110 clocks per wave instruction: most of its lanes hit the same two or three words.)
    constexpr int kChunk = 8;
    for (int32_t e = e0 + kChunk * (int32_t)threadIdx.x; e < e1; e += kChunk * kShareBuildThreads) {
        uint32_t c[kChunk];
#pragma unroll
        for (int u = 0; u < kChunk; ++u) c[u] = e + u < e1 ? (uint32_t)cols[e + u] : 0xFFFFFFFFu;
        uint32_t word = c[0] >> 5, acc = 0u;
#pragma unroll
        for (int u = 0; u < kChunk; ++u) {
            if (c[u] == 0xFFFFFFFFu) break;
            if ((c[u] >> 5) != word) {
                atomicOr(&bits[word], acc);
                word = c[u] >> 5;
                acc = 0u;
            }
            acc |= 1u << (c[u] & 31u);
        }
        if (acc) atomicOr(&bits[word], acc);
    }
    __syncthreads();
}

// First half of share_union spread over the machine: one workgroup per group writes the bitmap of the group's
// columns to parts[q * nbw ..] (whole, zero words included, so the array needs no clearing).  A super-group of
// 50 000 entries keeps one workgroup busy for 30 us; its eight groups side by side take a fifth of that.
__global__ __launch_bounds__(kShareBuildThreads) void share_mark_groups(const int32_t* __restrict__ gIdxes, const int32_t* __restrict__ cols,
                                                                       int64_t k, uint32_t* __restrict__ parts)
{
    extern __shared__ uint32_t share_union_lds[];
    const int32_t nbw = (int32_t)((k + 31) / 32);
    const int64_t q = blockIdx.x;
    share_mark(cols, gIdxes[q], gIdxes[q + 1], share_union_lds, nbw);
    uint32_t* out = parts + q * nbw;
    for (int32_t i = threadIdx.x; i < nbw; i += kShareBuildThreads) out[i] = share_union_lds[i];
}

// `parts` != nullptr: the bitmaps of the groups are there (share_mark_groups) and are ORed together instead of
// marking the entries here.
__global__ __launch_bounds__(kShareBuildThreads) void share_union(const int32_t* __restrict__ gIdxes, const int32_t* __restrict__ cols,
                                                               int64_t g, int64_t k, int32_t W,
                                                               int32_t* __restrict__ ucols, int32_t* __restrict__ ucount,
                                                               uint32_t* __restrict__ zeroed, const uint32_t* __restrict__ parts)
{
    if (zeroed && blockIdx.x == 0 && threadIdx.x == 0) *zeroed = 0u;   // a counter of the kernel that runs next
    extern __shared__ uint32_t share_union_lds[];
    __shared__ int32_t wsum[kShareBuildWaves];
    __shared__ int32_t total_s;
    const int32_t nbw = (int32_t)((k + 31) / 32);
    uint32_t* bits = share_union_lds;
    const int64_t Q = blockIdx.x;
    const int64_t q0 = Q * W, q1 = (q0 + W < g) ? q0 + W : g;
    const int32_t e0 = gIdxes[q0], e1 = gIdxes[q1];
    if (parts) {
        for (int32_t i = threadIdx.x; i < nbw; i += kShareBuildThreads) {
            uint32_t b = 0u;
            for (int64_t q = q0; q < q1; ++q) b |= parts[q * nbw + i];
            bits[i] = b;
        }
        __syncthreads();
    } else {
        share_mark(cols, e0, e1, bits, nbw);
    }
    // thread t owns the words [t*per, (t+1)*per)
    const int32_t per = (nbw + kShareBuildThreads - 1) / kShareBuildThreads;
    const int32_t w0 = (int32_t)threadIdx.x * per, w1 = (w0 + per < nbw) ? w0 + per : nbw;
    int32_t mine = 0;
    for (int32_t w = w0; w < w1; ++w) mine += __popc(bits[w]);
    int32_t at = e0 + share_block_scan(mine, wsum, &total_s);
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


// Where the entries of a (group, band) that spans [s, e) stand in their runs.  A run is a maximal stretch of one
// column, cut into stretches of kShareRunCap from its first entry; *x = the entry's place in its stretch, *len = the
// stretch's length.  `col_at(i)` = column of entry i.
// share_place_wave does it for the 64 entries cur .. cur+63 of the band at once (lane l: entry cur + l; every lane of the wave must
// call it), without a walk along the run per entry: the lanes mark where a run starts, a ballot gives every lane the
// start and the end of its run inside the 64, lane 0 alone walks back to the start of a run that began before them,
// and 32 lanes look at the 32 entries behind (a stretch ends at most kShareRunCap - 1 entries after one of its entries).
template <typename ColAt>
__device__ __forceinline__ void share_place_wave(ColAt col_at, int32_t s, int32_t e, int32_t cur, int lane, int32_t* x, int32_t* len)
{
    static_assert(kShareRunCap == 32, "the look-ahead below is 32 entries");
    const int32_t i = cur + lane;
    const bool valid = i < e;
    const int32_t c = valid ? col_at(i) : 0;
    const bool start = !valid || i == s || col_at(i - 1) != c;
    const uint64_t b1 = __ballot(start);
    const int32_t i2 = cur + 64 + lane;
    const bool start2 = lane < 32 && (i2 >= e || col_at(i2) != col_at(i2 - 1));
    const uint64_t b2 = __ballot(start2);
    int32_t carry = 0;                                // entries of the first run in front of cur
    if ((b1 & 1ull) == 0) {                           // (then cur < e and cur > s)
        if (lane == 0) {
            while (cur - 1 - carry >= s && col_at(cur - 1 - carry) == c) ++carry;
        }
        carry = __shfl(carry, 0, 64);
    }
    const uint64_t upto = b1 & (lane == 63 ? ~0ull : ((2ull << lane) - 1ull));
    const int32_t d = upto ? lane - (63 - __clzll(upto)) : lane + carry;     // entries of the run in front of entry i
    const int32_t pos = d % kShareRunCap;
    const uint64_t after = lane == 63 ? 0ull : (b1 & ~((2ull << lane) - 1ull));
    const int32_t run_end = after ? __ffsll((long long)after) - 1 : (b2 ? 64 + __ffsll((long long)b2) - 1 : 96);
    const int32_t n = run_end - (lane - pos);
    *x = pos;
    *len = n < kShareRunCap ? n : kShareRunCap;
}

typedef uint32_t share_u32x4 __attribute__((ext_vector_type(4)));

// One workgroup per stream q = 8Q + w, also for the groups behind the last one of the last super-group
// (their streams are empty, their headers zero).  Band b of the group is the entry range
// [bstart[b], bstart[b+1]).  Pass 1 (a wave per band): quads and singles of every band -> header, blocks
// of the band; prefix sum over the bands; the stream's place is taken from the atomic counter `alloc`
// (zero before the launch).  Pass 2 (the same waves): the records.
// The walk over a band is a chain of dependent reads of neighbouring columns (where does the run of this entry
// begin and end), and the band starts come from binary searches: from global memory each step is a memory
// latency and a stream of 170 bands took 60 us.  A group of at most `stage_cap` entries therefore copies its columns
// to LDS first and reads them there; a larger one reads global memory.
// Dynamic LDS: 4 * (ceil(k / 48) + 1) + stage_cap words.
__global__ __launch_bounds__(kShareBuildThreads) void share_fill(const int32_t* __restrict__ gIdxes, const int32_t* __restrict__ rows,
                                                                const int32_t* __restrict__ cols, const float* __restrict__ values,
                                                                int32_t p, int64_t g, int64_t k, const int32_t* __restrict__ ucols,
                                                                const int32_t* __restrict__ ucount, uint32_t* __restrict__ hdr,
                                                                uint32_t* __restrict__ blocks, int32_t* __restrict__ sbase,
                                                                uint32_t* __restrict__ alloc, int32_t stage_cap)
{
    extern __shared__ uint32_t share_lds[];
    __shared__ int32_t wsum[kShareBuildWaves];
    __shared__ int32_t total_s;
    __shared__ int32_t carry_s;
    __shared__ int32_t base_s;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int64_t q = blockIdx.x, Q = q / kShareW;
    const int w = (int)(q - Q * kShareW);
    const int32_t first = gIdxes[Q * kShareW < g ? Q * kShareW : g];
    const int32_t first_next = gIdxes[(Q + 1) * kShareW < g ? (Q + 1) * kShareW : g];
    const int32_t nU = ucount[Q];
    const int32_t NB = (nU + kShareBandRows - 1) / kShareBandRows;
    const int32_t* uc = ucols + first;
    const int32_t beg = gIdxes[q < g ? q : g], end = gIdxes[q < g ? q + 1 : g];
    const int32_t row0 = (int32_t)(q * p);
    const int64_t hb = share_hdr_base(first, Q), cap = share_hdr_base(first_next, Q + 1) - hb;
    uint32_t* hd = hdr + 2 * (hb * kShareW + w * cap);
    int32_t* bstart = reinterpret_cast<int32_t*>(share_lds);         // [NB + 1]
    const int32_t table = (int32_t)((k + kShareBandRows - 1) / kShareBandRows + 1);
    int32_t* boff = bstart + table;      // [NB + 1] blocks per band, then offsets
    int32_t* hq = boff + table;          // quads of band b
    int32_t* hs = hq + table;            // groups of four singles of band b
    int32_t* stage = hs + table;         // columns of the group's entries, if they fit
    const bool staged = end - beg <= stage_cap;
    if (staged) {
        for (int32_t i = beg + (int32_t)threadIdx.x; i < end; i += kShareBuildThreads) stage[i - beg] = cols[i];
        __syncthreads();
    }
    auto col_at = [&](int32_t i) -> int32_t { return staged ? stage[i - beg] : cols[i]; };

    for (int32_t b = threadIdx.x; b <= NB; b += kShareBuildThreads) {
        int32_t lo = beg, hi = end;
        if (b < NB) {
            const int32_t c = uc[b * kShareBandRows];
            while (lo < hi) {
                const int32_t mid = lo + (hi - lo) / 2;
                if (col_at(mid) < c) lo = mid + 1; else hi = mid;
            }
        } else {
            lo = end;
        }
        bstart[b] = lo;
    }
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();

    // pass 1
    for (int32_t b = wv; b < NB; b += kShareBuildWaves) {
        const int32_t s = bstart[b], e = bstart[b + 1];
        int32_t members = 0, singles = 0;
        for (int32_t cur = s; cur < e; cur += 64) {
            int32_t x, len;
            share_place_wave(col_at, s, e, cur, lane, &x, &len);
            const bool live = cur + lane < e;
            const bool member = live && x < (len & ~3);
            members += __popcll(__ballot(member));
            singles += __popcll(__ballot(live && !member));
        }
        const int32_t nq = members / 4, ns4 = (singles + 3) / 4;
        if (lane == 0) {
            hd[(int64_t)b * 2] = (uint32_t)nq;
            hd[(int64_t)b * 2 + 1] = (uint32_t)ns4;
            hq[b] = nq;
            hs[b] = ns4;
            boff[b] = (nq + 3) / 4 + (ns4 + 3) / 4;
        }
    }
    __syncthreads();
    // exclusive prefix sum of the blocks per band, kShareBuildThreads bands at a time
    for (int32_t t0 = 0; t0 < NB; t0 += kShareBuildThreads) {
        const int32_t b = t0 + (int32_t)threadIdx.x;
        const int32_t mine = b < NB ? boff[b] : 0;
        const int32_t off = share_block_scan(mine, wsum, &total_s);
        if (b < NB) boff[b] = carry_s + off;
        __syncthreads();
        if (threadIdx.x == 0) carry_s += total_s;
        __syncthreads();
    }
    // What pass 2 reads from global memory for a band (the band's columns, one per lane, ascending, lanes past the
    // end holding a column no entry has; value and row of the first 64 entries) is requested a band ahead: a wave
    // walks its bands one after another, and a memory latency per band would be most of its time.
    struct Ahead { int32_t band_col; float value; int32_t row; };
    auto fetch = [&](int32_t b) -> Ahead {
        Ahead a = {INT32_MAX, 0.0f, 0};
        if (b < NB) {
            const int32_t nc = (nU - b * kShareBandRows < kShareBandRows) ? nU - b * kShareBandRows : kShareBandRows;
            if (lane < nc) a.band_col = uc[b * kShareBandRows + lane];
            const int32_t i = bstart[b] + lane;
            if (i < bstart[b + 1]) {
                a.value = values[i];
                a.row = rows[i];
            }
        }
        return a;
    };
    Ahead ahead = fetch(wv);
    if (threadIdx.x == 0) {
        const int32_t base = (int32_t)atomicAdd(alloc, (uint32_t)carry_s);
        base_s = base;
        sbase[q] = base;
    }
    __syncthreads();
    share_u32x4* out = reinterpret_cast<share_u32x4*>(blocks) + (int64_t)base_s * 16;
    const share_u32x4 unused = {0u, (uint32_t)kShareSink, 0u, 0u};

    // pass 2
    for (int32_t b = wv; b < NB; b += kShareBuildWaves) {
        const Ahead now = ahead;
        ahead = fetch(b + kShareBuildWaves);
        const int32_t s = bstart[b], e = bstart[b + 1];
        if (s >= e) continue;
        // an entry's slot is a lower bound over the lanes' columns, six exchanges
        const int32_t band_col_of_lane = now.band_col;
        share_u32x4* qblk = out + (int64_t)boff[b] * 16;
        int32_t members_before = 0, singles_before = 0;         // in the tiles before this one
        int32_t nq_blocks = 0;                                    // known after the walk: S blocks sit behind the Q blocks
        // the Q blocks need the band's quad count first: pass 1 left it
        const int32_t nq = hq[b], ns4 = hs[b];
        nq_blocks = (nq + 3) / 4;
        share_u32x4* sblk = qblk + (int64_t)nq_blocks * 16;
        for (int32_t cur = s; cur < e; cur += 64) {
            const int32_t i = cur + lane;
            const bool live = i < e;
            int32_t x = 0, len = 0, col = 0;
            share_place_wave(col_at, s, e, cur, lane, &x, &len);
            if (live) col = col_at(i);
            float value = now.value;
            int32_t row = now.row;
            if (cur != s && live) {
                value = values[i];
                row = rows[i];
            }
            const bool member = live && x < (len & ~3);
            const bool single = live && !member;
            const uint64_t mm = __ballot(member), sm = __ballot(single);
            const uint64_t below = (1ull << lane) - 1ull;
            int32_t slot = 0;
#pragma unroll
            for (int step = 32; step >= 1; step >>= 1) {
                const int32_t probe = __shfl(band_col_of_lane, slot + step - 1, 64);
                if (probe < col) slot += step;
            }
            if (live) {
                const share_u32x4 rec = {__float_as_uint(value), (uint32_t)(row - row0), (uint32_t)slot * 1024u, 0u};
                if (member) {
                    const int32_t u = x & 3;
                    const int32_t rank = (members_before + __popcll(mm & below) - u) / 4;
                    qblk[(int64_t)(rank / 4) * 16 + (rank % 4) * 4 + u] = rec;
                } else {
                    const int32_t rank = singles_before + __popcll(sm & below);
                    sblk[(int64_t)(rank / 16) * 16 + rank % 16] = rec;
                }
            }
            members_before += __popcll(mm);
            singles_before += __popcll(sm);
        }
        // records that no entry owns
        {
            const int32_t used = nq * 4, room = nq_blocks * 16;
            if (used + lane < room) qblk[used + lane] = unused;
            const int32_t sused = singles_before, sroom = ((ns4 + 3) / 4) * 16;
            if (sused + lane < sroom) sblk[sused + lane] = unused;
        }
    }
}

}  // namespace gcoo
