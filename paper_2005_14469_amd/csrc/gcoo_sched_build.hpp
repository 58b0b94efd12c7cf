// Kernel that writes the run schedule (layout in gcoo_sched.hpp) from the finished GCOO arrays.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gcoo_sched.hpp"

namespace gcoo {

// Where the pieces of class L land.  `x` = chunk index inside the class, `j` = piece inside the chunk.
__device__ __forceinline__ int32_t sched_col_word(int L, int32_t x, int j)
{
    const int J = runs_per_chunk(L);
    if (x < 3) return (x + 1) * J + j;                                        // pre-block
    const int32_t b = (x - 3) / kBody, sl = (x - 3) % kBody;
    return pre_dwords(L) + b * block_dwords(L) + sl * J + j;
}
__device__ __forceinline__ int32_t sched_block_word(int L, int32_t x) { return pre_dwords(L) + (x / kBody) * block_dwords(L); }

// Writes piece (x, j) of class L: its column and its L (row, value) pairs, read from entry e on.
// rows == nullptr writes a dummy piece (row p, value 0).
__device__ __forceinline__ void sched_put_piece(uint32_t* __restrict__ seg, int L, int32_t x, int j, uint32_t col,
                                                const int32_t* rows, const float* values, int32_t e, int32_t row0, int32_t p)
{
    const int J = runs_per_chunk(L), c = x % kBody;
    seg[sched_col_word(L, x, j)] = col;
    uint32_t* blk = seg + sched_block_word(L, x);
    uint8_t* rp = reinterpret_cast<uint8_t*>(blk + blk_rowpack(L, c));
    uint32_t* vp = blk + blk_val(L, c);
    // all loads first: the stores below may alias them for all the compiler knows, and a load behind every store
    // makes a piece of eight entries a chain of eight memory latencies
    int32_t r[kMaxRun];
    uint32_t v[kMaxRun];
#pragma unroll
    for (int i = 0; i < kMaxRun; ++i) {
        r[i] = (rows && i < L) ? rows[e + i] - row0 : p;
        v[i] = (rows && i < L) ? __float_as_uint(values[e + i]) : 0u;
    }
#pragma unroll
    for (int i = 0; i < kMaxRun; ++i)
        if (i < L) {
            rp[j * L + i] = (uint8_t)r[i];
            vp[j * L + i] = v[i];
        }
    (void)J;
}

// The groups in order of falling size (ties: the lower index first) and those sizes, which the kernel for
// launches of few items takes its work from.  A workgroup of `threads` threads ranks the groups `part` * threads ..
// (part + 1) * threads - 1: each of them counts the groups that come before it in that order (g <= kOrderMaxGroups:
// the sizes of all groups fit `size_s` in LDS, 16-byte aligned, and the count is a loop over them, four at a time).
__device__ __forceinline__ void rank_groups_by_size(const int32_t* __restrict__ gIdxes, int32_t gi, int32_t* __restrict__ order,
                                                    int32_t* __restrict__ osize, int32_t* size_s, int tid, int threads, int32_t part)
{
    const int32_t g4 = (gi + 3) & ~3;
    for (int32_t i = tid; i < g4; i += threads) size_s[i] = i < gi ? gIdxes[i + 1] - gIdxes[i] : -1;
    __syncthreads();
    typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
    for (int32_t i = part * threads + tid; i < gi && i < (part + 1) * threads; i += threads) {
        const int32_t mine = size_s[i];
        int32_t before = 0;
#pragma unroll 4
        for (int32_t j = 0; j < g4; j += 4) {
            const i32x4 o = *reinterpret_cast<const i32x4*>(&size_s[j]);
            before += (o.x > mine || (o.x == mine && j < i)) ? 1 : 0;
            before += (o.y > mine || (o.y == mine && j + 1 < i)) ? 1 : 0;
            before += (o.z > mine || (o.z == mine && j + 2 < i)) ? 1 : 0;
            before += (o.w > mine || (o.w == mine && j + 3 < i)) ? 1 : 0;
        }
        order[before] = i;
        osize[before] = mine;
    }
}

__global__ __launch_bounds__(1024) void group_order_by_size(const int32_t* __restrict__ gIdxes, int32_t g,
                                                            int32_t* __restrict__ order, int32_t* __restrict__ osize)
{
    __shared__ __attribute__((aligned(16))) int32_t size_s[kOrderMaxGroups];
    rank_groups_by_size(gIdxes, g, order, osize, size_s, threadIdx.x, 1024, (int32_t)blockIdx.x);
}

// One workgroup (kBuildThreads threads) per (group, window): blockIdx.x = q*nw + w.  Pass 1 counts
// the pieces of each class, pass 2 gives every piece its rank inside its class (entries are
// visited in order; ranks come from ballots and running counts, so the listing is the same on
// every run) and writes it out.  The windows of a group do not wait for each other: window w
// (entries [wb, we) of the group) owns the words from 3*(wb - beg) + kSchedPad*w of the group's
// part of the stream, which the space bound of gcoo_sched.hpp (3 words per entry and kSchedPad
// per window) makes disjoint.
// kBuildThreads = 256 or 1024: the launcher takes the small workgroup when a window holds few
// entries, so that eight of them share a compute unit instead of two.
// Finding the piece of an entry is a chain of dependent reads of neighbouring columns, and the window's
// bounds come from searches in the group's columns: from global memory every step of either is a memory
// latency (config 2: 0.25 ms for 6.4 M entries, seven times what the traffic needs).  So the bounds are
// found by a wave each, 64 probes per step, and a window of at most kStage entries copies its columns to
// LDS first and reads them there.
template <int kBuildThreads>
__global__ __launch_bounds__(kBuildThreads) void build_schedule(const int32_t* __restrict__ gIdxes, const int32_t* __restrict__ rows,
                                                      const int32_t* __restrict__ cols, const float* __restrict__ values,
                                                      int32_t p, int64_t g, int32_t nw, int32_t window_cols,
                                                      SchedClass* __restrict__ hdr, uint32_t* __restrict__ stream,
                                                      int32_t* __restrict__ order, int32_t* __restrict__ osize)
{
    __shared__ int32_t wstart[2];                 // first entry of this window and of the next
    __shared__ int32_t cnt[kMaxRun];              // pieces per class
    __shared__ int32_t demote[kMaxRun];           // class listed as pieces of class 1
    __shared__ int32_t seg[kMaxRun];              // first word of the class segment
    __shared__ int32_t base[kMaxRun];             // pieces of the class already placed
    constexpr int kBuildWaves = kBuildThreads / 64;
    __shared__ int32_t wcnt[kBuildWaves][kMaxRun];          // per wave, per class, in the current tile
    constexpr int kStage = kBuildThreads == 256 ? 4096 : 12288;
    static_assert(kStage >= kOrderMaxGroups, "the workgroup that ranks the groups keeps their sizes here");
    (void)order;
    (void)osize;
    __shared__ __attribute__((aligned(16))) int32_t stage[kStage];
    __shared__ uint8_t piece_s[kStage];           // staged window: place in its piece (3 bits) and length of the piece - 1 (3 bits) of every entry
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int64_t q = blockIdx.x / nw;
    const int32_t w = (int32_t)(blockIdx.x - q * nw);
    if (q >= g) {
        // The small-workgroup instance (matrices of small windows, where a launch more would show in the conversion
        // time) has a workgroup more per 256 groups than there are (group, window) pairs where the matrix has few
        // groups: they rank the groups by size.  The large-workgroup instance leaves that to a launch of its own
        // (group_order_by_size): with this code inside, it ran 40 % slower on 6.4 M entries.
        if constexpr (kBuildThreads == 256) {
            if (order != nullptr) rank_groups_by_size(gIdxes, (int32_t)g, order, osize, stage, tid, kBuildThreads, (int32_t)(blockIdx.x - g * nw));
        }
        return;
    }
    const int32_t beg = gIdxes[q], end = gIdxes[q + 1];
    const int32_t row0 = (int32_t)(q * p);
    uint32_t* __restrict__ out = stream + sched_group_base(beg, q, nw);
    SchedClass* __restrict__ h = hdr + q * nw * kMaxRun;

    // window w = the entries whose column is in [w*window_cols, (w+1)*window_cols); the last window takes the rest
    if (wv < 2) {
        // first entry of the group whose column is >= lim: the probes of a step split [lo, hi) into 64 parts
        const int64_t lim = (int64_t)(w + wv) * window_cols;
        int32_t lo = beg, hi = end;
        while (lo < hi) {
            const int32_t stride = (hi - lo + 63) / 64;
            const int32_t at = lo + lane * stride;
            const bool less = at < hi && (int64_t)cols[at] < lim;
            const int below = __popcll(__ballot(less));          // the columns ascend: the probes that are less come first
            if (below == 0) {
                hi = lo;
            } else {
                const int32_t up = lo + below * stride;
                lo = lo + (below - 1) * stride + 1;
                hi = up < hi ? up : hi;
            }
        }
        if (lane == 0) wstart[wv] = (w + wv == nw) ? end : lo;
    }
    if (tid < kMaxRun) { cnt[tid] = 0; base[tid] = 0; demote[tid] = 0; }
    __syncthreads();

    const uint64_t lt = (1ull << lane) - 1ull;
    {
        const int32_t wb = wstart[0], we = wstart[1];
        const bool staged = we - wb <= kStage;
        if (staged) {
            for (int32_t e = wb + tid; e < we; e += kBuildThreads) stage[e - wb] = cols[e];
            __syncthreads();
        }
        auto col_at = [&](int32_t e) -> int32_t { return staged ? stage[e - wb] : cols[e]; };

        // Length of the natural piece (run cut every kMaxRun entries) that entry e belongs to,
        // and e's place in it.  A run has one column, so it lies inside one window.
        auto natural_piece = [&](int32_t e, int& pos) -> int {
            const int32_t c = col_at(e);
            int32_t rs = e;                               // first entry of the run
            while (rs > wb && col_at(rs - 1) == c) --rs;
            pos = (e - rs) % kMaxRun;
            const int32_t ps = e - pos;                   // first entry of the piece
            int len = pos + 1;
            while (len < kMaxRun && ps + len < we && col_at(ps + len) == c) ++len;
            return len;
        };

        // The same for a staged window, without a chain of dependent reads per entry: the entries of a wave
        // (64 in a row) mark where a run starts, a ballot gives every lane the start and the end of its run inside
        // the wave, lane 0 alone walks back to the start of a run that began before the wave, and eight lanes look
        // at the eight entries behind the wave (a piece ends at most seven entries after one of its entries).
        // ew = the wave's first entry.  Every lane of the wave must call it.
        auto staged_piece = [&](int32_t e, int32_t ew, int& pos) -> int {
            const bool valid = e < we;
            const int32_t c = valid ? stage[e - wb] : 0;
            const bool start = !valid || e == wb || stage[e - 1 - wb] != c;
            const uint64_t b1 = __ballot(start);
            const int32_t e2 = ew + 64 + lane;
            const bool start2 = lane < 8 && (e2 >= we || stage[e2 - wb] != stage[e2 - 1 - wb]);
            const uint64_t b2 = __ballot(start2);
            int32_t carry = 0;                           // entries of the wave's first run in front of the wave
            if ((b1 & 1ull) == 0) {                      // (then ew < we and ew > wb)
                if (lane == 0) {
                    while (ew - 1 - carry >= wb && stage[ew - 1 - carry - wb] == c) ++carry;
                }
                carry = __shfl(carry, 0, 64);
            }
            const uint64_t upto = b1 & (lane == 63 ? ~0ull : ((2ull << lane) - 1ull));
            const int32_t d = upto ? lane - (63 - __clzll(upto)) : lane + carry;      // entries of the run in front of e
            pos = d % kMaxRun;
            const uint64_t after = lane == 63 ? 0ull : (b1 & ~((2ull << lane) - 1ull));
            const int32_t run_end = after ? __ffsll((long long)after) - 1 : (b2 ? 64 + __ffsll((long long)b2) - 1 : 72);
            const int32_t len = run_end - (lane - pos);
            return len < kMaxRun ? len : kMaxRun;
        };

        if (staged) {
            for (int32_t t0 = wb; t0 < we; t0 += kBuildThreads) {
                const int32_t e = t0 + tid;
                int pos;
                const int L = staged_piece(e, t0 + wv * 64, pos);
                if (e < we) {
                    piece_s[e - wb] = (uint8_t)(pos | ((L - 1) << 3));
                    if (pos == 0) atomicAdd(&cnt[L - 1], 1);      // a count: the order of the adds is irrelevant
                }
            }
        } else {
            for (int32_t e = wb + tid; e < we; e += kBuildThreads) {
                int pos;
                const int L = natural_piece(e, pos);
                if (pos == 0) atomicAdd(&cnt[L - 1], 1);
            }
        }
        __syncthreads();
        if (tid == 0) {
            for (int L = 2; L <= kMaxRun; ++L)
                if (cnt[L - 1] > 0 && cnt[L - 1] * L < kMinClassEntries) {
                    demote[L - 1] = 1;
                    cnt[0] += cnt[L - 1] * L;
                    cnt[L - 1] = 0;
                }
            int32_t at = 3 * (wb - beg) + kSchedPad * w;
            for (int L = 1; L <= kMaxRun; ++L) {
                const int per_body = kBody * runs_per_chunk(L);
                const int32_t bodies = (cnt[L - 1] + per_body - 1) / per_body;
                seg[L - 1] = at;
                h[w * kMaxRun + (L - 1)] = SchedClass{at, bodies};
                if (bodies > 0) at += pre_dwords(L) + bodies * block_dwords(L);
            }
        }
        __syncthreads();

        for (int32_t t0 = wb; t0 < we; t0 += kBuildThreads) {
            const int32_t e = t0 + tid;
            int L = 0;                                    // class of the piece that starts at e (0: none)
            if (e < we) {
                int pos, nat;
                if (staged) {
                    const int pl = piece_s[e - wb];
                    pos = pl & 7;
                    nat = (pl >> 3) + 1;
                } else {
                    nat = natural_piece(e, pos);
                }
                if (demote[nat - 1]) L = 1;
                else if (pos == 0) L = nat;
            }
            int32_t before = 0;
#pragma unroll
            for (int c = 1; c <= kMaxRun; ++c) {
                const uint64_t mk = __ballot(L == c);
                if (L == c) before = __popcll(mk & lt);
                if (lane == 0) wcnt[wv][c - 1] = __popcll(mk);
            }
            __syncthreads();
            if (L) {
                int32_t rank = base[L - 1] + before;
                for (int x = 0; x < wv; ++x) rank += wcnt[x][L - 1];
                const int J = runs_per_chunk(L);
                sched_put_piece(out + seg[L - 1], L, rank / J, rank % J, (uint32_t)col_at(e), rows, values, e, row0, p);
            }
            __syncthreads();
            if (tid < kMaxRun) {
                int32_t add = 0;
                for (int x = 0; x < kBuildWaves; ++x) add += wcnt[x][tid];
                base[tid] += add;
            }
            __syncthreads();
        }

        // dummy pieces up to whole bodies, and a valid column in every column slot that belongs
        // to no chunk (slot 0 of the pre-block, the three chunks after the last one)
        if (tid < kMaxRun && cnt[tid] > 0) {
            const int L = tid + 1, J = runs_per_chunk(L), per_body = kBody * J;
            const int32_t padded = (cnt[tid] + per_body - 1) / per_body * per_body;
            const uint32_t any_col = (uint32_t)col_at(wb);
            uint32_t* sg = out + seg[tid];
            for (int32_t r = cnt[tid]; r < padded; ++r) sched_put_piece(sg, L, r / J, r % J, any_col, nullptr, nullptr, 0, row0, p);
            const int32_t nch = padded / J;
            for (int j = 0; j < J; ++j) {
                sg[j] = any_col;
                for (int32_t x = nch; x < nch + 3; ++x) sg[sched_col_word(L, x, j)] = any_col;
            }
        }
    }
}

}  // namespace gcoo
