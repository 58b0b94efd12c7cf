// SpDM kernel in which the waves of a workgroup share the rows of B through LDS.
//
// Work unit = (super-group Q of W groups, column tile of 256 columns): wave w computes group
// W*Q + w exactly as the register kernel does (partial sums of p x 4 columns per lane in VGPRs, row
// selected through the VGPR index mode), but the B row segment of a run comes from LDS.  The
// workgroup walks the bands of the band schedule (gcoo_band.hpp): while band b is multiplied,
// every wave fetches its rows of band b+1 and the first block of its own stream for that band
// from global memory into the other LDS buffer, and one barrier per band separates the two uses
// of a buffer.  A row of B that several of the W groups need is fetched once per workgroup
// instead of once per group (Algorithm 2 shares B only through the caches; Section 3.3 counts
// these fetches as the cost to reduce).
//
// Two instances.  W = 8 (groups of up to 32 rows): the partial sums fill v[124:255], a wave has all
// 256 VGPRs and two waves share a SIMD; rows and blocks pass through registers on their way to
// LDS.  W = 16 (groups of up to 16 rows): the partial sums fill v[60:127], a wave has 128 VGPRs and
// four waves share a SIMD, which hides twice as much of every wave's instruction and LDS latency;
// with so few registers the rows and blocks go from global memory straight to LDS (the
// global_load ... lds form: M0 holds the LDS address of lane 0, every lane adds 16 bytes).
//
// All loads are plain C++ or compiler builtins and the compiler places the waits, with one
// exception that is stated where it happens: the arrival of the straight-to-LDS loads is awaited
// explicitly (s_waitcnt vmcnt(0)) before the barrier or the read that makes them visible.  The
// ring and band reads are volatile so that they stay behind the barriers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gcoo_band.hpp"
#include "gcoo_spdm_kernels.hpp"

namespace gcoo {

constexpr int kBandBufBytes = kBandRows * 1024;                 // one band: 64 rows x 256 columns x 4 bytes
constexpr int kBandRingSlots = 3;                               // first block of this band, of the next band, a further block of this band
// both shapes: 2 bands + W rings of 3 blocks = 128 KB + 24 KB
constexpr int kBandLdsBytes = 2 * kBandBufBytes + 8 * kBandRingSlots * 256 * 4;
static_assert(16 * kBandRingSlots * band_block_max(16) * 4 == 8 * kBandRingSlots * band_block_max(8) * 4, "");

typedef __attribute__((address_space(3))) f32x4 lds_f32x4;

// ---------------------------------------------------------------------------------------------
// The small accumulator file of the W = 16 instance: (16+1) x 4 partial sums in v[60:127],
//     sum(v, r) = v[60 + 17*v + r],
// used exactly like AccFile (gcoo_spdm_kernels.hpp).
// ---------------------------------------------------------------------------------------------
struct AccFile16 {
    f32x4 t0;                 // v[60:63]
    f32x32 t1, t2;            // v[64:95] v[96:127]
};
#define GCOO16_ACC_OPERANDS(acc) "+{v[60:63]}"((acc).t0), "+{v[64:95]}"((acc).t1), "+{v[96:127]}"((acc).t2)
#define GCOO16_FMA(i)                                  \
    "v_fma_f32 v60, %[a" #i "], %[b0], v60\n\t"         \
    "v_fma_f32 v77, %[a" #i "], %[b1], v77\n\t"         \
    "v_fma_f32 v94, %[a" #i "], %[b2], v94\n\t"         \
    "v_fma_f32 v111, %[a" #i "], %[b3], v111\n\t"
#define GCOO16_RUN_ASM(L) \
    asm volatile(GCOO_RUN##L(GCOO16_FMA) GCOO_OFF : GCOO16_ACC_OPERANDS(acc) : GCOO_E##L(c, a), GCOO_B_V4(b) : "m0")

// Four entries of four different columns (a chunk of type 1) in one span of the index mode.
#define GCOO16_FMA_E(i)                                      \
    "v_fma_f32 v60, %[a" #i "], %[b" #i "0], v60\n\t"         \
    "v_fma_f32 v77, %[a" #i "], %[b" #i "1], v77\n\t"         \
    "v_fma_f32 v94, %[a" #i "], %[b" #i "2], v94\n\t"         \
    "v_fma_f32 v111, %[a" #i "], %[b" #i "3], v111\n\t"
#define GCOO16_B_E(i, b) [b##i##0] "v"((b)[i][0]), [b##i##1] "v"((b)[i][1]), [b##i##2] "v"((b)[i][2]), [b##i##3] "v"((b)[i][3])
// The four entries of a chunk of type 1.
__device__ __forceinline__ void singles4_fma16(AccFile16& acc, const uint32_t (&c)[4], const float (&a)[4], const float (&b)[4][4])
{
    asm volatile("s_set_gpr_idx_on %[c0], gpr_idx(SRC2,DST)\n\t" GCOO16_FMA_E(0) "s_set_gpr_idx_idx %[c1]\n\t" GCOO16_FMA_E(1)
                 "s_set_gpr_idx_idx %[c2]\n\t" GCOO16_FMA_E(2) "s_set_gpr_idx_idx %[c3]\n\t" GCOO16_FMA_E(3) GCOO_OFF
                 : GCOO16_ACC_OPERANDS(acc)
                 : GCOO_E4(c, a), GCOO16_B_E(0, b), GCOO16_B_E(1, b), GCOO16_B_E(2, b), GCOO16_B_E(3, b)
                 : "m0");
}

template <int L>
__device__ __forceinline__ void run_fma16(AccFile16& acc, const uint32_t* c, const float* a, const float (&b)[4])
{
    static_assert(L == 1 || L == 2 || L == 4 || L == 8, "");
    if constexpr (L == 1) { GCOO16_RUN_ASM(1); }
    else if constexpr (L == 2) { GCOO16_RUN_ASM(2); }
    else if constexpr (L == 4) { GCOO16_RUN_ASM(4); }
    else { GCOO16_RUN_ASM(8); }
}

// What differs between the two instances.
struct BandShape8 {
    static constexpr int W = 8, R = 8, kBlock = band_block_max(8), kStride = 33, kFirst = kAccFirst, kDirect = 0;
    typedef AccFile Acc;
    static __device__ __forceinline__ void clear(Acc& a) { a.t0 = 0.0f; a.t1 = 0.0f; a.t2 = 0.0f; a.t3 = 0.0f; a.t4 = 0.0f; }
    template <int L>
    static __device__ __forceinline__ void fma(Acc& a, const uint32_t* c, const float* v, const float (&b)[4]) { run_fma<L, 4>(a, c, v, b); }
    static __device__ __forceinline__ float get(const Acc& a, int reg) { return acc_get(a, reg); }
};
struct BandShape16 {
    static constexpr int W = 16, R = 4, kBlock = band_block_max(16), kStride = 17, kFirst = 60, kDirect = 1;
    typedef AccFile16 Acc;
    static __device__ __forceinline__ void clear(Acc& a) { a.t0 = 0.0f; a.t1 = 0.0f; a.t2 = 0.0f; }
    template <int L>
    static __device__ __forceinline__ void fma(Acc& a, const uint32_t* c, const float* v, const float (&b)[4]) { run_fma16<L>(a, c, v, b); }
    static __device__ __forceinline__ float get(const Acc& a, int reg)
    {
        const int s = reg - kFirst;
        if (s < 4) return a.t0[s];
        return s < 36 ? a.t1[s - 4] : a.t2[s - 36];
    }
};

__device__ __forceinline__ u32x4 ring_read4(const lds_u32* p)
{
    return *(const volatile lds_u32x4*)p;
}
__device__ __forceinline__ uint32_t uni(uint32_t x) { return __builtin_amdgcn_readfirstlane(x); }

// 16 bytes per lane from global memory straight to LDS: lane i's bytes land at lds0 + 16*i (lds0 is
// the same in every lane).  Completion is counted by vmcnt like any vector load.
__device__ __forceinline__ void load_to_lds16(const void* src_lane, const lds_u32* lds0)
{
    __builtin_amdgcn_global_load_lds((__attribute__((address_space(1))) const void*)src_lane,
                                     (__attribute__((address_space(3))) void*)lds0, 16, 0, 0);
}
// s_waitcnt vmcnt(0), the other counters left alone: every vector load of this wave has arrived,
// those that write LDS included.
__device__ __forceinline__ void wait_vector_loads() { __builtin_amdgcn_s_waitcnt(0x0f70); }

// The B segment of a run: this lane's four columns of the row at byte offset `off` of the band.
__device__ __forceinline__ void band_b(const char __attribute__((address_space(3)))* band_lane, uint32_t off, float (&b)[4])
{
    const f32x4 t = *(const volatile lds_f32x4*)(band_lane + off);
    b[0] = t.x; b[1] = t.y; b[2] = t.z; b[3] = t.w;
}

// The words of one chunk of type T, as read from the ring.
template <int T>
struct BandChunk {
    static constexpr int kReads = band_chunk_words(T) / 4;
    u32x4 w[kReads];
};

template <int T>
__device__ __forceinline__ BandChunk<T> band_chunk_read(const lds_u32* cp)
{
    BandChunk<T> c;
#pragma unroll
    for (int i = 0; i < BandChunk<T>::kReads; ++i) c.w[i] = ring_read4(cp + 4 * i);
    return c;
}

// Byte offset inside the band of the B row of piece j.
template <int T>
__device__ __forceinline__ uint32_t band_chunk_offset(const BandChunk<T>& c, int j)
{
    const uint32_t word = (j < 2) ? c.w[0].x : c.w[0].y;
    return (j & 1) ? word >> 16 : word & 0xffffu;
}

// Piece j of the chunk times its B segment: rows to SGPRs, values stay in VGPRs.
template <int T, class S>
__device__ __forceinline__ void band_chunk_fma(typename S::Acc& acc, const BandChunk<T>& c, int j, const uint32_t (&rowword)[2],
                                               const float (&b)[4])
{
    // row bytes of piece j start at byte j*T of the row words; values at word 4 + j*T
    uint32_t r[T];
    float a[T];
#pragma unroll
    for (int u = 0; u < T; ++u) {
        const int byte = j * T + u;
        r[u] = rowword[byte / 4] >> (8 * (byte % 4));
        const int vw = 4 + j * T + u;
        const u32x4 q = c.w[vw / 4];
        const uint32_t bits = (vw % 4 == 0) ? q.x : (vw % 4 == 1) ? q.y : (vw % 4 == 2) ? q.z : q.w;
        a[u] = __uint_as_float(bits);
    }
    S::template fma<T>(acc, r, a, b);
}

// All n chunks of type T that start at cp.  Software pipeline: the ring words of a chunk are read
// two chunks ahead (one chunk ahead where registers are scarce); the B segment of piece j of the
// next chunk is read from the band as soon as piece j of this chunk has been multiplied (into the
// registers that piece just freed), so those reads are in flight behind the multiply-adds of the
// other pieces.
// rem (type 1 only): piece slots in use in the last chunk, 0 = all four.  The sixteen-wave
// instance multiplies only those; the eight-wave instance multiplies the unused slots too (they
// add zero to the sink row).
template <int T, class S>
__device__ __forceinline__ const lds_u32* band_chunks(typename S::Acc& acc, const lds_u32* cp, int32_t n,
                                                       const char __attribute__((address_space(3)))* band_lane, uint32_t rem = 0)
{
    constexpr int J = band_pieces_per_chunk(T), W = band_chunk_words(T);
    if (n <= 0) return cp;
    float b[J][4];
    auto multiply = [&](const BandChunk<T>& c0, const BandChunk<T>& c1) {
        // the row words sit behind the offset words: T = 1, 2: words 2, 3; T = 4, 8: words 1, 2
        const uint32_t rowword[2] = {uni(T <= 2 ? c0.w[0].z : c0.w[0].y), uni(T <= 2 ? c0.w[0].w : c0.w[0].z)};
#pragma unroll
        for (int j = 0; j < J; ++j) {
            band_chunk_fma<T, S>(acc, c0, j, rowword, b[j]);
            band_b(band_lane, band_chunk_offset<T>(c1, j), b[j]);  // piece j of the next chunk (of this one again after the last)
        }
    };
    if constexpr (S::kDirect) {
        // No software pipeline here: with four waves per SIMD the other waves cover a chunk's two
        // LDS round trips, and the fewest instructions win (measured: 4-5 % over the pipelined loop).
        const int32_t full = (T == 1 && rem) ? n - 1 : n;         // chunks that are multiplied whole
        for (int32_t c = 0; c < full; ++c) {
            const BandChunk<T> w = band_chunk_read<T>(cp);
#pragma unroll
            for (int j = 0; j < J; ++j) band_b(band_lane, band_chunk_offset<T>(w, j), b[j]);
            if constexpr (T == 1) {
                const uint32_t rw = uni(w.w[0].z);
                const uint32_t r[4] = {rw, rw >> 8, rw >> 16, rw >> 24};
                const float a[4] = {__uint_as_float(w.w[1].x), __uint_as_float(w.w[1].y), __uint_as_float(w.w[1].z),
                                    __uint_as_float(w.w[1].w)};
                singles4_fma16(acc, r, a, b);
            } else {
                const uint32_t rowword[2] = {uni(T <= 2 ? w.w[0].z : w.w[0].y), uni(T <= 2 ? w.w[0].w : w.w[0].z)};
#pragma unroll
                for (int j = 0; j < J; ++j) band_chunk_fma<T, S>(acc, w, j, rowword, b[j]);
            }
            cp += W;
        }
        if constexpr (T == 1) {
            if (rem) {                                            // the last chunk: only the slots in use
                const BandChunk<T> w = band_chunk_read<T>(cp);
#pragma unroll
                for (int j = 0; j < 3; ++j) band_b(band_lane, band_chunk_offset<T>(w, j), b[j]);   // an unused slot names offset 0
                const uint32_t rw = uni(w.w[0].z);
                const uint32_t r[4] = {rw, rw >> 8, rw >> 16, rw >> 24};
                const float a[4] = {__uint_as_float(w.w[1].x), __uint_as_float(w.w[1].y), __uint_as_float(w.w[1].z),
                                    __uint_as_float(w.w[1].w)};
                run_fma16<1>(acc, &r[0], &a[0], b[0]);
                if (rem >= 2) run_fma16<1>(acc, &r[1], &a[1], b[1]);
                if (rem >= 3) run_fma16<1>(acc, &r[2], &a[2], b[2]);
                cp += W;
            }
        }
    } else {
        // three register sets take turns (this chunk, the next, the one being read), so that no
        // words are copied from set to set: the loop body is written out three times
        BandChunk<T> s0 = band_chunk_read<T>(cp);
        BandChunk<T> s1 = band_chunk_read<T>(cp + (n > 1 ? W : 0));
        BandChunk<T> s2 = s1;
#pragma unroll
        for (int j = 0; j < J; ++j) band_b(band_lane, band_chunk_offset<T>(s0, j), b[j]);
        auto turn = [&](const BandChunk<T>& c0, const BandChunk<T>& c1, BandChunk<T>& c2, int32_t c) {
            const int32_t ahead = c + 2 < n ? 2 : n - 1 - c;      // the last chunks are read again instead of reading past the end
            c2 = band_chunk_read<T>(cp + ahead * W);
            multiply(c0, c1);
            cp += W;
        };
        for (int32_t c = 0; c < n; c += 3) {
            turn(s0, s1, s2, c);
            if (c + 1 < n) turn(s1, s2, s0, c + 1);
            if (c + 2 < n) turn(s2, s0, s1, c + 2);
        }
    }
    return cp;
}

// All chunks of one block (in the ring at `blk`) against the band whose LDS address, plus this
// lane's place in a row, is band_lane.
template <class S>
__device__ __forceinline__ void band_block(typename S::Acc& acc, const lds_u32* blk, const char __attribute__((address_space(3)))* band_lane,
                                           uint32_t counts, uint32_t flags)
{
    const lds_u32* cp = blk + kBandHdr;
    cp = band_chunks<1, S>(acc, cp, (int32_t)(counts & 255u), band_lane, (flags >> 1) & 3u);
    if (S::kDirect && (counts >> 8) == 0) return;                 // nothing but single entries: the usual block of a very sparse matrix
    cp = band_chunks<2, S>(acc, cp, (int32_t)((counts >> 8) & 255u), band_lane);
    cp = band_chunks<4, S>(acc, cp, (int32_t)((counts >> 16) & 255u), band_lane);
    band_chunks<8, S>(acc, cp, (int32_t)(counts >> 24), band_lane);
}

template <class S>
__global__ __launch_bounds__(64 * S::W) void spdm_band(const uint32_t* __restrict__ stream, const int32_t* __restrict__ gIdxes,
                                                      const int32_t* __restrict__ ucount, int64_t m, int32_t p, int64_t g, int64_t k,
                                                      int64_t nq, const float* __restrict__ B, int64_t ldb, int64_t N,
                                                      float* __restrict__ C, int64_t ldc, int64_t total)
{
    constexpr int W = S::W, R = S::R, kBlock = S::kBlock;
    extern __shared__ __attribute__((aligned(16))) uint32_t band_smem[];
    // XCD-aware order as in spdm_sched: XCD x walks the contiguous slice [x*per, (x+1)*per) of the
    // tile-major list, so the super-groups that run on it together read the same tile of B.
    const uint32_t bid = blockIdx.x;
    const uint32_t per = gridDim.x >> 3;
    const int64_t item = (int64_t)(bid & 7u) * per + (bid >> 3);
    if (item >= total) return;                                   // the whole workgroup
    const int64_t tile = item / nq, Q = item - tile * nq;

    const int lane = threadIdx.x & 63;
    const int wv = (int)uni(threadIdx.x >> 6);
    const int64_t q = Q * W + wv;
    const int64_t j0 = tile * 256 + (int64_t)lane * 4;
    const bool in = j0 < N;
    // Row bases are wave-uniform (SGPRs); the lane's place inside the tile is a 32-bit byte
    // offset.  Lanes beyond N read the first columns of the tile instead (always inside B).
    const char* Bbytes = reinterpret_cast<const char*>(B + tile * 256);
    const uint32_t lane_off = in ? (uint32_t)lane * 16u : 0u;
    const uint32_t ldb4 = (uint32_t)ldb * 4u;                     // the launcher checks that ldb*4 fits 32 bits
    const int32_t nb = (int32_t)((uni((uint32_t)ucount[Q]) + kBandRows - 1) / kBandRows);
    const uint32_t* st = stream + band_stream_base((int32_t)uni((uint32_t)gIdxes[q < g ? q : g]), q, k);

    const lds_u32* lds = (const lds_u32*)band_smem;
    const char __attribute__((address_space(3)))* band0 = (const char __attribute__((address_space(3)))*)lds;
    const lds_u32* ring = lds + 2 * kBandBufBytes / 4 + wv * (kBandRingSlots * kBlock);
    lds_u32x4* ring_w = (lds_u32x4*)ring;                         // this wave's ring, 16 bytes per lane
    lds_f32x4* band_w = (lds_f32x4*)band0;

    typename S::Acc acc;
    S::clear(acc);

    // kBlock words from `pos`: a block and what follows it
    auto fetch_block = [&](int64_t pos) -> u32x4 {
        return *reinterpret_cast<const u32x4*>(st + pos + lane * 4);
    };
    auto block_to_ring = [&](int64_t pos, int slot) {             // the same, straight to ring slot `slot`
        if (lane * 4 < kBlock) load_to_lds16(st + pos + lane * 4, ring + slot * kBlock);
    };
    // The header of a band's first block is also read one step ahead with scalar loads (the
    // address is the same for the whole wave), so that the step can start its fetches from
    // SGPRs at once instead of reading the ring and moving the words to SGPRs.
    struct Head { u32x4 a, b, c; };                               // words 0..3, 4..7, 8..11 of a block
    // (constant address space: the stream is read-only here, and that is what makes these scalar
    // loads also next to loads that write LDS, which the compiler takes for possible writers)
    typedef __attribute__((address_space(4))) const u32x4 const_u32x4;
    auto head_at = [&](int64_t pos) -> Head {
        const_u32x4* hp = (const_u32x4*)(st + pos);
        if constexpr (R > 4) return Head{hp[0], hp[1], hp[2]};
        else return Head{hp[0], hp[1], hp[1]};
    };
    // A wave always fetches its R rows of a band: where the band has fewer than 64 rows the
    // header names row 0 of B and the slot is never read.
    f32x4 pr[S::kDirect ? 1 : R];
    auto fetch_rows = [&](const Head& h, int buf) {               // this wave's rows of the band that the header announces
        const uint32_t id[8] = {h.b.x, h.b.y, h.b.z, h.b.w, h.c.x, h.c.y, h.c.z, h.c.w};
#pragma unroll
        for (int t = 0; t < R; ++t) {
            const char* src = Bbytes + (uint64_t)id[t] * ldb4 + lane_off;
            if constexpr (S::kDirect) load_to_lds16(src, lds + buf * (kBandBufBytes / 4) + (t * W + wv) * 256);
            else pr[t] = *reinterpret_cast<const f32x4*>(src);
        }
    };
    auto store_rows = [&](int buf) {
        if constexpr (!S::kDirect) {
#pragma unroll
            for (int t = 0; t < R; ++t) band_w[buf * (kBandBufBytes / 16) + (t * W + wv) * 64 + lane] = pr[t];
        }
    };

    // start: the pre-block says what to fetch for band 0
    int64_t pos;
    Head hd;
    {
        const Head pre = head_at(0);
        pos = (int64_t)pre.a.z;
        fetch_rows(pre, 0);
        if constexpr (S::kDirect) {
            block_to_ring(pos, 1);
            hd = head_at(pos);
            wait_vector_loads();
        } else {
            const u32x4 first = fetch_block(pos);
            hd = head_at(pos);
            store_rows(0);
            ring_w[1 * (kBlock / 4) + lane] = first;
        }
    }
    __syncthreads();

    for (int32_t b = 0; b < nb; ++b) {
        // band b+1: rows, first block and its header on their way while band b is multiplied (after
        // the last band the header names row 0 and the reads stay inside the stream's slack)
        const int64_t next_pos = pos + (int64_t)hd.a.z;
        const Head hn = head_at(next_pos);
        fetch_rows(hd, (b + 1) & 1);
        u32x4 next_block;
        if constexpr (S::kDirect) block_to_ring(next_pos, b & 1);
        else next_block = fetch_block(next_pos);

        const char __attribute__((address_space(3)))* band_lane = band0 + (b & 1) * kBandBufBytes + lane * 16;
        const lds_u32* blk = ring + ((b + 1) & 1) * kBlock;      // this band's first block
        band_block<S>(acc, blk, band_lane, hd.a.x, hd.a.y);
        if (!(hd.a.y & 1u)) {                                     // further blocks of this band: a group with many entries in it
            int64_t bpos = pos + (int64_t)hd.a.w;
            for (;;) {
                if constexpr (S::kDirect) {
                    __builtin_amdgcn_s_waitcnt(0xc07f);           // lgkmcnt(0): no read of the slot's last block is still on its way
                    block_to_ring(bpos, 2);
                    wait_vector_loads();                          // the block is in LDS before it is read
                } else {
                    ring_w[2 * (kBlock / 4) + lane] = fetch_block(bpos);
                }
                blk = ring + 2 * kBlock;
                const u32x4 h = ring_read4(blk);
                band_block<S>(acc, blk, band_lane, uni(h.x), uni(h.y));
                if (uni(h.y) & 1u) break;
                bpos += (int64_t)uni(h.w);
            }
        }

        if constexpr (S::kDirect) {
            wait_vector_loads();                                  // rows and block of band b+1 are in LDS before the barrier
        } else {
            store_rows((b + 1) & 1);
            ring_w[(b & 1) * (kBlock / 4) + lane] = next_block;
        }
        pos = next_pos;
        hd = hn;
        __syncthreads();
    }

    if (q < g && in) {
        constexpr int St = S::kStride;
        const int64_t row0 = q * p;
        float* __restrict__ Cl = C + j0;
#pragma unroll
        for (int r = 0; r < St - 1; ++r) {
            if (r < p && row0 + r < m) {
                f32x4 o = {S::get(acc, S::kFirst + r), S::get(acc, S::kFirst + St + r), S::get(acc, S::kFirst + 2 * St + r),
                           S::get(acc, S::kFirst + 3 * St + r)};
                __builtin_nontemporal_store(o, reinterpret_cast<f32x4*>(Cl + (row0 + r) * ldc));
            }
        }
    }
}

}  // namespace gcoo
