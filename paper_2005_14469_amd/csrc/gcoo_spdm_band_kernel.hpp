// SpDM kernel in which the eight waves of a workgroup share the rows of B through LDS.
//
// Work unit = (super-group Q of eight groups, column tile of 256 columns): wave w computes group
// 8Q + w exactly as the register kernel does (partial sums of p x 4 columns per lane in VGPRs, row
// selected through the VGPR index mode), but the B row segment of a run comes from LDS.  The
// workgroup walks the bands of the band schedule (gcoo_band.hpp): while band b is multiplied,
// every wave fetches its eight rows of band b+1 and the first block of its own stream for that
// band from global memory into registers, then stores them to the other LDS buffer, and one
// barrier per band separates the two uses of a buffer.  A row of B that several of the eight
// groups need is fetched once per workgroup instead of once per group (Algorithm 2 shares B only
// through the caches; Section 3.3 counts these fetches as the cost to reduce).
//
// Nothing here is issued behind the compiler's back: all loads are plain C++ and the compiler
// places the waits.  The ring and band reads are volatile so that they stay behind the barriers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gcoo_band.hpp"
#include "gcoo_spdm_kernels.hpp"

namespace gcoo {

constexpr int kBandBufBytes = kBandRows * 1024;                 // one band: 64 rows x 256 columns x 4 bytes
constexpr int kBandRingSlots = 3;                               // first block of this band, of the next band, a further block of this band
constexpr int kBandLdsBytes = 2 * kBandBufBytes + kBandWaves * kBandRingSlots * kBandBlockMax * 4;

typedef __attribute__((address_space(3))) f32x4 lds_f32x4;

__device__ __forceinline__ u32x4 ring_read4(const lds_u32* p)
{
    return *(const volatile lds_u32x4*)p;
}
__device__ __forceinline__ uint32_t uni(uint32_t x) { return __builtin_amdgcn_readfirstlane(x); }

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
template <int T>
__device__ __forceinline__ void band_chunk_fma(AccFile& acc, const BandChunk<T>& c, int j, const uint32_t (&rowword)[2],
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
    run_fma<T, 4>(acc, r, a, b);
}

// All n chunks of type T that start at cp.  Software pipeline: the ring words of a chunk are read
// two chunks ahead; the B segment of piece j of the next chunk is read from the band as soon as
// piece j of this chunk has been multiplied (into the registers that piece just freed), so those
// reads are in flight behind the multiply-adds of the other pieces.
template <int T>
__device__ __forceinline__ const lds_u32* band_chunks(AccFile& acc, const lds_u32* cp, int32_t n,
                                                       const char __attribute__((address_space(3)))* band_lane)
{
    constexpr int J = band_pieces_per_chunk(T), W = band_chunk_words(T);
    if (n <= 0) return cp;
    // three register sets take turns (this chunk, the next, the one being read), so that no
    // words are copied from set to set: the loop body is written out three times
    BandChunk<T> s0 = band_chunk_read<T>(cp);
    BandChunk<T> s1 = band_chunk_read<T>(cp + (n > 1 ? W : 0));
    BandChunk<T> s2 = s1;
    float b[J][4];
#pragma unroll
    for (int j = 0; j < J; ++j) band_b(band_lane, band_chunk_offset<T>(s0, j), b[j]);
    auto turn = [&](const BandChunk<T>& c0, const BandChunk<T>& c1, BandChunk<T>& c2, int32_t c) {
        const int32_t ahead = c + 2 < n ? 2 : n - 1 - c;          // the last chunks are read again instead of reading past the end
        c2 = band_chunk_read<T>(cp + ahead * W);
        // the row words sit behind the offset words: T = 1, 2: words 2, 3; T = 4, 8: words 1, 2
        const uint32_t rowword[2] = {uni(T <= 2 ? c0.w[0].z : c0.w[0].y), uni(T <= 2 ? c0.w[0].w : c0.w[0].z)};
#pragma unroll
        for (int j = 0; j < J; ++j) {
            band_chunk_fma<T>(acc, c0, j, rowword, b[j]);
            band_b(band_lane, band_chunk_offset<T>(c1, j), b[j]);  // piece j of the next chunk (of this one again after the last)
        }
        cp += W;
    };
    for (int32_t c = 0; c < n; c += 3) {
        turn(s0, s1, s2, c);
        if (c + 1 < n) turn(s1, s2, s0, c + 1);
        if (c + 2 < n) turn(s2, s0, s1, c + 2);
    }
    return cp;
}

// All chunks of one block (in the ring at `blk`) against the band whose LDS address, plus this
// lane's place in a row, is band_lane.
__device__ __forceinline__ void band_block(AccFile& acc, const lds_u32* blk, const char __attribute__((address_space(3)))* band_lane,
                                           uint32_t counts)
{
    const lds_u32* cp = blk + kBandHdr;
    cp = band_chunks<1>(acc, cp, (int32_t)(counts & 255u), band_lane);
    cp = band_chunks<2>(acc, cp, (int32_t)((counts >> 8) & 255u), band_lane);
    cp = band_chunks<4>(acc, cp, (int32_t)((counts >> 16) & 255u), band_lane);
    band_chunks<8>(acc, cp, (int32_t)(counts >> 24), band_lane);
}

__global__ __launch_bounds__(64 * kBandWaves) void spdm_band(const uint32_t* __restrict__ stream, const int32_t* __restrict__ gIdxes,
                                                            const int32_t* __restrict__ ucount, int64_t m, int32_t p, int64_t g,
                                                            int64_t k, int64_t nq, const float* __restrict__ B, int64_t ldb, int64_t N,
                                                            float* __restrict__ C, int64_t ldc, int64_t total)
{
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
    const int64_t q = Q * kBandWaves + wv;
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
    const lds_u32* ring = lds + 2 * kBandBufBytes / 4 + wv * (kBandRingSlots * kBandBlockMax);
    lds_u32x4* ring_w = (lds_u32x4*)ring;                         // this wave's ring, 16 bytes per lane and slot
    lds_f32x4* band_w = (lds_f32x4*)band0;

    AccFile acc;
    acc.t0 = 0.0f; acc.t1 = 0.0f; acc.t2 = 0.0f; acc.t3 = 0.0f; acc.t4 = 0.0f;

    auto fetch_block = [&](int64_t pos) -> u32x4 {                // 256 words from `pos`: a block and what follows it
        return *reinterpret_cast<const u32x4*>(st + pos + lane * 4);
    };
    // The header of a band's first block is also read one step ahead with scalar loads (the
    // address is the same for the whole wave), so that the step can start its fetches from
    // SGPRs at once instead of reading the ring and moving eleven words to SGPRs.
    struct Head { u32x4 a, b, c; };                               // words 0..3, 4..7, 8..11 of a block
    auto head_at = [&](int64_t pos) -> Head {
        const u32x4* hp = reinterpret_cast<const u32x4*>(st + pos);
        return Head{hp[0], hp[1], hp[2]};
    };
    // A wave always fetches and stores its eight rows of a band: where the band has fewer than 64
    // rows the header names row 0 of B and the slot is never read.
    f32x4 pr[8];
    auto fetch_rows = [&](const Head& h) {                        // this wave's rows of the band that the header announces
        const uint32_t id[8] = {h.b.x, h.b.y, h.b.z, h.b.w, h.c.x, h.c.y, h.c.z, h.c.w};
#pragma unroll
        for (int t = 0; t < 8; ++t) pr[t] = *reinterpret_cast<const f32x4*>(Bbytes + (uint64_t)id[t] * ldb4 + lane_off);
    };
    auto store_rows = [&](int buf) {
#pragma unroll
        for (int t = 0; t < 8; ++t) band_w[buf * (kBandBufBytes / 16) + (t * 8 + wv) * 64 + lane] = pr[t];
    };

    // start: the pre-block says what to fetch for band 0
    int64_t pos;
    Head hd;
    {
        const Head pre = head_at(0);
        pos = (int64_t)pre.a.z;
        fetch_rows(pre);
        const u32x4 first = fetch_block(pos);
        hd = head_at(pos);
        store_rows(0);
        ring_w[1 * 64 + lane] = first;
    }
    __syncthreads();

    for (int32_t b = 0; b < nb; ++b) {
        // band b+1: rows, first block and its header on their way while band b is multiplied (after
        // the last band the header names row 0 eight times and the reads stay inside the stream's slack)
        const int64_t next_pos = pos + (int64_t)hd.a.z;
        const Head hn = head_at(next_pos);
        fetch_rows(hd);
        const u32x4 next_block = fetch_block(next_pos);

        const char __attribute__((address_space(3)))* band_lane = band0 + (b & 1) * kBandBufBytes + lane * 16;
        const lds_u32* blk = ring + ((b + 1) & 1) * kBandBlockMax;   // this band's first block
        band_block(acc, blk, band_lane, hd.a.x);
        if (!(hd.a.y & 1u)) {                                     // further blocks of this band: a group with many entries in it
            int64_t bpos = pos + (int64_t)hd.a.w;
            for (;;) {
                ring_w[2 * 64 + lane] = fetch_block(bpos);
                blk = ring + 2 * kBandBlockMax;
                const u32x4 h = ring_read4(blk);
                band_block(acc, blk, band_lane, uni(h.x));
                if (uni(h.y) & 1u) break;
                bpos += (int64_t)uni(h.w);
            }
        }

        store_rows((b + 1) & 1);
        ring_w[(b & 1) * 64 + lane] = next_block;
        pos = next_pos;
        hd = hn;
        __syncthreads();
    }

    if (q < g && in) {
        constexpr int S = acc_stride<4>();
        const int64_t row0 = q * p;
        float* __restrict__ Cl = C + j0;
#pragma unroll
        for (int r = 0; r < S - 1; ++r) {
            if (r < p && row0 + r < m) {
                f32x4 o = {acc_get(acc, kAccFirst + r), acc_get(acc, kAccFirst + S + r), acc_get(acc, kAccFirst + 2 * S + r),
                           acc_get(acc, kAccFirst + 3 * S + r)};
                __builtin_nontemporal_store(o, reinterpret_cast<f32x4*>(Cl + (row0 + r) * ldc));
            }
        }
    }
}

}  // namespace gcoo
