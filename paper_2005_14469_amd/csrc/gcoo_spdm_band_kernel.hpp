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

// All chunks of one block (in the ring at `blk`) against the band whose LDS address, plus this
// lane's place in a row, is band_lane.
__device__ __forceinline__ void band_block(AccFile& acc, const lds_u32* blk, const char __attribute__((address_space(3)))* band_lane,
                                           uint32_t counts)
{
    const int32_t n1 = counts & 255u, n2 = (counts >> 8) & 255u, n4 = (counts >> 16) & 255u, n8 = counts >> 24;
    const lds_u32* cp = blk + kBandHdr;
    for (int32_t c = 0; c < n1; ++c, cp += 8) {
        const u32x4 h = ring_read4(cp), v = ring_read4(cp + 4);
        float b0[4], b1[4], b2[4], b3[4];
        band_b(band_lane, h.x & 0xffffu, b0);
        band_b(band_lane, h.x >> 16, b1);
        band_b(band_lane, h.y & 0xffffu, b2);
        band_b(band_lane, h.y >> 16, b3);
        const uint32_t rw = uni(h.z);
        const uint32_t r0 = rw, r1 = rw >> 8, r2 = rw >> 16, r3 = rw >> 24;
        const float a0 = __uint_as_float(v.x), a1 = __uint_as_float(v.y), a2 = __uint_as_float(v.z), a3 = __uint_as_float(v.w);
        run_fma<1, 4>(acc, &r0, &a0, b0);
        run_fma<1, 4>(acc, &r1, &a1, b1);
        run_fma<1, 4>(acc, &r2, &a2, b2);
        run_fma<1, 4>(acc, &r3, &a3, b3);
    }
    for (int32_t c = 0; c < n2; ++c, cp += 12) {
        const u32x4 h = ring_read4(cp), v0 = ring_read4(cp + 4), v1 = ring_read4(cp + 8);
        float b0[4], b1[4], b2[4], b3[4];
        band_b(band_lane, h.x & 0xffffu, b0);
        band_b(band_lane, h.x >> 16, b1);
        band_b(band_lane, h.y & 0xffffu, b2);
        band_b(band_lane, h.y >> 16, b3);
        const uint32_t ra = uni(h.z), rb = uni(h.w);
        const uint32_t r0[2] = {ra, ra >> 8}, r1[2] = {ra >> 16, ra >> 24}, r2[2] = {rb, rb >> 8}, r3[2] = {rb >> 16, rb >> 24};
        const float a0[2] = {__uint_as_float(v0.x), __uint_as_float(v0.y)}, a1[2] = {__uint_as_float(v0.z), __uint_as_float(v0.w)};
        const float a2[2] = {__uint_as_float(v1.x), __uint_as_float(v1.y)}, a3[2] = {__uint_as_float(v1.z), __uint_as_float(v1.w)};
        run_fma<2, 4>(acc, r0, a0, b0);
        run_fma<2, 4>(acc, r1, a1, b1);
        run_fma<2, 4>(acc, r2, a2, b2);
        run_fma<2, 4>(acc, r3, a3, b3);
    }
    for (int32_t c = 0; c < n4; ++c, cp += 12) {
        const u32x4 h = ring_read4(cp), v0 = ring_read4(cp + 4), v1 = ring_read4(cp + 8);
        float b0[4], b1[4];
        band_b(band_lane, h.x & 0xffffu, b0);
        band_b(band_lane, h.x >> 16, b1);
        const uint32_t ra = uni(h.y), rb = uni(h.z);
        const uint32_t r0[4] = {ra, ra >> 8, ra >> 16, ra >> 24}, r1[4] = {rb, rb >> 8, rb >> 16, rb >> 24};
        const float a0[4] = {__uint_as_float(v0.x), __uint_as_float(v0.y), __uint_as_float(v0.z), __uint_as_float(v0.w)};
        const float a1[4] = {__uint_as_float(v1.x), __uint_as_float(v1.y), __uint_as_float(v1.z), __uint_as_float(v1.w)};
        run_fma<4, 4>(acc, r0, a0, b0);
        run_fma<4, 4>(acc, r1, a1, b1);
    }
    for (int32_t c = 0; c < n8; ++c, cp += 12) {
        const u32x4 h = ring_read4(cp), v0 = ring_read4(cp + 4), v1 = ring_read4(cp + 8);
        float b0[4];
        band_b(band_lane, h.x & 0xffffu, b0);
        const uint32_t ra = uni(h.y), rb = uni(h.z);
        const uint32_t r0[8] = {ra, ra >> 8, ra >> 16, ra >> 24, rb, rb >> 8, rb >> 16, rb >> 24};
        const float a0[8] = {__uint_as_float(v0.x), __uint_as_float(v0.y), __uint_as_float(v0.z), __uint_as_float(v0.w),
                             __uint_as_float(v1.x), __uint_as_float(v1.y), __uint_as_float(v1.z), __uint_as_float(v1.w)};
        run_fma<8, 4>(acc, r0, a0, b0);
    }
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
    const float* Bl = B + tile * 256 + (in ? lane * 4 : 0);      // lanes beyond N re-read the first columns of the tile
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
    // A wave always fetches and stores its eight rows of a band: where the band has fewer than 64
    // rows the header names row 0 of B and the slot is never read.
    f32x4 pr[8];
    auto fetch_rows = [&](const lds_u32* hdr) {                   // this wave's rows of the band that the header announces
        const u32x4 ia = ring_read4(hdr + 4), ib = ring_read4(hdr + 8);
        const uint32_t id[8] = {uni(ia.x), uni(ia.y), uni(ia.z), uni(ia.w), uni(ib.x), uni(ib.y), uni(ib.z), uni(ib.w)};
#pragma unroll
        for (int t = 0; t < 8; ++t) pr[t] = *reinterpret_cast<const f32x4*>(Bl + (int64_t)id[t] * ldb);
    };
    auto store_rows = [&](int buf) {
#pragma unroll
        for (int t = 0; t < 8; ++t) band_w[buf * (kBandBufBytes / 16) + (t * 8 + wv) * 64 + lane] = pr[t];
    };

    // start: the pre-block says what to fetch for band 0
    int64_t pos = 0;
    {
        ring_w[0 * 64 + lane] = fetch_block(0);
        const u32x4 h = ring_read4(ring);
        pos = (int64_t)uni(h.z);
        fetch_rows(ring);
        const u32x4 first = fetch_block(pos);
        store_rows(0);
        ring_w[1 * 64 + lane] = first;
    }
    __syncthreads();

    for (int32_t b = 0; b < nb; ++b) {
        const lds_u32* blk = ring + ((b + 1) & 1) * kBandBlockMax;   // this band's first block
        const int64_t next_pos = pos + (int64_t)uni(ring_read4(blk).z);
        // band b+1: rows and first block on their way while band b is multiplied (after the last
        // band the header names row 0 eight times and the block read stays inside the stream's slack)
        fetch_rows(blk);
        const u32x4 next_block = fetch_block(next_pos);

        const char __attribute__((address_space(3)))* band_lane = band0 + (b & 1) * kBandBufBytes + lane * 16;
        int64_t bpos = pos;
        for (;;) {                                                // the blocks of this band: one, unless the group has many entries in it
            const u32x4 h = ring_read4(blk);
            band_block(acc, blk, band_lane, uni(h.x));
            if (uni(h.y) & 1u) break;
            bpos += (int64_t)uni(h.w);
            ring_w[2 * 64 + lane] = fetch_block(bpos);
            blk = ring + 2 * kBandBlockMax;
        }

        store_rows((b + 1) & 1);
        ring_w[(b & 1) * 64 + lane] = next_block;
        pos = next_pos;
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
