// SpDM kernel in which the eight waves of a workgroup share the rows of B through LDS
// (Algorithm 2 of the paper re-cut for CDNA4; the schedule it reads is described in gcoo_share.hpp).
//
// Work unit = (super-group Q of 8 groups, column tile of 256 columns).  Wave w owns group 8Q + w:
// every lane keeps (48 + 1) x 4 partial sums in v[60:255] (four adjacent columns of up to 48 rows,
// plus the sink row of the padding records).  The workgroup walks the bands of Q.  LDS holds three
// band buffers of 48 KB (48 rows of B x 256 columns): while band b is multiplied, band b+1 has
// landed or is landing and the rows of band b+2 are requested, by global->LDS loads (no registers
// in between), six rows per wave in three parts spread over the band.  One barrier per band; the
// wait in front of it lets the loads of band b+2 stay in flight, so the path from L2 to LDS never
// drains.
//
// Per entry the wave issues
//     v_add_u32_dpp   address = record.offset (broadcast inside each row of 16 lanes) + lane * 16
//     ds_read_b128    the lane's four columns of the B row, a group of four entries ahead of their use
//     s_set_gpr_idx_on + s_lshr_b32   the entry's row selects the partial sums (index mode); the rows
//                     of four entries travel in one scalar register
//     4 x v_fmac_f32_dpp   sum[row][c] += record.value (broadcast the same way) * b[c]
// and for a quad (four entries of one column) the first two only once.  The records are never
// moved to scalar registers one by one: a block of 16 records is read from LDS with one
// ds_read_b128 in which each row of 16 lanes receives the same 16 records, and the DPP
// row broadcast picks record i inside the instruction that uses it.  This is the staging of the
// entries in shared memory and their broadcast to all threads of Algorithm 2, and the reuse of
// the fetched B value along a run of equal columns (Section 3.3).
//
// What a wave needs of the schedule beside the records comes in vectors, ahead of its use: the
// columns of the six rows it fetches for a band, one load per band, two bands before the rows are
// requested (a DPP row broadcast picks the row); the (quads, singles) pairs of its bands, 64 bands
// per load (v_readlane picks the lane).
// The stream of blocks reaches LDS through a ring of eight blocks per wave, filled 1 KB at a time
// by global->LDS loads one piece ahead.
//
// The main loop is one asm statement: the index mode and the global->LDS loads both use M0, the
// reads from LDS are issued ahead of their use with counted waits, and a compiler-scheduled
// version of such a loop cannot be kept free of spills next to 196 pinned registers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gcoo_share.hpp"
#include "gcoo_spdm_launch.hpp"

namespace gcoo {

constexpr int kShareBandBytes = kShareBandRows * 1024;                       // one band: 48 rows x 256 columns x 4 bytes
constexpr int kShareRingBytes = kShareRingBlocks * kShareBlockWords * 4;     // per wave
constexpr int kShareLdsBytes = 3 * kShareBandBytes + kShareW * kShareRingBytes;
static_assert(kShareBandBytes == 0xC000 && kShareRingBytes == 0x800 && kShareBandRows == 6 * kShareW,
              "the asm text below uses these numbers");

typedef float sh_f32x32 __attribute__((ext_vector_type(32)));
typedef float sh_f32x4 __attribute__((ext_vector_type(4)));

// sum(c, r) = v[60 + 49 * c + r], c = 0..3, r = 0..48
struct ShareAcc {
    sh_f32x4 t0;                         // v[60:63]
    sh_f32x32 t1, t2, t3, t4, t5, t6;    // v[64:255]
};
constexpr int kShareAccFirst = 60;
constexpr int kShareAccStride = kShareMaxP + 1;
static_assert(kShareAccFirst + 4 * kShareAccStride == 256, "");

__device__ __forceinline__ float share_acc_get(const ShareAcc& a, int reg)
{
    const int s = reg - kShareAccFirst;
    if (s < 4) return a.t0[s];
    const int t = (s - 4) >> 5, i = (s - 4) & 31;
    return t == 0 ? a.t1[i] : t == 1 ? a.t2[i] : t == 2 ? a.t3[i] : t == 3 ? a.t4[i] : t == 4 ? a.t5[i] : a.t6[i];
}

// ---- asm text -----------------------------------------------------------------------------------
// Fixed registers of the main loop (named in the clobber list, but for the inputs, which are pinned to theirs):
//   v[20:35]  four sets of B values (sets 0..3)   v[4:19]  four more (sets 4..7: the singles of a band alternate between the two)
//   v[36:39]  four LDS addresses
//   inputs that stay as they are: v3 the place in ucols, inside a band, of the row whose offset the lane holds in v49;
//             v43 the shift that packs a record's row; v51 what that offset carries beside the row's place in B;
//             v53 the lane's place in the wave's ring; v58 lane*16 (0 for lanes beyond N); v59 lane*16
//   v40 v41 v42  values, packed rows (the four rows of a record's group of four, one byte each), offsets of this block
//   v[44:47]  records of the next block    v48 lane*16 + band buffer
//   v49  byte offsets of the rows to fetch for the band after next     v50 scratch     v52 columns of the band after that
//   v[54:55]  (quads, singles) of 64 bands  v[56:57] of the 64 bands after those
//   s64 band  s65 bands  s66 s67 quads and groups of four singles of this band (of the next one from the band's end on)
//   s68 blocks read from the ring x 0x100  s69 pieces of the stream requested  s82 of which known to have landed  s83 s69 at the start of the band
//   s70 s86 packed rows  s71 scratch  s72 where this wave's rows of the band after next go in LDS  s73 loop count
//   s[74:75] header pointer (next 64 bands)  s[76:77] stream pointer (next piece)  s[78:79] ucols of the super-group
//   s80 first place in ucols of the band whose columns are requested next
//   s88 LDS address of this band's buffer  s89 of the buffer that the next rows go to
#define SH_DPP(i) " row_newbcast:" #i " row_mask:0xf bank_mask:0xf\n\t"
#define SH_ADDR(dst, src, i) "v_add_u32_dpp " #dst ", " #src ", v48" SH_DPP(i)
#define SH_ROWS(reg, i) "v_readlane_b32 " #reg ", v41, " #i "\n\t"
// Timing ablations (GCOO_SHARE_ABLATE, a set of bits): the kernel with one of its parts taken out, to see what that
// part costs.  Such a build computes WRONG products; every address it forms is one the whole kernel forms too.
// Only the micro-benchmark builds them, into libraries of their own; libgcoo.so is always built with 0.
//   1 no row of B is requested (the bands in LDS hold whatever was there)      2 no multiply-adds, no index mode
//   4 no barrier between bands      8 the singles read no B values from LDS    16 the wait in front of the barrier
//   leaves the rows of two bands in flight instead of one
#ifndef GCOO_SHARE_ABLATE
#define GCOO_SHARE_ABLATE 0
#endif
#if GCOO_SHARE_ABLATE & 1
#define SH_FILL_LOAD(off) ""
#else
#define SH_FILL_LOAD(off) "global_load_lds_dwordx4 v50, %[bt] offset:" #off "\n\t"
#endif
#if GCOO_SHARE_ABLATE & 4
#define SH_BAND_BARRIER ""
#else
#define SH_BAND_BARRIER "s_barrier\n\t"
#endif
#if GCOO_SHARE_ABLATE & 8
#define SH_GROUP_READS(x) ""
#else
#define SH_GROUP_READS(x) x
#endif
#if GCOO_SHARE_ABLATE & 16
#define SH_WAIT_FILLS "s_waitcnt vmcnt(12)\n\t"
#else
#define SH_WAIT_FILLS "s_waitcnt vmcnt(6)\n\t"
#endif
// one entry: record i of this block, its row in the low byte of `rows`, its B values in b0..b3
// (SH_FMACL: the last entry of its group of four, after which the packed rows are not needed any more)
#if GCOO_SHARE_ABLATE & 2
#define SH_FMACL(i, rows, b0, b1, b2, b3) ""
#else
#define SH_FMACL(i, rows, b0, b1, b2, b3)                   \
    "s_set_gpr_idx_on " #rows ", gpr_idx(SRC2,DST)\n\t"      \
    "v_fmac_f32_dpp v60, v40, " #b0 SH_DPP(i)                \
    "v_fmac_f32_dpp v109, v40, " #b1 SH_DPP(i)               \
    "v_fmac_f32_dpp v158, v40, " #b2 SH_DPP(i)               \
    "v_fmac_f32_dpp v207, v40, " #b3 SH_DPP(i)
#endif
#define SH_FMAC(i, rows, b0, b1, b2, b3) SH_FMACL(i, rows, b0, b1, b2, b3) "s_lshr_b32 " #rows ", " #rows ", 8\n\t"
#define SH_FMAC_SET0(i, rows) SH_FMAC(i, rows, v20, v21, v22, v23)
#define SH_FMAC_SET1(i, rows) SH_FMAC(i, rows, v24, v25, v26, v27)
#define SH_FMAC_SET2(i, rows) SH_FMAC(i, rows, v28, v29, v30, v31)
#define SH_FMAC_SET3(i, rows) SH_FMAC(i, rows, v32, v33, v34, v35)
#define SH_FMAC_SET4(i, rows) SH_FMAC(i, rows, v4, v5, v6, v7)
#define SH_FMAC_SET5(i, rows) SH_FMAC(i, rows, v8, v9, v10, v11)
#define SH_FMAC_SET6(i, rows) SH_FMAC(i, rows, v12, v13, v14, v15)
#define SH_FMAC_SET7(i, rows) SH_FMAC(i, rows, v16, v17, v18, v19)
#define SH_FMACL_SET0(i, rows) SH_FMACL(i, rows, v20, v21, v22, v23)
#define SH_FMACL_SET1(i, rows) SH_FMACL(i, rows, v24, v25, v26, v27)
#define SH_FMACL_SET2(i, rows) SH_FMACL(i, rows, v28, v29, v30, v31)
#define SH_FMACL_SET3(i, rows) SH_FMACL(i, rows, v32, v33, v34, v35)
#define SH_FMACL_SET4(i, rows) SH_FMACL(i, rows, v4, v5, v6, v7)
#define SH_FMACL_SET5(i, rows) SH_FMACL(i, rows, v8, v9, v10, v11)
#define SH_FMACL_SET6(i, rows) SH_FMACL(i, rows, v12, v13, v14, v15)
#define SH_FMACL_SET7(i, rows) SH_FMACL(i, rows, v16, v17, v18, v19)
#define SH_READ_SET0 "ds_read_b128 v[20:23], v36\n\t"
#define SH_READ_SET1 "ds_read_b128 v[24:27], v37\n\t"
#define SH_READ_SET2 "ds_read_b128 v[28:31], v38\n\t"
#define SH_READ_SET3 "ds_read_b128 v[32:35], v39\n\t"
#define SH_READ_SET4 "ds_read_b128 v[4:7], v36\n\t"
#define SH_READ_SET5 "ds_read_b128 v[8:11], v37\n\t"
#define SH_READ_SET6 "ds_read_b128 v[12:15], v38\n\t"
#define SH_READ_SET7 "ds_read_b128 v[16:19], v39\n\t"
#define SH_WAIT3 "s_waitcnt lgkmcnt(3)\n\t"
#define SH_OFF "s_set_gpr_idx_off\n\t"

// The next block becomes this block (its four row bytes per group of four records are packed into one word
// on the way: a shift by the record's place in its group, then an OR across each quad of lanes); one more
// block is read from the ring (each row of 16 lanes reads the same 16 records).  Every fourth block the
// wave enters a new 1 KB piece of the stream: it has landed if it was requested before the band before
// this one began (s82), otherwise all loads are awaited here; and the piece after it is requested for the
// half of the ring whose blocks have all been read.
// Index mode must be off.  L = a number unique to the expansion (local labels).  s68 counts blocks in steps of
// 0x100, their size in bytes; the rare part (SH_ADVANCE_PIECE) stands out of line, behind the loop.
#define SH_ADVANCE(L)                                                                         \
    "v_lshlrev_b32 v41, v43, v45\n\t"                                                         \
    "v_mov_b32 v40, v44\n\t"                                                                  \
    "v_mov_b32 v42, v46\n\t"                                                                  \
    "v_or_b32_dpp v50, v41, v41 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"           \
    "s_add_u32 s68, s68, 0x100\n\t"                                                           \
    "s_and_b32 s71, s68, 0x300\n\t"                                                           \
    "v_or_b32_dpp v41, v50, v50 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"           \
    "s_cbranch_scc0 .Lsh_adv_piece" #L "_%=\n"                                                \
    ".Lsh_adv_read" #L "_%=:\n\t"                                                             \
    "s_and_b32 s71, s68, 0x700\n\t"                                                           \
    "v_add_u32 v50, s71, v53\n\t"                                                             \
    "ds_read_b128 v[44:47], v50\n\t"
#define SH_ADVANCE_PIECE(L)                                                                   \
    ".Lsh_adv_piece" #L "_%=:\n\t"                                                            \
    "s_lshr_b32 s71, s68, 10\n\t"                                                             \
    "s_cmp_lt_u32 s71, s82\n\t"                                                               \
    "s_cbranch_scc1 .Lsh_adv_req" #L "_%=\n\t"                                                \
    "s_waitcnt vmcnt(0)\n\t"                                                                  \
    "s_mov_b32 s82, s69\n"                                                                    \
    ".Lsh_adv_req" #L "_%=:\n\t"                                                              \
    "s_and_b32 s71, s68, 0x400\n\t"                                                           \
    "s_xor_b32 s71, s71, 0x400\n\t"                                                           \
    "s_add_u32 m0, s71, %[ring]\n\t"                                                          \
    "s_add_u32 s69, s69, 1\n\t"                                                               \
    "global_load_lds_dwordx4 v59, s[76:77]\n\t"                                               \
    "s_add_u32 s76, s76, 0x400\n\t"                                                           \
    "s_addc_u32 s77, s77, 0\n\t"                                                              \
    "s_branch .Lsh_adv_read" #L "_%=\n"

// The byte offsets in B of the six rows this wave fetches for a band sit in v49 at places 0..5 of every row of 16
// lanes (the other places repeat the sixth), so that a DPP row broadcast puts a row's offset in front of every
// lane's column offset in one instruction.  Every offset carries +3072 - 1024 * (t & 3), t = the row's place among
// the six, and the base pointer -3072: the loads of rows 0..3 and 4..5 then differ only in their immediate offsets,
// which also move the LDS address, and M0 is written once per part instead of once per row.
// The six rows of the band after next (band s64 + 2) go to the buffer at s89 in three parts, spread over the band
// (all eight waves asking for all their rows at once right behind the barrier holds every one of them up at the
// compute unit's one address path): HEAD at the band's start, which also makes the offsets from the columns in v52
// and requests the columns of the band after (s80 = its first place in ucols; places past the last column of the
// super-group repeat it), MID behind the first entries, TAIL at the band's end.
#define SH_FILL_ROW(r, off) "v_add_u32_dpp v50, v49, v58 row_newbcast:" #r " row_mask:0xf bank_mask:0xf\n\t" SH_FILL_LOAD(off)
#define SH_FILL_OFFSETS(cols)                                         \
    "v_mul_lo_u32 v49, " #cols ", %[ldb4]\n\t"                        \
    "s_add_u32 s72, s89, %[fillw]\n\t"                                \
    "v_add_u32 v49, v49, v51\n\t"
#define SH_FILL_HEAD                                                  \
    SH_FILL_OFFSETS(v52)                                              \
    "v_add_u32 v50, s80, v3\n\t"                                      \
    "v_min_u32 v50, v50, %[last]\n\t"                                 \
    "v_lshlrev_b32 v50, 2, v50\n\t"                                   \
    "global_load_dword v52, v50, s[78:79]\n\t"                        \
    "s_add_u32 s80, s80, 48\n\t"                                      \
    "s_mov_b32 m0, s72\n\t"                                           \
    SH_FILL_ROW(0, 0) SH_FILL_ROW(1, 1024)
#define SH_FILL_MID                                                   \
    "s_mov_b32 m0, s72\n\t"                                           \
    SH_FILL_ROW(2, 2048) SH_FILL_ROW(3, 3072)
#define SH_FILL_TAIL                                                  \
    "s_add_u32 m0, s72, 0x1000\n\t"                                   \
    SH_FILL_ROW(4, 0) SH_FILL_ROW(5, 1024)

__global__ __launch_bounds__(64 * kShareW) void spdm_share(ShareArgs a, int64_t total)
{
    extern __shared__ __attribute__((aligned(16))) uint32_t share_smem[];
    // XCD-aware order: XCD x walks the contiguous slice [x*per, (x+1)*per) of the tile-major list, so
    // the super-groups that run on it together read the same column tile of B.
    const uint32_t bid = blockIdx.x;
    const uint32_t per = gridDim.x >> 3;
    const int64_t item = (int64_t)(bid & 7u) * per + (bid >> 3);
    if (item >= total) return;                                   // the whole workgroup
    const int64_t tile = item / a.nq, Q = item - tile * a.nq;

    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t q = Q * kShareW + wv;
    const int64_t j0 = tile * 256 + (int64_t)lane * 4;
    const bool in = j0 < a.N;

    ShareAcc acc;
    acc.t0 = 0.0f; acc.t1 = 0.0f; acc.t2 = 0.0f; acc.t3 = 0.0f; acc.t4 = 0.0f; acc.t5 = 0.0f; acc.t6 = 0.0f;

    const int32_t nU = __builtin_amdgcn_readfirstlane(a.ucount[Q]);
    const int32_t nb = (nU + kShareBandRows - 1) / kShareBandRows;
    if (nb > 0) {
        const int64_t qn = (Q + 1) * kShareW;
        const int32_t first = __builtin_amdgcn_readfirstlane(a.gIdxes[Q * kShareW]);
        const int32_t first_next = __builtin_amdgcn_readfirstlane(a.gIdxes[qn < a.g ? qn : a.g]);
        const int64_t hb = share_hdr_base(first, Q), cap = share_hdr_base(first_next, Q + 1) - hb;
        const uint32_t* hdr = a.hdr + 2 * (hb * kShareW + wv * cap);
        const uint32_t* strm = a.blocks + (int64_t)__builtin_amdgcn_readfirstlane(a.sbase[q]) * kShareBlockWords;
        const int32_t* uc = a.ucols + first;
        const char* bt = reinterpret_cast<const char*>(a.B + tile * 256) - 3072;   // see SH_FILL_SIX
        const uint32_t ldb4 = (uint32_t)a.ldb * 4u;                // the launcher checks that every row offset fits 32 bits
        const uint32_t l16 = (uint32_t)lane * 16u;
        const uint32_t l16g = in ? l16 : 0u;                       // lanes beyond N fetch the first columns of the tile
        const uint32_t sh8 = (uint32_t)(lane & 3) * 8u;
        // place t of every row of 16 lanes (the places from the sixth on repeat it): row t of the wave's six in a band
        const int li = (lane & 15) < 6 ? (lane & 15) : 5;
        const uint32_t cidx = (uint32_t)(wv * 6 + li);
        const uint32_t fbias = 3072u - (uint32_t)(li & 3) * 1024u;
        const uint32_t ring = (uint32_t)(3 * kShareBandBytes + wv * kShareRingBytes);
        const uint32_t rl = ring + (uint32_t)(lane & 15) * 16u;
        const uint32_t fillw = (uint32_t)wv * 6144u;               // the wave's six rows inside a band buffer
        const uint32_t last = (uint32_t)(nU - 1);
        asm volatile(
            // ---- start-up: two pieces of the stream, the headers of 128 bands, the columns of 20 bands, the rows of bands 0 and 1
            "s_mov_b64 s[74:75], %[hdr]\n\t"
            "s_mov_b64 s[76:77], %[strm]\n\t"
            "s_mov_b64 s[78:79], %[uc]\n\t"
            "s_mov_b32 s64, 0\n\t"
            "s_mov_b32 s65, %[nb]\n\t"
            "s_mov_b32 s68, 0\n\t"
            "s_mov_b32 s69, 2\n\t"
            "s_mov_b32 s82, 2\n\t"
            "s_mov_b32 s88, 0\n\t"
            "s_mov_b32 s80, 3 * 48\n\t"
            "s_mov_b32 m0, %[ring]\n\t"
            "s_nop 0\n\t"
            "global_load_lds_dwordx4 v59, s[76:77]\n\t"
            "s_add_u32 s76, s76, 0x400\n\t"
            "s_addc_u32 s77, s77, 0\n\t"
            "s_add_u32 m0, %[ring], 0x400\n\t"
            "s_nop 0\n\t"
            "global_load_lds_dwordx4 v59, s[76:77]\n\t"
            "s_add_u32 s76, s76, 0x400\n\t"
            "s_addc_u32 s77, s77, 0\n\t"
            "v_lshrrev_b32 v50, 1, v59\n\t"
            "global_load_dwordx2 v[54:55], v50, s[74:75]\n\t"
            "global_load_dwordx2 v[56:57], v50, s[74:75] offset:512\n\t"
            "s_add_u32 s74, s74, 0x400\n\t"
            "s_addc_u32 s75, s75, 0\n\t"
            // the columns of bands 0, 1 and 2
            "v_min_u32 v50, v3, %[last]\n\t"
            "v_lshlrev_b32 v50, 2, v50\n\t"
            "global_load_dword v40, v50, s[78:79]\n\t"
            "v_add_u32 v50, 48, v3\n\t"
            "v_min_u32 v50, v50, %[last]\n\t"
            "v_lshlrev_b32 v50, 2, v50\n\t"
            "global_load_dword v42, v50, s[78:79]\n\t"
            "v_add_u32 v50, 96, v3\n\t"
            "v_min_u32 v50, v50, %[last]\n\t"
            "v_lshlrev_b32 v50, 2, v50\n\t"
            "global_load_dword v52, v50, s[78:79]\n\t"
            "s_waitcnt vmcnt(0)\n\t"
            "v_readlane_b32 s66, v54, 0\n\t"
            "v_readlane_b32 s67, v55, 0\n\t"
            "ds_read_b128 v[44:47], v53\n\t"
            // (bands beyond the last one are requested like any other: their columns are clamped to the last
            // column of the super-group, their rows go to a buffer that nobody reads)
            "s_mov_b32 s89, 0\n\t"
            SH_FILL_OFFSETS(v40)
            "s_mov_b32 m0, s72\n\t"
            SH_FILL_ROW(0, 0) SH_FILL_ROW(1, 1024) SH_FILL_ROW(2, 2048) SH_FILL_ROW(3, 3072)
            SH_FILL_TAIL
            "s_mov_b32 s89, 0x18000\n\t"
            SH_FILL_OFFSETS(v42)
            "s_mov_b32 m0, s72\n\t"
            SH_FILL_ROW(0, 0) SH_FILL_ROW(1, 1024) SH_FILL_ROW(2, 2048) SH_FILL_ROW(3, 3072)
            SH_FILL_TAIL
            "s_mov_b32 s89, 0xC000\n\t"
            "s_waitcnt vmcnt(6) lgkmcnt(0)\n\t"
            "s_barrier\n\t"
            SH_ADVANCE(0)
            // ---- one band
            ".Lsh_band_%=:\n\t"
            "v_add_u32 v48, s88, v59\n\t"
            "s_mov_b32 s83, s69\n\t"
            // One decision per band: quads first, singles only, or nothing for this wave.  In each case the first B
            // rows of the band's first part are read while the rows of the band after next are requested.
            "s_cmp_eq_u32 s66, 0\n\t"
            "s_cbranch_scc1 .Lsh_noq_%=\n\t"
            SH_ADDR(v36, v42, 0) SH_ADDR(v37, v42, 4) SH_ADDR(v38, v42, 8) SH_ADDR(v39, v42, 12)
            SH_READ_SET0 SH_READ_SET1 SH_READ_SET2 SH_READ_SET3
            SH_FILL_HEAD
            // ---- quads
            "s_mov_b32 s73, s66\n"
            ".Lsh_qblk_%=:\n\t"
            SH_ROWS(s70, 0)
            // quad 0; after it everything read from LDS so far has arrived, the records of the next block included
            "s_sub_u32 s73, s73, 1\n\t"
            "s_cbranch_scc1 .Lsh_qend_%=\n\t"
            SH_ROWS(s86, 4)
            SH_WAIT3
            SH_FMAC_SET0(0, s70) SH_FMAC_SET0(1, s70) SH_FMAC_SET0(2, s70) SH_FMACL_SET0(3, s70)
            SH_OFF
            "s_waitcnt lgkmcnt(0)\n\t"
            SH_ADDR(v36, v46, 0)
            SH_READ_SET0
            // quad 1
            "s_sub_u32 s73, s73, 1\n\t"
            "s_cbranch_scc1 .Lsh_qend_%=\n\t"
            SH_ROWS(s70, 8)
            SH_ADDR(v37, v46, 4)
            "s_waitcnt lgkmcnt(1)\n\t"
            SH_FMAC_SET1(4, s86) SH_FMAC_SET1(5, s86) SH_FMAC_SET1(6, s86) SH_FMACL_SET1(7, s86)
            SH_READ_SET1
            SH_OFF
            // quad 2
            "s_sub_u32 s73, s73, 1\n\t"
            "s_cbranch_scc1 .Lsh_qend_%=\n\t"
            SH_ROWS(s86, 12)
            SH_ADDR(v38, v46, 8)
            "s_waitcnt lgkmcnt(2)\n\t"
            SH_FMAC_SET2(8, s70) SH_FMAC_SET2(9, s70) SH_FMAC_SET2(10, s70) SH_FMACL_SET2(11, s70)
            SH_READ_SET2
            SH_OFF
            // quad 3
            "s_sub_u32 s73, s73, 1\n\t"
            "s_cbranch_scc1 .Lsh_qend_%=\n\t"
            SH_ADDR(v39, v46, 12)
            SH_WAIT3
            SH_FMAC_SET3(12, s86) SH_FMAC_SET3(13, s86) SH_FMAC_SET3(14, s86) SH_FMACL_SET3(15, s86)
            SH_READ_SET3
            SH_OFF
            "s_cmp_eq_u32 s73, 0\n\t"
            "s_cbranch_scc1 .Lsh_qend_%=\n\t"
            SH_ADVANCE(1)
            "s_branch .Lsh_qblk_%=\n"
            // (reads issued for a block that is not of this part stay in flight: LDS answers in order, their
            // values are never used)
            ".Lsh_qend_%=:\n\t"
            SH_FILL_MID
            SH_ADVANCE(2)
            "s_mov_b32 s73, s67\n\t"
            "s_cmp_eq_u32 s67, 0\n\t"
            "s_cbranch_scc1 .Lsh_nos_%=\n\t"
            SH_ADDR(v36, v42, 0) SH_ADDR(v37, v42, 1) SH_ADDR(v38, v42, 2) SH_ADDR(v39, v42, 3)
            SH_READ_SET0 SH_READ_SET1 SH_READ_SET2 SH_READ_SET3
            "s_branch .Lsh_sblk_%=\n"
            ".Lsh_noq_%=:\n\t"
            "s_cmp_eq_u32 s67, 0\n\t"
            "s_cbranch_scc1 .Lsh_empty_%=\n\t"
            SH_ADDR(v36, v42, 0) SH_ADDR(v37, v42, 1) SH_ADDR(v38, v42, 2) SH_ADDR(v39, v42, 3)
            SH_READ_SET0 SH_READ_SET1 SH_READ_SET2 SH_READ_SET3
            SH_FILL_HEAD
// a group of four singles: its B values were requested a whole group ahead into one bank of four sets (sets 0..3 or
// 4..7: the groups of a band alternate), so that one wait covers them: first the addresses of the four records
// after them (records n0..n3 of `src`) and their reads into the other bank (R0..R3), where there is one the rows of
// the next group, then the wait that leaves only those four reads outstanding, then the multiply-adds (F0..F3)
#define SH_GROUP(src, n0, n1, n2, n3, R0, R1, R2, R3, nextrows, F0, F1, F2, F3)           \
            "s_sub_u32 s73, s73, 1\n\t"                                               \
            "s_cbranch_scc1 .Lsh_send_%=\n\t"                                         \
            SH_GROUP_READS(SH_ADDR(v36, src, n0) SH_ADDR(v37, src, n1) SH_ADDR(v38, src, n2) SH_ADDR(v39, src, n3) R0 R1 R2 R3) \
            nextrows                                                                  \
            "s_waitcnt lgkmcnt(4)\n\t"                                                \
            F0 F1 F2 F3                                                               \
            SH_OFF
#define SH_GROUP_0 SH_ROWS(s70, 0)                                                                                      \
            SH_GROUP(v42, 4, 5, 6, 7, SH_READ_SET4, SH_READ_SET5, SH_READ_SET6, SH_READ_SET7, SH_ROWS(s86, 4),         \
                     SH_FMAC_SET0(0, s70), SH_FMAC_SET1(1, s70), SH_FMAC_SET2(2, s70), SH_FMACL_SET3(3, s70))
#define SH_GROUP_1                                                                                                      \
            SH_GROUP(v42, 8, 9, 10, 11, SH_READ_SET0, SH_READ_SET1, SH_READ_SET2, SH_READ_SET3, SH_ROWS(s70, 8),       \
                     SH_FMAC_SET4(4, s86), SH_FMAC_SET5(5, s86), SH_FMAC_SET6(6, s86), SH_FMACL_SET7(7, s86))
#define SH_GROUP_2                                                                                                      \
            SH_GROUP(v42, 12, 13, 14, 15, SH_READ_SET4, SH_READ_SET5, SH_READ_SET6, SH_READ_SET7, SH_ROWS(s86, 12),    \
                     SH_FMAC_SET0(8, s70), SH_FMAC_SET1(9, s70), SH_FMAC_SET2(10, s70), SH_FMACL_SET3(11, s70))
#define SH_GROUP_3                                                                                                      \
            SH_GROUP(v46, 0, 1, 2, 3, SH_READ_SET0, SH_READ_SET1, SH_READ_SET2, SH_READ_SET3, "",                      \
                     SH_FMAC_SET4(12, s86), SH_FMAC_SET5(13, s86), SH_FMAC_SET6(14, s86), SH_FMACL_SET7(15, s86))
            // ---- singles, four at a time; in a band without quads the second part of the rows is requested behind
            // the first group
            "s_mov_b32 s73, s67\n\t"
            SH_GROUP_0
            SH_FILL_MID
            "s_branch .Lsh_sgroup1_%=\n"
            ".Lsh_sblk_%=:\n\t"
            SH_GROUP_0
            ".Lsh_sgroup1_%=:\n\t"
            SH_GROUP_1 SH_GROUP_2 SH_GROUP_3
            "s_cmp_eq_u32 s73, 0\n\t"
            "s_cbranch_scc1 .Lsh_send_%=\n\t"
            SH_ADVANCE(3)
            "s_branch .Lsh_sblk_%=\n"
            ".Lsh_send_%=:\n\t"
            SH_ADVANCE(4)
            ".Lsh_nos_%=:\n\t"
            // ---- (quads, singles) of the next band; every 64 bands the pairs of the following 64 take over
            // (out of line, behind the loop).  The buffers turn on meanwhile: band b lives in buffer -b mod 3, so
            // the rows of band b + 3 go where band b was.
            SH_FILL_TAIL
            "s_add_u32 s64, s64, 1\n\t"
            "s_and_b32 s71, s64, 63\n\t"
            "s_cbranch_scc0 .Lsh_newhdr_%=\n"
            ".Lsh_samehdr_%=:\n\t"
            "s_mov_b32 s89, s88\n\t"
            "s_sub_u32 s88, s88, 0xC000\n\t"
            "s_cselect_b32 s88, 0x18000, s88\n\t"
            "s_nop 0\n\t"
            "v_readlane_b32 s66, v54, s71\n\t"
            "v_readlane_b32 s67, v55, s71\n\t"
            // ---- the rows of band b+1 have landed (those of band b+2, requested in this band, may still be on
            // their way) and so has everything requested before this band began; all waves are done with band b
            SH_WAIT_FILLS
            SH_BAND_BARRIER
            "s_max_u32 s82, s82, s83\n\t"
            "s_cmp_lt_u32 s64, s65\n\t"
            "s_cbranch_scc1 .Lsh_band_%=\n\t"
            "s_branch .Lsh_done_%=\n"
            // a band in which this wave has no entry
            ".Lsh_empty_%=:\n\t"
            SH_FILL_HEAD
            SH_FILL_MID
            "s_branch .Lsh_nos_%=\n"
            ".Lsh_newhdr_%=:\n\t"
            "v_mov_b32 v54, v56\n\t"
            "v_mov_b32 v55, v57\n\t"
            "v_lshrrev_b32 v50, 1, v59\n\t"
            "global_load_dwordx2 v[56:57], v50, s[74:75]\n\t"
            "s_add_u32 s74, s74, 0x200\n\t"
            "s_addc_u32 s75, s75, 0\n\t"
            "s_branch .Lsh_samehdr_%=\n"
            SH_ADVANCE_PIECE(0) SH_ADVANCE_PIECE(1) SH_ADVANCE_PIECE(2) SH_ADVANCE_PIECE(3) SH_ADVANCE_PIECE(4)
            // the rows requested for the bands beyond the last one arrive before the wave gives up its LDS
            ".Lsh_done_%=:\n\t"
            "s_waitcnt vmcnt(0)\n\t"
            : "+{v[60:63]}"(acc.t0), "+{v[64:95]}"(acc.t1), "+{v[96:127]}"(acc.t2), "+{v[128:159]}"(acc.t3),
              "+{v[160:191]}"(acc.t4), "+{v[192:223]}"(acc.t5), "+{v[224:255]}"(acc.t6)
            : [hdr] "s"(hdr), [strm] "s"(strm), [uc] "s"(uc), [bt] "s"(bt), [nb] "s"(nb), [ldb4] "s"(ldb4), [ring] "s"(ring),
              [fillw] "s"(fillw), [last] "s"(last), "{v59}"(l16), "{v58}"(l16g), "{v43}"(sh8), "{v3}"(cidx), "{v53}"(rl), "{v51}"(fbias)
            : "m0", "scc", "memory", "v20", "v21", "v22", "v23", "v24", "v25", "v26", "v27", "v28", "v29", "v30", "v31", "v32", "v33",
              "v34", "v35", "v36", "v37", "v38", "v39", "v40", "v41", "v42", "v44", "v45", "v46", "v47", "v48", "v49", "v50",
              "v52", "v54", "v55", "v56", "v57", "v4", "v5", "v6", "v7", "v8", "v9", "v10", "v11", "v12", "v13", "v14", "v15",
              "v16", "v17", "v18", "v19", "s64", "s65", "s66", "s67", "s68", "s69", "s70", "s71", "s73",
              "s74", "s75", "s76", "s77", "s78", "s79", "s80", "s82", "s83", "s84", "s85", "s86", "s87", "s88", "s89");
    }

    // The lane's columns once more, from a thread index the compiler cannot connect with the one above: the loop
    // leaves it three registers, too few to carry the lane's place in C across it.
    uint32_t tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int64_t jc = tile * 256 + (int64_t)(tid & 63u) * 4;
    if (q < a.g && jc < a.N) {
        const int64_t row0 = q * a.p;
        float* __restrict__ Cl = a.C + jc;
#pragma unroll
        for (int r = 0; r < kShareMaxP; ++r) {
            if (r < a.p && row0 + r < a.m) {
                sh_f32x4 o = {share_acc_get(acc, kShareAccFirst + r), share_acc_get(acc, kShareAccFirst + kShareAccStride + r),
                              share_acc_get(acc, kShareAccFirst + 2 * kShareAccStride + r),
                              share_acc_get(acc, kShareAccFirst + 3 * kShareAccStride + r)};
                __builtin_nontemporal_store(o, reinterpret_cast<sh_f32x4*>(Cl + (row0 + r) * a.ldc));
            }
        }
    }
}

}  // namespace gcoo
