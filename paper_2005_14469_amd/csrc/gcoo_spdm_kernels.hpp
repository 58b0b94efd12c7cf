// SpDM kernel with the partial sums in registers (Algorithm 2 of the paper, re-cut for CDNA4).
//
// Work unit = (group q, column tile): one wave64 computes a  p x (64*V)  tile of C.  Every lane
// owns V adjacent columns and keeps (p+1) x V partial sums.  The entries of the group are
// wave-uniform data: the wave streams them from global memory into LDS with coalesced loads, far
// ahead of their use, and reads them back with broadcast reads (the staging in shared memory of
// Algorithm 2); the B row segment of a run of entries is one coalesced vector load per lane, and
// all entries of the run multiply out of those registers (the reuse of a fetched value of B that
// Section 3.3 builds the kernel around).  The entries are read from the run
// schedule (gcoo_sched.hpp), in which runs are sorted by length, so the code for a run of L
// entries is straight-line: no "is the next column the same" test at run time.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gcoo_sched.hpp"
#include "gcoo_spdm_launch.hpp"

// Two layouts of the accumulator file, one per translation unit (everything below is compiled
// inside an inline namespace named after the layout, so the two sets of kernels do not collide):
//   standard  v[124:255]: 33 x 4, 65 x 2 or 129 x 1 partial sums (p <= 32 / 64 / 128)
//   tall      v[100:255]: 39 x 4 partial sums (p <= 38), for which the compiler is left 100 VGPRs
//             (with fewer it parks values in AGPRs, also ones whose load is still in flight, which
//             the build's check of the generated code refuses);
//             taller groups mean fewer fetched B rows per multiply-add where groups are dense
//             enough to touch most columns (Section 3.3)
#ifdef GCOO_ACC_TALL
#define GCOO_ACC_NS acc_tall
#else
#define GCOO_ACC_NS acc_std
#endif

namespace gcoo {
inline namespace GCOO_ACC_NS {

// ---------------------------------------------------------------------------------------------
// Accumulator file.  The (p+1) x V partial sums of a lane sit in the fixed VGPR range v[124:255]:
//     sum(v, r) = v[124 + v*stride + r],   stride = 33 (V = 4, p <= 32), 65 (V = 2, p <= 64), 129 (V = 1, p <= 128)
// Row p of a group is the sink of the dummy entries of the schedule.  Which row an entry adds to
// is known only at run time but is the same for the whole wave, so the add uses the VGPR index
// mode of the GFX9 scalar unit: s_set_gpr_idx_on / s_set_gpr_idx_idx load M0[7:0] with the row
// and make the destination and the third source of the following VALU instructions relative to
// it; one v_fma_f32 per column then updates the right register with no select chain and no
// memory traffic.  The five register tuples are passed to every asm statement as read-write
// operands pinned to those registers, so the compiler knows what is read and written.
// ---------------------------------------------------------------------------------------------
typedef float f32x32 __attribute__((ext_vector_type(32)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

#ifdef GCOO_ACC_TALL
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
struct AccFile {
    f32x4 t0;                 // v[100:103]
    f32x32 t1, t2, t3, t4;    // v[104:135] v[136:167] v[168:199] v[200:231]
    f32x16 t5;                // v[232:247]
    f32x8 t6;                 // v[248:255]
};
constexpr int kAccFirst = 100;

#define GCOO_ACC_OPERANDS(acc)                                                                                      \
    "+{v[100:103]}"((acc).t0), "+{v[104:135]}"((acc).t1), "+{v[136:167]}"((acc).t2), "+{v[168:199]}"((acc).t3),   \
        "+{v[200:231]}"((acc).t4), "+{v[232:247]}"((acc).t5), "+{v[248:255]}"((acc).t6)

template <int V>
__host__ __device__ constexpr int acc_stride()
{
    static_assert(V == 4, "the tall layout exists for four columns per lane only");
    return 39;
}

__device__ __forceinline__ void acc_clear(AccFile& acc)
{
    acc.t0 = 0.0f; acc.t1 = 0.0f; acc.t2 = 0.0f; acc.t3 = 0.0f; acc.t4 = 0.0f; acc.t5 = 0.0f; acc.t6 = 0.0f;
}

__device__ __forceinline__ float acc_get(const AccFile& acc, int reg)
{
    const int s = reg - kAccFirst;
    if (s < 4) return acc.t0[s];
    if (s >= 148) return acc.t6[s - 148];
    if (s >= 132) return acc.t5[s - 132];
    const int t = (s - 4) >> 5, i = (s - 4) & 31;
    return t == 0 ? acc.t1[i] : (t == 1 ? acc.t2[i] : (t == 2 ? acc.t3[i] : acc.t4[i]));
}

__device__ __forceinline__ void acc_add(AccFile& acc, int reg, float x)
{
    const int s = reg - kAccFirst;
    if (s < 4) { acc.t0[s] += x; return; }
    if (s >= 148) { acc.t6[s - 148] += x; return; }
    if (s >= 132) { acc.t5[s - 132] += x; return; }
    const int t = (s - 4) >> 5, i = (s - 4) & 31;
    if (t == 0) acc.t1[i] += x; else if (t == 1) acc.t2[i] += x; else if (t == 2) acc.t3[i] += x; else acc.t4[i] += x;
}
#else
struct AccFile {
    f32x4 t0;                 // v[124:127]
    f32x32 t1, t2, t3, t4;    // v[128:159] v[160:191] v[192:223] v[224:255]
};
constexpr int kAccFirst = 124;

#define GCOO_ACC_OPERANDS(acc)                                                                     \
    "+{v[124:127]}"((acc).t0), "+{v[128:159]}"((acc).t1), "+{v[160:191]}"((acc).t2), "+{v[192:223]}"((acc).t3), \
        "+{v[224:255]}"((acc).t4)

template <int V>
__host__ __device__ constexpr int acc_stride()
{
    return V == 4 ? 33 : (V == 2 ? 65 : 129);
}

__device__ __forceinline__ void acc_clear(AccFile& acc)
{
    acc.t0 = 0.0f; acc.t1 = 0.0f; acc.t2 = 0.0f; acc.t3 = 0.0f; acc.t4 = 0.0f;
}

__device__ __forceinline__ float acc_get(const AccFile& acc, int reg)
{
    const int s = reg - kAccFirst;
    if (s < 4) return acc.t0[s];
    const int t = (s - 4) >> 5, i = (s - 4) & 31;
    return t == 0 ? acc.t1[i] : (t == 1 ? acc.t2[i] : (t == 2 ? acc.t3[i] : acc.t4[i]));
}

__device__ __forceinline__ void acc_add(AccFile& acc, int reg, float x)
{
    const int s = reg - kAccFirst;
    if (s < 4) { acc.t0[s] += x; return; }
    const int t = (s - 4) >> 5, i = (s - 4) & 31;
    if (t == 0) acc.t1[i] += x; else if (t == 1) acc.t2[i] += x; else if (t == 2) acc.t3[i] += x; else acc.t4[i] += x;
}
#endif

// Instruction text.  GCOO_FMA_Vn(i): the V multiply-adds of entry i of a run (operands a<i> =
// the entry's value, the same in every lane of a VGPR; b0..b3 = the run's B segment).  GCOO_ENT(i) = select row c<i>, then those.
#ifdef GCOO_ACC_TALL
// (the one- and two-column texts are parsed but never instantiated in this layout: acc_stride refuses them)
#define GCOO_FMA_V1(i) "v_fma_f32 v100, %[a" #i "], %[b0], v100\n\t"
#define GCOO_FMA_V2(i) GCOO_FMA_V1(i) "v_fma_f32 v139, %[a" #i "], %[b1], v139\n\t"
#define GCOO_FMA_V4(i)                                  \
    GCOO_FMA_V2(i)                                      \
    "v_fma_f32 v178, %[a" #i "], %[b2], v178\n\t"        \
    "v_fma_f32 v217, %[a" #i "], %[b3], v217\n\t"
#else
#define GCOO_FMA_V1(i) "v_fma_f32 v124, %[a" #i "], %[b0], v124\n\t"
#define GCOO_FMA_V2(i) GCOO_FMA_V1(i) "v_fma_f32 v189, %[a" #i "], %[b1], v189\n\t"
#define GCOO_FMA_V4(i)                                  \
    GCOO_FMA_V1(i)                                      \
    "v_fma_f32 v157, %[a" #i "], %[b1], v157\n\t"        \
    "v_fma_f32 v190, %[a" #i "], %[b2], v190\n\t"        \
    "v_fma_f32 v223, %[a" #i "], %[b3], v223\n\t"
#endif
#define GCOO_ENT0(FMA) "s_set_gpr_idx_on %[c0], gpr_idx(SRC2,DST)\n\t" FMA(0)
#define GCOO_ENT(FMA, i) "s_set_gpr_idx_idx %[c" #i "]\n\t" FMA(i)
#define GCOO_RUN1(FMA) GCOO_ENT0(FMA)
#define GCOO_RUN2(FMA) GCOO_RUN1(FMA) GCOO_ENT(FMA, 1)
#define GCOO_RUN3(FMA) GCOO_RUN2(FMA) GCOO_ENT(FMA, 2)
#define GCOO_RUN4(FMA) GCOO_RUN3(FMA) GCOO_ENT(FMA, 3)
#define GCOO_RUN5(FMA) GCOO_RUN4(FMA) GCOO_ENT(FMA, 4)
#define GCOO_RUN6(FMA) GCOO_RUN5(FMA) GCOO_ENT(FMA, 5)
#define GCOO_RUN7(FMA) GCOO_RUN6(FMA) GCOO_ENT(FMA, 6)
#define GCOO_RUN8(FMA) GCOO_RUN7(FMA) GCOO_ENT(FMA, 7)
#define GCOO_OFF "s_set_gpr_idx_off"

#define GCOO_B_V1(b) [b0] "v"((b)[0])
#define GCOO_B_V2(b) GCOO_B_V1(b), [b1] "v"((b)[1])
#define GCOO_B_V4(b) GCOO_B_V2(b), [b2] "v"((b)[2]), [b3] "v"((b)[3])
#define GCOO_E1(c, a) [c0] "s"((c)[0]), [a0] "v"((a)[0])
#define GCOO_E2(c, a) GCOO_E1(c, a), [c1] "s"((c)[1]), [a1] "v"((a)[1])
#define GCOO_E3(c, a) GCOO_E2(c, a), [c2] "s"((c)[2]), [a2] "v"((a)[2])
#define GCOO_E4(c, a) GCOO_E3(c, a), [c3] "s"((c)[3]), [a3] "v"((a)[3])
#define GCOO_E5(c, a) GCOO_E4(c, a), [c4] "s"((c)[4]), [a4] "v"((a)[4])
#define GCOO_E6(c, a) GCOO_E5(c, a), [c5] "s"((c)[5]), [a5] "v"((a)[5])
#define GCOO_E7(c, a) GCOO_E6(c, a), [c6] "s"((c)[6]), [a6] "v"((a)[6])
#define GCOO_E8(c, a) GCOO_E7(c, a), [c7] "s"((c)[7]), [a7] "v"((a)[7])

// The index mode keeps the row in M0, which the compiler otherwise owns (it loads M0 in front of
// every instruction of its own that reads it): the clobber tells it that the value is gone.
#define GCOO_RUN_ASM(L, VN) \
    asm volatile(GCOO_RUN##L(GCOO_FMA_V##VN) GCOO_OFF : GCOO_ACC_OPERANDS(acc) : GCOO_E##L(c, a), GCOO_B_V##VN(b) : "m0")
#define GCOO_RUN_CASE(L)                           \
    if constexpr (V == 4) GCOO_RUN_ASM(L, 4);      \
    else if constexpr (V == 2) GCOO_RUN_ASM(L, 2); \
    else GCOO_RUN_ASM(L, 1)

// One run of L entries: sums(:, c[i]) += a[i] * b(:) for i = 0..L-1, one asm statement.
template <int L, int V>
__device__ __forceinline__ void run_fma(AccFile& acc, const uint32_t* c, const float* a, const float (&b)[V])
{
    static_assert(L >= 1 && L <= kMaxRun && (V == 1 || V == 2 || V == 4), "");
    if constexpr (L == 1) { GCOO_RUN_CASE(1); }
    else if constexpr (L == 2) { GCOO_RUN_CASE(2); }
    else if constexpr (L == 3) { GCOO_RUN_CASE(3); }
    else if constexpr (L == 4) { GCOO_RUN_CASE(4); }
    else if constexpr (L == 5) { GCOO_RUN_CASE(5); }
    else if constexpr (L == 6) { GCOO_RUN_CASE(6); }
    else if constexpr (L == 7) { GCOO_RUN_CASE(7); }
    else { GCOO_RUN_CASE(8); }
}

// A lane's V adjacent values of a row of B, issued from an asm statement: the compiler does not
// know that the result is still in flight, so it puts no s_waitcnt in front of the uses and the
// pipelined loop places its own.  The destination may be read only by asm statements that come
// after such a wait (the build verifies the generated code for that: isa_check.py).
// Address = 64-bit scalar row base + 32-bit per-lane byte offset.
template <int V>
__device__ __forceinline__ void load_b_async(const char* row_base, uint32_t lane_off, float (&b)[V])
{
    if constexpr (V == 4) {
        f32x4 t;
        asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(t) : "v"(lane_off), "s"(row_base));
        b[0] = t.x; b[1] = t.y; b[2] = t.z; b[3] = t.w;
    } else if constexpr (V == 2) {
        f32x2 t;
        asm volatile("global_load_dwordx2 %0, %1, %2" : "=v"(t) : "v"(lane_off), "s"(row_base));
        b[0] = t.x; b[1] = t.y;
    } else {
        asm volatile("global_load_dword %0, %1, %2" : "=v"(b[0]) : "v"(lane_off), "s"(row_base));
    }
}

// Wait until at most N vector-memory loads are still in flight (they complete in order, so
// everything issued before the youngest N has arrived).
template <int N>
__device__ __forceinline__ void wait_vm()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N));
}

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// One 512-byte line of the schedule stream, 8 bytes per lane, issued from asm like the B loads.
__device__ __forceinline__ u32x2 load_line_async(const uint32_t* line, uint32_t lane8)
{
    u32x2 t;
    asm volatile("global_load_dwordx2 %0, %1, %2" : "=v"(t) : "v"(lane8), "s"(line));
    return t;
}

// The line goes to LDS at lds_addr (this lane's 8 bytes).  Issued from asm because its source is
// an asm-loaded register.  The compiler does not see this store, so the ring is only ever read
// through volatile pointers (read_ring4): those reads are neither removed nor moved across asm
// statements, and LDS executes a wave's operations in order.
__device__ __forceinline__ void store_line_lds(uint32_t lds_addr, u32x2 v)
{
    asm volatile("ds_write_b64 %0, %1" : : "v"(lds_addr), "v"(v));
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

typedef __attribute__((address_space(3))) uint32_t lds_u32;
typedef __attribute__((address_space(3))) u32x4 lds_u32x4;

// N words (a multiple of 4) of the ring, one 16-byte broadcast read each.
template <int N>
__device__ __forceinline__ void read_ring4(const lds_u32* p, uint32_t (&out)[N])
{
    static_assert(N % 4 == 0, "");
#pragma unroll
    for (int i = 0; i < N / 4; ++i) {
        const u32x4 t = *(const volatile lds_u32x4*)(p + 4 * i);
        out[4 * i] = t.x; out[4 * i + 1] = t.y; out[4 * i + 2] = t.z; out[4 * i + 3] = t.w;
    }
}

// LDS ring of the stream: kRing lines of 128 words per wave.
constexpr int kRing = 3;
constexpr int kLineWords = 128;

// All bodies of one length class of one (group, window).
//
// Turn b of the loop multiplies chunks 4b .. 4b+3 (kBody = 4) and starts the B loads of chunks
// 4b+3 .. 4b+6, so three chunks of loads are always in flight behind the one being used.  Line b
// of the stream = the 128 words from word b*BD of the segment: the pre-block-sized lead (for
// b = 0 the pre-block itself), then block b.  It was loaded two turns earlier and sits in LDS:
// its columns and row bytes are read back and moved to SGPRs (v_readfirstlane), its values are
// read back into VGPRs, where every lane holds the same number.  Per turn the vector-memory
// order is
//     line(b+2), B(4b+3) | B(4b+4) | B(4b+5) | B(4b+6)
// so the wait before chunk 4b+st leaves 3J+1 loads in flight for st = 0..2 and 3J for st = 3; after
// that last wait line(b+2) has arrived and is written to LDS.  Loads are in flight across the
// back-edge of the loop and from the start-up into the loop; the class ends with vmcnt(0).
//
// SUB: the caller works on bodies [b0, b1) of the segment only (a group shared by the waves of
// a workgroup).  The columns of the first three chunks of body b0 > 0 are not in a pre-block of
// their own: they are the last three column slots of block b0-1, so that block's line is
// fetched once at start-up.  The loads that the last turn starts for chunks past b1 fetch rows
// that belong to the next part of the segment (or the padding columns): valid rows, ignored.
template <int L, int V, bool SUB = false>
__device__ __forceinline__ void run_class(AccFile& acc, const uint32_t* seg, int32_t b0, int32_t b1, const char* Bbytes,
                                          uint32_t ldb4, uint32_t lane_off, const lds_u32* ring, uint32_t ring_lds, int lane)
{
    constexpr int J = runs_per_chunk(L), RP = rowpack_dwords(L), VS = val_stride(L), BD = block_dwords(L), PRE = pre_dwords(L);
    static_assert(kBody == 4 && PRE + BD <= kLineWords, "a line holds the lead and one block; four load buffers rotate");
    if (b1 <= b0) return;
    float bq[kBody][J][V];
    const uint32_t lane8 = (uint32_t)lane * 8u;

    auto issue = [&](const uint32_t* col, float (&dst)[J][V]) {
#pragma unroll
        for (int j = 0; j < J; ++j) load_b_async<V>(Bbytes + (uint64_t)col[j] * ldb4, lane_off, dst[j]);
    };

    // start: lines b0 and b0+1 to LDS, then chunks 0..2 of body b0 in flight
    {
        u32x2 l0 = load_line_async(seg + (int64_t)b0 * BD, lane8);
        u32x2 l1 = load_line_async(seg + (int64_t)(b0 + 1 < b1 ? b0 + 1 : b0) * BD, lane8);
        const lds_u32* pre = ring;                                         // the three chunks' columns sit at pre[J .. 4J)
        if constexpr (SUB) {
            // (b0 > 0 is wave-uniform; both sides issue the same number of loads so that the
            // waits below hold on either path)
            u32x2 lp = load_line_async(seg + (int64_t)(b0 > 0 ? b0 - 1 : 0) * BD, lane8);
            wait_vm<0>();
            store_line_lds(ring_lds + 2 * kLineWords * 4 + lane8, lp);
            if (b0 > 0) pre = ring + 2 * kLineWords + PRE;
        } else {
            wait_vm<0>();
        }
        store_line_lds(ring_lds + lane8, l0);
        store_line_lds(ring_lds + kLineWords * 4 + lane8, l1);
        uint32_t c0[PRE];
        read_ring4<PRE>(pre, c0);
#pragma unroll
        for (int i = J; i < PRE; ++i) c0[i] = __builtin_amdgcn_readfirstlane(c0[i]);
        issue(&c0[J], bq[0]);
        issue(&c0[2 * J], bq[1]);
        issue(&c0[3 * J], bq[2]);
    }

    int32_t slot = 0;                                                      // (b - b0) % kRing
    for (int32_t b = b0; b < b1; ++b) {
        const lds_u32* blk = ring + slot * kLineWords + PRE;
        const int32_t nxt = b + 2 < b1 ? b + 2 : b1 - 1;
        u32x2 ln = load_line_async(seg + (int64_t)nxt * BD, lane8);
        uint32_t col[kBody * J], rpk[kBody * RP];
        read_ring4<kBody * J>(blk, col);
        read_ring4<kBody * RP>(blk + kBody * J, rpk);
#pragma unroll
        for (int i = 0; i < kBody * J; ++i) col[i] = __builtin_amdgcn_readfirstlane(col[i]);
#pragma unroll
        for (int i = 0; i < kBody * RP; ++i) rpk[i] = __builtin_amdgcn_readfirstlane(rpk[i]);
        // the values of a chunk are read back one chunk ahead, so that the read is in flight
        // behind the multiply-adds of the chunk before
        uint32_t vnext[VS];
        read_ring4<VS>(blk + blk_val(L, 0), vnext);
#pragma unroll
        for (int st = 0; st < kBody; ++st) {
            issue(&col[st * J], bq[(st + 3) % kBody]);
            float va[VS];
#pragma unroll
            for (int i = 0; i < VS; ++i) va[i] = __uint_as_float(vnext[i]);
            if (st + 1 < kBody) read_ring4<VS>(blk + blk_val(L, st + 1), vnext);
            if (st < 3) wait_vm<3 * J + 1>(); else wait_vm<3 * J>();
#pragma unroll
            for (int j = 0; j < J; ++j) {
                uint32_t r[L];
#pragma unroll
                for (int i = 0; i < L; ++i) r[i] = rpk[st * RP + (j * L + i) / 4] >> (8 * ((j * L + i) % 4));
                run_fma<L, V>(acc, r, &va[j * L], bq[st][j]);
            }
        }
        const int32_t wslot = slot == 0 ? 2 : slot - 1;                    // (b - b0 + 2) % kRing
        store_line_lds(ring_lds + (uint32_t)wslot * (kLineWords * 4) + lane8, ln);
        slot = slot == kRing - 1 ? 0 : slot + 1;
    }
    wait_vm<0>();                                                          // the loads of chunks past the end
}

// The V adjacent columns a lane computes.  Lane l of tile t owns columns j0 = t*64V + l*V .. j0+V-1.  When N is not
// a multiple of V, the last lane with a column inside C would reach beyond N: it computes columns N-V .. N-1 instead
// and stores only those of them that are its own (first_own .. V-1 of its vector); lanes wholly beyond N compute some
// columns inside B and store nothing.  So every 4V-byte access stays inside the N columns of a row, whatever ldb and
// ldc are; it may then be aligned to 4 bytes only, which the hardware serves (the compiler itself emits 16-byte
// accesses for data aligned to 4).  The launcher checks N >= V.
struct LaneCols {
    bool in;             // the lane owns at least one column of C
    int64_t jc;          // first column it computes
    int first_own;       // elements [first_own, V) of its vector are its own
};
template <int V>
__device__ __forceinline__ LaneCols lane_cols(int64_t tile, int lane, int64_t N)
{
    const int64_t j0 = tile * (64 * V) + (int64_t)lane * V;
    LaneCols c;
    c.in = j0 < N;
    const int64_t want = c.in ? j0 : tile * (64 * V);
    c.jc = want + V <= N ? want : N - V;
    c.first_own = c.in ? (int)(j0 - c.jc) : V;
    return c;
}

// Stores one row of a lane's columns (o[v] = column jc + v) with the non-temporal hint.
template <int V, typename Vec>
__device__ __forceinline__ void store_lane_row(float* __restrict__ dst, const Vec& o, int first_own)
{
    if (first_own == 0) {
        __builtin_nontemporal_store(o, reinterpret_cast<Vec*>(dst));
    } else {
#pragma unroll
        for (int v = 1; v < V; ++v)
            if (v >= first_own) __builtin_nontemporal_store(o[v], dst + v);
    }
}

template <int V>
__global__ __launch_bounds__(64) void spdm_sched(const SchedClass* __restrict__ hdr, const uint32_t* __restrict__ stream,
                                                 const int32_t* __restrict__ gIdxes, int64_t m, int32_t p, int64_t g,
                                                 int32_t nw, const float* __restrict__ B, int64_t ldb, int64_t N, float* __restrict__ C,
                                                 int64_t ldc, int64_t total, int64_t nnz, const unsigned long long* __restrict__ stats)
{
    // XCD-aware order: workgroup ids go round-robin over the 8 XCDs, so XCD x is given the
    // contiguous slice [x*per, (x+1)*per) of the (tile-major) work list: it walks through all
    // groups of one column tile of B before moving to the next tile, which keeps that tile of
    // B in its own L2.
    const uint32_t bid = blockIdx.x;
    const uint32_t per = gridDim.x >> 3;
    const int64_t w = (int64_t)(bid & 7u) * per + (bid >> 3);
    if (w >= total) return;
    const int64_t tile = w / g, q = w - tile * g;
    // a matrix with heavy groups (a launch of few items, `stats` given) is left to spdm_sched_coop altogether
    if (stats && sched_heavy_min(nnz, g, (N + 64 * V - 1) / (64 * V), (int64_t)__builtin_amdgcn_readfirstlane((uint32_t)stats[1])) != 0x7fffffff)
        return;
    const int32_t first_entry = __builtin_amdgcn_readfirstlane(gIdxes[q]);

    const int lane = threadIdx.x;
    const LaneCols lc = lane_cols<V>(tile, lane, N);
    const bool in = lc.in;
    // Row bases are wave-uniform (SGPRs); the lane's place inside the row is a 32-bit byte offset.
    const char* Bbytes = reinterpret_cast<const char*>(B);
    const uint32_t lane_off = (uint32_t)(lc.jc * 4);       // the launcher checks that ldb*4 fits 32 bits
    const uint32_t ldb4 = (uint32_t)ldb * 4u;

    AccFile acc;
    acc_clear(acc);

    // the wave's ring of stream lines (one wave per workgroup)
    __shared__ __attribute__((aligned(16))) uint32_t ring_mem[kRing * kLineWords];
    const lds_u32* ring = (const lds_u32*)ring_mem;
    const uint32_t ring_lds = (uint32_t)(uintptr_t)ring;

    // window by window (a band of B that stays in L2), class by class.  The header words are
    // made scalar by hand: after the volatile LDS reads the compiler no longer does it itself.
    const uint32_t* gs = stream + sched_group_base(first_entry, q, nw);
    const SchedClass* h = hdr + q * nw * kMaxRun;
    for (int32_t w8 = 0; w8 < nw * kMaxRun; w8 += kMaxRun) {
        int32_t fw[kMaxRun], nb[kMaxRun];
#pragma unroll
        for (int i = 0; i < kMaxRun; ++i) {
            fw[i] = __builtin_amdgcn_readfirstlane(h[w8 + i].first_word);
            nb[i] = __builtin_amdgcn_readfirstlane(h[w8 + i].bodies);
        }
        run_class<1, V>(acc, gs + fw[0], 0, nb[0], Bbytes, ldb4, lane_off, ring, ring_lds, lane);
        run_class<2, V>(acc, gs + fw[1], 0, nb[1], Bbytes, ldb4, lane_off, ring, ring_lds, lane);
        run_class<3, V>(acc, gs + fw[2], 0, nb[2], Bbytes, ldb4, lane_off, ring, ring_lds, lane);
        run_class<4, V>(acc, gs + fw[3], 0, nb[3], Bbytes, ldb4, lane_off, ring, ring_lds, lane);
        run_class<5, V>(acc, gs + fw[4], 0, nb[4], Bbytes, ldb4, lane_off, ring, ring_lds, lane);
        run_class<6, V>(acc, gs + fw[5], 0, nb[5], Bbytes, ldb4, lane_off, ring, ring_lds, lane);
        run_class<7, V>(acc, gs + fw[6], 0, nb[6], Bbytes, ldb4, lane_off, ring, ring_lds, lane);
        run_class<8, V>(acc, gs + fw[7], 0, nb[7], Bbytes, ldb4, lane_off, ring, ring_lds, lane);
    }

    // epilogue: each lane stores its V adjacent columns of every row of the group (coalesced
    // along N); rows beyond m (last group), the sink row p and lanes beyond N are skipped.
    // C is written once and not read again by this kernel: the stores carry the non-temporal
    // hint so that they do not push the B band out of L2 (measured: 15 % less time at 0.5 %
    // density, 6 % at 10 %).
    if (in) {
        constexpr int S = acc_stride<V>();
        const int64_t row0 = q * p;
        float* __restrict__ Cl = C + lc.jc;
#pragma unroll
        for (int r = 0; r < S - 1; ++r) {
            if (r < p && row0 + r < m) {
                float* dst = Cl + (row0 + r) * ldc;
                if constexpr (V == 4) {
                    f32x4 o = {acc_get(acc, kAccFirst + r), acc_get(acc, kAccFirst + S + r), acc_get(acc, kAccFirst + 2 * S + r),
                               acc_get(acc, kAccFirst + 3 * S + r)};
                    store_lane_row<4>(dst, o, lc.first_own);
                } else {
                    static_assert(V == 2, "");
                    f32x2 o = {acc_get(acc, kAccFirst + r), acc_get(acc, kAccFirst + S + r)};
                    store_lane_row<2>(dst, o, lc.first_own);
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Launches of few (group, tile) items, where the longest group would set the run time (the nnz-balanced
// splitting that the paper leaves as future work, Section 5).  One kernel serves all groups; its workgroups
// have kCoopWaves waves and take their work from the groups in order of falling size (`order`, `osize`: written
// at conversion), so that the hardware's dispatcher hands the long items out first:
//   * a heavy group (heavy_min entries or more) has a workgroup to itself: its class segments, laid end to
//     end, are cut into kCoopWaves stretches of equal entries, each wave keeps partial sums of its own, and the
//     partial sums are added up through LDS in a fixed tree order, so the result does not depend on timing.
//     Wave 0 stores C.
//   * the other groups go `bundle` to a workgroup, one wave each, neighbours in size (bundle = 1 .. 8: as few as
//     keeps every compute unit busy, chosen by the launcher from the number of items).
// A matrix without a heavy group is not served here but by spdm_sched, which keeps the groups of a column tile
// together on an XCD: both kernels are launched, and each decides from the statistics on the device whether the
// launch is its own (the other returns at once).
// Workgroup b < nheavy * tiles (nheavy = number of heavy groups) takes heavy group order[b / tiles], tile b % tiles; the
// workgroups after those take bundles of eight.  The launch has g * tiles workgroups, which is enough for any count of heavy groups;
// the rest return at once.
// ---------------------------------------------------------------------------------------------
constexpr int kCoopWaves = 8;
// entries of one body (kBody chunks) of class L, padding included
__host__ __device__ constexpr int body_entries(int L) { return kBody * runs_per_chunk(L) * L; }

template <int V>
__global__ __launch_bounds__(64 * kCoopWaves) void spdm_sched_coop(const SchedClass* __restrict__ hdr, const uint32_t* __restrict__ stream,
                                                                   const int32_t* __restrict__ gIdxes, int64_t m, int32_t p, int64_t g,
                                                                   int32_t nw, const float* __restrict__ B, int64_t ldb, int64_t N,
                                                                   float* __restrict__ C, int64_t ldc, int64_t total, int64_t nnz,
                                                                   const unsigned long long* __restrict__ stats,
                                                                   const int32_t* __restrict__ order, const int32_t* __restrict__ osize,
                                                                   int32_t bundle)
{
    constexpr int S = acc_stride<V>(), P = S - 1;          // rows an instance can hold
    __shared__ __attribute__((aligned(16))) uint32_t ring_mem[kCoopWaves][kRing * kLineWords];
    // partial sums on their way from wave to wave: [wave][row][lane][V].  Four columns per lane: a tree, the upper
    // half of the waves writes at a time; two columns per lane: one wave at a time (the tree, compiled for that
    // instance, made the compiler move partial sums through registers that still have loads in flight: the
    // build's check of the generated code refused it)
    constexpr int kParts = V == 4 ? kCoopWaves / 2 : 1;
    __shared__ __attribute__((aligned(16))) float part[kParts][P * 64 * V];

    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t tiles = (N + 64 * V - 1) / (64 * V);
    const int32_t heavy_min = sched_heavy_min(nnz, g, tiles, (int64_t)__builtin_amdgcn_readfirstlane((uint32_t)stats[1]));
    // nheavy = groups of heavy_min entries or more = first place in the falling list osize[] that is smaller:
    // two steps of 64 probes (g <= 4096)
    if (heavy_min == 0x7fffffff) return;                   // no heavy group: spdm_sched, launched beside this kernel, does it all
    int32_t nheavy = 0;
    {
        int32_t lo = 0, hi = (int32_t)g;
        while (lo < hi) {
            const int32_t stride = (hi - lo + 63) / 64;
            const int32_t at = lo + lane * stride;
            const bool big = at < hi && osize[at] >= heavy_min;
            const int n = __popcll(__ballot(big));             // the sizes fall: the probes that are big come first
            if (n == 0) {
                hi = lo;
            } else {
                const int32_t up = lo + n * stride;
                lo = lo + (n - 1) * stride + 1;
                hi = up < hi ? up : hi;
            }
        }
        nheavy = lo;
    }
    const int64_t b = blockIdx.x;
    const bool heavy = b < (int64_t)nheavy * tiles;
    int64_t tile, q;
    if (heavy) {
        tile = b % tiles;
        q = order[b / tiles];
    } else {
        const int64_t bb = b - (int64_t)nheavy * tiles;
        tile = bb % tiles;
        const int64_t at = nheavy + (bb / tiles) * bundle + wv;
        if (wv >= bundle || at >= g) return;               // a wave without a group, or a workgroup without work: no barrier follows on this path
        q = order[at];
    }
    q = __builtin_amdgcn_readfirstlane((int32_t)q);
    (void)total;
    const int32_t first_entry = __builtin_amdgcn_readfirstlane(gIdxes[q]);

    const LaneCols lc = lane_cols<V>(tile, lane, N);
    const bool in = lc.in;
    const char* Bbytes = reinterpret_cast<const char*>(B);
    const uint32_t lane_off = (uint32_t)(lc.jc * 4);
    const uint32_t ldb4 = (uint32_t)ldb * 4u;

    AccFile acc;
    acc_clear(acc);

    const lds_u32* ring = (const lds_u32*)ring_mem[wv];
    const uint32_t ring_lds = (uint32_t)(uintptr_t)ring;

    const uint32_t* gs = stream + sched_group_base(first_entry, q, nw);
    const SchedClass* h = hdr + q * nw * kMaxRun;
    // The group's class segments, window after window, laid end to end and measured in entries, are cut into
    // kCoopWaves equal stretches: wave wv takes the bodies that begin in [lo, hi).  A wave then works through one
    // or two long pieces of segments instead of a sliver of every segment (each piece costs a start and a drain
    // of the load pipeline), and the waves carry equal numbers of entries wherever the group's columns lie.
    int64_t all = 0;
    for (int32_t i = lane; i < nw * kMaxRun; i += 64) all += (int64_t)h[i].bodies * body_entries(i % kMaxRun + 1);
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) all += __shfl_xor(all, d, 64);
    const int64_t total_entries = ((int64_t)__builtin_amdgcn_readfirstlane((uint32_t)(all >> 32)) << 32) |
                                  (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)all);
    const int64_t lo = heavy ? total_entries * wv / kCoopWaves : 0, hi = heavy ? total_entries * (wv + 1) / kCoopWaves : total_entries;
    int64_t seg_lo = 0;                                    // entries in the segments before this one
    for (int32_t w8 = 0; w8 < nw * kMaxRun; w8 += kMaxRun) {
        int32_t fw[kMaxRun], b0[kMaxRun], b1[kMaxRun];
#pragma unroll
        for (int i = 0; i < kMaxRun; ++i) {
            fw[i] = __builtin_amdgcn_readfirstlane(h[w8 + i].first_word);
            const int32_t nb = __builtin_amdgcn_readfirstlane(h[w8 + i].bodies);
            const int32_t per = body_entries(i + 1);
            // bodies of this segment that begin before entry x of the whole: ceil((x - seg_lo) / per), within [0, nb]
            auto before = [&](int64_t x) -> int32_t {
                const int64_t d = x - seg_lo;
                if (d <= 0) return 0;
                if (d >= (int64_t)nb * per) return nb;
                return (int32_t)(((uint32_t)d + (uint32_t)per - 1u) / (uint32_t)per);   // a constant divisor
            };
            b0[i] = before(lo);
            b1[i] = before(hi);
            seg_lo += (int64_t)nb * per;
        }
        run_class<1, V, true>(acc, gs + fw[0], b0[0], b1[0], Bbytes, ldb4, lane_off, ring, ring_lds, lane);
        run_class<2, V, true>(acc, gs + fw[1], b0[1], b1[1], Bbytes, ldb4, lane_off, ring, ring_lds, lane);
        run_class<3, V, true>(acc, gs + fw[2], b0[2], b1[2], Bbytes, ldb4, lane_off, ring, ring_lds, lane);
        run_class<4, V, true>(acc, gs + fw[3], b0[3], b1[3], Bbytes, ldb4, lane_off, ring, ring_lds, lane);
        run_class<5, V, true>(acc, gs + fw[4], b0[4], b1[4], Bbytes, ldb4, lane_off, ring, ring_lds, lane);
        run_class<6, V, true>(acc, gs + fw[5], b0[5], b1[5], Bbytes, ldb4, lane_off, ring, ring_lds, lane);
        run_class<7, V, true>(acc, gs + fw[6], b0[6], b1[6], Bbytes, ldb4, lane_off, ring, ring_lds, lane);
        run_class<8, V, true>(acc, gs + fw[7], b0[7], b1[7], Bbytes, ldb4, lane_off, ring, ring_lds, lane);
    }

    // The look-ahead loads of the last class may still be on their way into registers that the compiler is free
    // to use from here on.
    wait_vm<0>();
    // The partial sums of the eight waves are added up in a fixed order, so the bits are the same on every run;
    // every wave of a heavy group's workgroup reaches every barrier (nothing above or below leaves the kernel
    // early on this path).
    if constexpr (V == 4) {
        // a tree, in three rounds: the upper half of the waves still in the round writes, the lower half adds its
        // partner's: ((w0 + w4) + (w2 + w6)) + ((w1 + w5) + (w3 + w7))
        for (int half = kCoopWaves / 2; heavy && half >= 1; half >>= 1) {
            if (wv >= half && wv < 2 * half) {
                float* mine = part[wv - half];
#pragma unroll
                for (int r = 0; r < P; ++r)
#pragma unroll
                    for (int v = 0; v < V; ++v) mine[(r * 64 + lane) * V + v] = acc_get(acc, kAccFirst + v * S + r);
            }
            __syncthreads();
            if (wv < half) {
                const float* theirs = part[wv];
#pragma unroll
                for (int r = 0; r < P; ++r)
#pragma unroll
                    for (int v = 0; v < V; ++v) acc_add(acc, kAccFirst + v * S + r, theirs[(r * 64 + lane) * V + v]);
            }
            __syncthreads();
        }
    } else {
        // one wave after the other into wave 0: ((w0 + w1) + w2) + ...
        for (int src = 1; heavy && src < kCoopWaves; ++src) {
            if (wv == src) {
#pragma unroll
                for (int r = 0; r < P; ++r)
#pragma unroll
                    for (int v = 0; v < V; ++v) part[0][(r * 64 + lane) * V + v] = acc_get(acc, kAccFirst + v * S + r);
            }
            __syncthreads();
            if (wv == 0) {
#pragma unroll
                for (int r = 0; r < P; ++r)
#pragma unroll
                    for (int v = 0; v < V; ++v) acc_add(acc, kAccFirst + v * S + r, part[0][(r * 64 + lane) * V + v]);
            }
            __syncthreads();
        }
    }

    if ((wv == 0 || !heavy) && in) {
        const int64_t row0 = q * p;
        float* __restrict__ Cl = C + lc.jc;
#pragma unroll
        for (int r = 0; r < P; ++r) {
            if (r < p && row0 + r < m) {
                float* dst = Cl + (row0 + r) * ldc;
                if constexpr (V == 4) {
                    f32x4 o = {acc_get(acc, kAccFirst + r), acc_get(acc, kAccFirst + S + r), acc_get(acc, kAccFirst + 2 * S + r),
                               acc_get(acc, kAccFirst + 3 * S + r)};
                    store_lane_row<4>(dst, o, lc.first_own);
                } else {
                    static_assert(V == 2, "");
                    f32x2 o = {acc_get(acc, kAccFirst + r), acc_get(acc, kAccFirst + S + r)};
                    store_lane_row<2>(dst, o, lc.first_own);
                }
            }
        }
    }
}

template <int V>
hipError_t launch_spdm_sched_instance(const SpdmArgs& a, hipStream_t s)
{
    const int64_t tiles = (a.N + 64 * V - 1) / (64 * V);
    const int64_t total = a.g * tiles;
    const int64_t grid = (total + 7) / 8 * 8;              // whole rounds over the 8 XCDs
    if (grid <= 0 || grid > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    if (a.ldb > 0x3fffffffLL) return hipErrorInvalidValue;   // row pitch in bytes is kept in 32 bits
    if (a.p + 1 > acc_stride<V>()) return hipErrorInvalidValue;
    if (a.N < V) return hipErrorInvalidValue;               // lane_cols() places a lane's columns inside [0, N)
#ifndef GCOO_ACC_TALL
    // A launch of few items, on a matrix that carries the list of its groups by size: the kernel that splits heavy
    // groups and bundles the others (no version of it in the tall layout: with 100 VGPRs it does not fit without
    // spilling registers whose loads are in flight)
    if (a.stats && a.order) {
        int64_t bundle = (total + 255) / 256;              // light groups per workgroup: one workgroup per compute unit and round
        bundle = bundle < 1 ? 1 : (bundle > kCoopWaves ? kCoopWaves : bundle);
        spdm_sched_coop<V><<<dim3((unsigned)total), dim3(64 * kCoopWaves), 0, s>>>(a.hdr, a.stream, a.gIdxes, a.m, a.p, a.g, a.nw, a.B,
                                                                                  a.ldb, a.N, a.C, a.ldc, total, a.nnz, a.stats,
                                                                                  a.order, a.order + a.g, (int32_t)bundle);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
#endif
    spdm_sched<V><<<dim3((unsigned)grid), dim3(64), 0, s>>>(a.hdr, a.stream, a.gIdxes, a.m, a.p, a.g, a.nw, a.B, a.ldb, a.N,
                                                            a.C, a.ldc, total, a.nnz, a.stats);
    return hipGetLastError();
}

}  // inline namespace
}  // namespace gcoo
