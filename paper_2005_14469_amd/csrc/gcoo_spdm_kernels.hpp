// SpDM kernels with the partial sums in registers (Algorithm 2 of the paper, re-cut for CDNA4).
//
// Work unit = (group q, column tile): one wave64 computes a  p x (64*V)  tile of C.  Every lane
// owns V adjacent columns and keeps p x V partial sums.  The entries of the group are wave-uniform
// data: they are fetched with scalar loads into SGPRs (the role shared memory plus broadcast plays
// in Algorithm 2), the B row segment of an entry is one coalesced vector load per lane, and while
// consecutive entries share a column the fetched segment is reused from registers (Section 3.3,
// "high computation-to-memory ratio").
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gcoo_spdm_launch.hpp"

namespace gcoo {

// ---------------------------------------------------------------------------------------------
// Register variants.
//
// The P x V partial sums of a lane sit in the fixed VGPR range v[128:255], laid out as
// sum(v, r) = v[128 + v*P + r]  (P*V = 128 or less).  Which row an entry adds to is only known at
// run time but is the same for the whole wave, so the add uses the VGPR index mode of the GFX9
// scalar unit: s_set_gpr_idx_on loads M0[7:0] with the row and makes the destination and the
// third source of the next VALU instructions relative to it; one v_fma_f32 per column then
// updates the right register with no select chain and no memory traffic.  The four 32-register
// tuples are passed to every asm statement as read-write operands pinned to those registers,
// so the compiler knows what is read and written.
// ---------------------------------------------------------------------------------------------
typedef float f32x32 __attribute__((ext_vector_type(32)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

struct AccFile {
    f32x32 t0, t1, t2, t3;
};

#define GCOO_ACC_OPERANDS(acc) \
    "+{v[128:159]}"((acc).t0), "+{v[160:191]}"((acc).t1), "+{v[192:223]}"((acc).t2), "+{v[224:255]}"((acc).t3)

// Instruction text for V columns per lane.  Column slot v of the accumulator file starts at
// v128 (V = 1), v128/v192 (V = 2, P = 64) or v128/v160/v192/v224 (V = 4, P <= 32).
#define GCOO_FMA_V1(x) "v_fma_f32 v128, %[a], %[" x "0], v128\n\t"
#define GCOO_FMA_V2(x) GCOO_FMA_V1(x) "v_fma_f32 v192, %[a], %[" x "1], v192\n\t"
#define GCOO_FMA_V4(x)                                 \
    GCOO_FMA_V1(x)                                     \
    "v_fma_f32 v160, %[a], %[" x "1], v160\n\t"         \
    "v_fma_f32 v192, %[a], %[" x "2], v192\n\t"         \
    "v_fma_f32 v224, %[a], %[" x "3], v224\n\t"
#define GCOO_MOV_V1(d, x) "v_mov_b32 %[" d "0], %[" x "0]\n\t"
#define GCOO_MOV_V2(d, x) GCOO_MOV_V1(d, x) "v_mov_b32 %[" d "1], %[" x "1]\n\t"
#define GCOO_MOV_V4(d, x) GCOO_MOV_V2(d, x) "v_mov_b32 %[" d "2], %[" x "2]\n\t" "v_mov_b32 %[" d "3], %[" x "3]\n\t"

#define GCOO_IDX_ON "s_set_gpr_idx_on %[c], gpr_idx(SRC2,DST)\n\t"
#define GCOO_IDX_OFF "s_set_gpr_idx_off\n\t"

// One entry, no run logic: sums(:, row) += a * s(:).  The low 8 bits of ctl are the row; the
// hardware ignores the rest.
#define GCOO_ITEM_PLAIN(FMA) GCOO_IDX_ON FMA("s") GCOO_IDX_OFF

// One entry with run logic, all inside one asm statement so that the accumulator file never
// crosses a branch the compiler can see:
//   first entry of a run (ctl < 0): multiply out of its own load buffer s;
//   otherwise: if the previous entry (ctl cp) was the first of the run, keep its buffer q in k
//              first (one copy per run of two or more), then multiply out of k.
#define GCOO_ITEM_RUN(FMA, MOV)                        \
    "s_cmp_lt_i32 %[c], 0\n\t"                         \
    "s_cbranch_scc1 1f\n\t"                            \
    "s_cmp_lt_i32 %[cp], 0\n\t"                        \
    "s_cbranch_scc0 2f\n\t"                            \
    MOV("k", "q")                                      \
    "2:\n\t"                                           \
    GCOO_IDX_ON FMA("k")                               \
    "s_branch 3f\n\t"                                  \
    "1:\n\t"                                           \
    GCOO_IDX_ON FMA("s")                               \
    "3:\n\t"                                           \
    GCOO_IDX_OFF

// k = s if ctl says "first of a run": done for the last entry of a chunk, whose load buffer
// is refilled while the run may still go on.
#define GCOO_KEEP_IF_HEAD(MOV)                         \
    "s_cmp_lt_i32 %[c], 0\n\t"                         \
    "s_cbranch_scc0 4f\n\t"                            \
    MOV("k", "s")                                      \
    "4:\n\t"

template <int V>
struct BSeg {
    float x[V];
};

// sums(:, row(ctl)) += a * s   (no reuse of B across entries)
template <int P, int V>
__device__ __forceinline__ void item_plain(AccFile& acc, uint32_t c, float a, const float (&s)[V])
{
    static_assert((V == 4 && P <= 32) || (V == 2 && P == 64) || (V == 1 && P == 128), "accumulator file layout");
    if constexpr (V == 4)
        asm volatile(GCOO_ITEM_PLAIN(GCOO_FMA_V4)
                     : GCOO_ACC_OPERANDS(acc)
                     : [c] "s"(c), [a] "s"(a), [s0] "v"(s[0]), [s1] "v"(s[1]), [s2] "v"(s[2]), [s3] "v"(s[3]));
    else if constexpr (V == 2)
        asm volatile(GCOO_ITEM_PLAIN(GCOO_FMA_V2) : GCOO_ACC_OPERANDS(acc) : [c] "s"(c), [a] "s"(a), [s0] "v"(s[0]), [s1] "v"(s[1]));
    else
        asm volatile(GCOO_ITEM_PLAIN(GCOO_FMA_V1) : GCOO_ACC_OPERANDS(acc) : [c] "s"(c), [a] "s"(a), [s0] "v"(s[0]));
}

// One entry with run reuse.  c/cp: control words of this and of the previous entry; s/q: their
// load buffers; k: the kept segment of the open run.
template <int P, int V>
__device__ __forceinline__ void item_run(AccFile& acc, uint32_t c, uint32_t cp, float a, const float (&s)[V],
                                         const float (&q)[V], float (&k)[V])
{
    static_assert((V == 4 && P <= 32) || (V == 2 && P == 64) || (V == 1 && P == 128), "accumulator file layout");
    if constexpr (V == 4)
        asm volatile(GCOO_ITEM_RUN(GCOO_FMA_V4, GCOO_MOV_V4)
                     : GCOO_ACC_OPERANDS(acc), [k0] "+v"(k[0]), [k1] "+v"(k[1]), [k2] "+v"(k[2]), [k3] "+v"(k[3])
                     : [c] "s"(c), [cp] "s"(cp), [a] "s"(a), [s0] "v"(s[0]), [s1] "v"(s[1]), [s2] "v"(s[2]), [s3] "v"(s[3]),
                       [q0] "v"(q[0]), [q1] "v"(q[1]), [q2] "v"(q[2]), [q3] "v"(q[3])
                     : "scc");
    else if constexpr (V == 2)
        asm volatile(GCOO_ITEM_RUN(GCOO_FMA_V2, GCOO_MOV_V2)
                     : GCOO_ACC_OPERANDS(acc), [k0] "+v"(k[0]), [k1] "+v"(k[1])
                     : [c] "s"(c), [cp] "s"(cp), [a] "s"(a), [s0] "v"(s[0]), [s1] "v"(s[1]), [q0] "v"(q[0]), [q1] "v"(q[1])
                     : "scc");
    else
        asm volatile(GCOO_ITEM_RUN(GCOO_FMA_V1, GCOO_MOV_V1)
                     : GCOO_ACC_OPERANDS(acc), [k0] "+v"(k[0])
                     : [c] "s"(c), [cp] "s"(cp), [a] "s"(a), [s0] "v"(s[0]), [q0] "v"(q[0])
                     : "scc");
}

// k = s when c marks the first entry of a run.
template <int V>
__device__ __forceinline__ void keep_if_head(uint32_t c, const float (&s)[V], float (&k)[V])
{
    if constexpr (V == 4)
        asm volatile(GCOO_KEEP_IF_HEAD(GCOO_MOV_V4)
                     : [k0] "+v"(k[0]), [k1] "+v"(k[1]), [k2] "+v"(k[2]), [k3] "+v"(k[3])
                     : [c] "s"(c), [s0] "v"(s[0]), [s1] "v"(s[1]), [s2] "v"(s[2]), [s3] "v"(s[3])
                     : "scc");
    else if constexpr (V == 2)
        asm volatile(GCOO_KEEP_IF_HEAD(GCOO_MOV_V2) : [k0] "+v"(k[0]), [k1] "+v"(k[1]) : [c] "s"(c), [s0] "v"(s[0]), [s1] "v"(s[1]) : "scc");
    else
        asm volatile(GCOO_KEEP_IF_HEAD(GCOO_MOV_V1) : [k0] "+v"(k[0]) : [c] "s"(c), [s0] "v"(s[0]) : "scc");
}

// Register slot of sum(v, r) inside the 128-register file, as laid out by fma_row.
template <int P, int V>
__device__ __forceinline__ constexpr int acc_slot(int v, int r)
{
    return (V == 4) ? 32 * v + r : (V == 2 ? 64 * v + r : r);
}

__device__ __forceinline__ float acc_get(const AccFile& acc, int slot)
{
    const int t = slot >> 5, i = slot & 31;
    return t == 0 ? acc.t0[i] : (t == 1 ? acc.t1[i] : (t == 2 ? acc.t2[i] : acc.t3[i]));
}

// One lane's V adjacent values of row `col` of B, loaded by the compiler (waits inserted by
// the compiler).  Used outside the pipelined loop.  Lanes of a tile that lie beyond N were
// pointed at column 0 by the caller, so every address is inside B.
template <int V>
__device__ __forceinline__ void load_b(const float* __restrict__ Bl, int64_t ldb, int32_t col, float (&b)[V])
{
    const float* ptr = Bl + (int64_t)col * ldb;
    if constexpr (V == 4) {
        const f32x4 t = *reinterpret_cast<const f32x4*>(ptr);
        b[0] = t.x; b[1] = t.y; b[2] = t.z; b[3] = t.w;
    } else if constexpr (V == 2) {
        const f32x2 t = *reinterpret_cast<const f32x2*>(ptr);
        b[0] = t.x; b[1] = t.y;
    } else {
        b[0] = *ptr;
    }
}

// The same load issued from an asm statement: the compiler does not know that the result is
// still in flight, so it puts no s_waitcnt in front of the uses and the pipelined loop places
// its own (wait_vm below).  The destination may be touched only by asm statements that come
// after such a wait; the build checks the generated code for that.
// Address = 64-bit scalar row base + 32-bit per-lane byte offset.
template <int V>
__device__ __forceinline__ void load_b_async(const float* row_base, uint32_t lane_off, float (&b)[V])
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

// Wait until at most `younger` vector-memory loads are still in flight (they complete in order,
// so everything issued before the youngest `younger` ones has arrived).
template <int N>
__device__ __forceinline__ void wait_vm_imm()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N));
}
// The same with a run-time count 0..8: s_waitcnt takes an immediate only, so a three-level
// compare tree picks one of nine.  Kept in one asm statement so that no compiler code lands
// between the branches.
template <int J>
__device__ __forceinline__ void wait_vm(uint32_t younger)
{
    static_assert(J == 8, "one case per possible number of loads of a chunk");
    asm volatile(
        "s_cmp_gt_u32 %0, 3\n\t"
        "s_cbranch_scc1 14f\n\t"
        "s_cmp_gt_u32 %0, 1\n\t"
        "s_cbranch_scc1 12f\n\t"
        "s_cmp_eq_u32 %0, 0\n\t"
        "s_cbranch_scc1 10f\n\t"
        "s_waitcnt vmcnt(1)\n\t"
        "s_branch 19f\n\t"
        "10:\n\t"
        "s_waitcnt vmcnt(0)\n\t"
        "s_branch 19f\n\t"
        "12:\n\t"
        "s_cmp_eq_u32 %0, 2\n\t"
        "s_cbranch_scc1 13f\n\t"
        "s_waitcnt vmcnt(3)\n\t"
        "s_branch 19f\n\t"
        "13:\n\t"
        "s_waitcnt vmcnt(2)\n\t"
        "s_branch 19f\n\t"
        "14:\n\t"
        "s_cmp_gt_u32 %0, 5\n\t"
        "s_cbranch_scc1 16f\n\t"
        "s_cmp_eq_u32 %0, 4\n\t"
        "s_cbranch_scc1 15f\n\t"
        "s_waitcnt vmcnt(5)\n\t"
        "s_branch 19f\n\t"
        "15:\n\t"
        "s_waitcnt vmcnt(4)\n\t"
        "s_branch 19f\n\t"
        "16:\n\t"
        "s_cmp_gt_u32 %0, 7\n\t"
        "s_cbranch_scc1 18f\n\t"
        "s_cmp_eq_u32 %0, 6\n\t"
        "s_cbranch_scc1 17f\n\t"
        "s_waitcnt vmcnt(7)\n\t"
        "s_branch 19f\n\t"
        "17:\n\t"
        "s_waitcnt vmcnt(6)\n\t"
        "s_branch 19f\n\t"
        "18:\n\t"
        "s_waitcnt vmcnt(8)\n\t"
        "19:"
        :
        : "s"(younger)
        : "scc");
}

// J entries of a group held in SGPRs.
template <int J>
struct Chunk {
    uint32_t ctl[J];
    int32_t col[J];
    float a[J];
};

template <int J>
__device__ __forceinline__ void load_chunk(Chunk<J>& c, const uint32_t* __restrict__ ctl, const int32_t* __restrict__ cols,
                                           const float* __restrict__ values, int32_t at)
{
#pragma unroll
    for (int j = 0; j < J; ++j) {
        c.ctl[j] = ctl[at + j];
        c.col[j] = cols[at + j];
        c.a[j] = values[at + j];
    }
}

// P: rows of partial sums kept (>= p of the matrix); V: columns per lane; J: entries per
// pipeline step (= kChunk, the chunk length the ctl words were built for); REUSE: follow runs
// of equal columns (one B load per run) or load per entry.
//
// Pipeline, per step n over chunks of J entries:
//   issue the B loads of chunk n+1  |  scalar-load chunk n+2  |  wait for chunk n  |  multiply-add chunk n
// Chunk buffers rotate with period 3, B buffers with period 2; the loop body is unrolled six
// steps so that every buffer index is a compile-time constant.  The wait lets the loads of
// chunk n+1 stay in flight: their number is the head count stored in the chunk's first ctl word.
template <int P, int V, int J, bool REUSE>
__global__ __launch_bounds__(64) void spdm_reg(const float* __restrict__ values, const int32_t* __restrict__ cols,
                                               const uint32_t* __restrict__ ctl, const int32_t* __restrict__ gIdxes,
                                               int64_t m, int32_t p, int64_t g, const float* __restrict__ B, int64_t ldb,
                                               int64_t N, float* __restrict__ C, int64_t ldc, int64_t total)
{
    static_assert(J == kChunk, "ctl words carry per-chunk head counts for chunks of kChunk entries");
    // XCD-aware order: workgroup ids go round-robin over the 8 XCDs, so XCD x is given the
    // contiguous slice [x*per, (x+1)*per) of the (tile-major) work list: it walks through all
    // groups of one column tile of B before moving to the next tile, which keeps that tile of
    // B in its own L2.
    const uint32_t bid = blockIdx.x;
    const uint32_t per = gridDim.x >> 3;
    const int64_t w = (int64_t)(bid & 7u) * per + (bid >> 3);
    if (w >= total) return;
    const int64_t tile = w / g, q = w - tile * g;

    const int lane = threadIdx.x;
    const int64_t j0 = tile * (64 * V) + (int64_t)lane * V;
    const bool in = j0 < N;                                // N % V == 0: a lane is all in or all out
    // Row bases are wave-uniform (SGPRs); the lane's place inside the tile is a 32-bit byte
    // offset.  Lanes beyond N read the first columns of the tile instead (always inside B).
    const float* __restrict__ Bt = B + tile * (64 * V);
    const char* Bbytes = reinterpret_cast<const char*>(Bt);
    const uint32_t ldb4 = (uint32_t)ldb * 4u;              // the launcher checks that ldb*4 fits 32 bits
    const uint32_t lane_off = in ? (uint32_t)(lane * V * 4) : 0u;
    const float* __restrict__ Bl = Bt + (in ? lane * V : 0);
    const int32_t beg = gIdxes[q], end = gIdxes[q + 1];
    const int32_t nch = (end - beg) / J;

    AccFile acc;
    acc.t0 = 0.0f; acc.t1 = 0.0f; acc.t2 = 0.0f; acc.t3 = 0.0f;

    Chunk<J> ck[3];
    float bq[2][J][V];
    float bcur[V];
#pragma unroll
    for (int v = 0; v < V; ++v) bcur[v] = 0.0f;
    // every load buffer starts defined: a slot that gets no load (not a run head) is still named
    // as an operand of the multiply-add statement, which then ignores it
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < J; ++j)
#pragma unroll
            for (int v = 0; v < V; ++v) bq[i][j][v] = 0.0f;

    auto issue = [&](const Chunk<J>& c, float (&dst)[J][V]) {
#pragma unroll
        for (int j = 0; j < J; ++j)
            if (!REUSE || (c.ctl[j] & kHeadBit))
                load_b_async<V>(reinterpret_cast<const float*>(Bbytes + (uint64_t)(uint32_t)c.col[j] * ldb4), lane_off, dst[j]);
    };
    // Number of loads `issue` starts for a chunk.
    auto loads_of = [&](const Chunk<J>& c) -> uint32_t { return REUSE ? ((c.ctl[0] >> kCountShift) & 15u) : (uint32_t)J; };
    // The first entry of a run multiplies straight out of its load buffer.  Only when a run goes
    // on to a second entry is the segment copied to `bcur` (once per run of length >= 2), and a
    // run that is still open at the end of a chunk is copied too, because its buffer is about
    // to be refilled.  The first entry of a chunk never has a previous buffer to copy from
    // (ctl word 0 = "not a head" is passed for it).
    auto compute = [&](const Chunk<J>& c, const float (&src)[J][V]) {
#pragma unroll
        for (int j = 0; j < J; ++j) {
            if constexpr (REUSE)
                item_run<P, V>(acc, c.ctl[j], j > 0 ? c.ctl[j - 1] : 0u, c.a[j], src[j], src[j > 0 ? j - 1 : 0], bcur);
            else
                item_plain<P, V>(acc, c.ctl[j], c.a[j], src[j]);
        }
        if constexpr (REUSE) keep_if_head<V>(c.ctl[J - 1], src[J - 1], bcur);
    };

    // Loads issued by asm are invisible to the compiler, so they may be in flight only where the
    // compiler has no reason to move their destination registers: inside the body of the
    // steady-state loop.  The loop is entered and left with nothing in flight (vmcnt(0) before
    // the first step and at the end of the last one).
    int32_t n = 0;
    if (nch >= 8) {
        load_chunk<J>(ck[0], ctl, cols, values, beg);
        load_chunk<J>(ck[1], ctl, cols, values, beg + J);
        issue(ck[0], bq[0]);
        wait_vm_imm<0>();
        // steady state: every step has a next and a next-but-one chunk, so nothing is conditional
        do {
#pragma unroll
            for (int s = 0; s < 6; ++s) {
                issue(ck[(s + 1) % 3], bq[(s + 1) % 2]);
                load_chunk<J>(ck[(s + 2) % 3], ctl, cols, values, beg + (n + s + 2) * J);
                if constexpr (REUSE) wait_vm<J>(loads_of(ck[(s + 1) % 3])); else wait_vm_imm<J>();
                compute(ck[s % 3], bq[s % 2]);
            }
            n += 6;
            if (n + 8 > nch) wait_vm_imm<0>();           // last round: drain before leaving
        } while (n + 8 <= nch);
        // chunk n has arrived in load buffer 0; chunks n, n+1 are in the scalar buffers 0 and 1
        compute(ck[0], bq[0]);
        issue(ck[1], bq[1]);
        wait_vm_imm<0>();
        compute(ck[1], bq[1]);
        n += 2;
    }
    // the last (up to seven) chunks, one at a time
    for (; n < nch; ++n) {
        load_chunk<J>(ck[0], ctl, cols, values, beg + n * J);
        issue(ck[0], bq[0]);
        wait_vm_imm<0>();
        compute(ck[0], bq[0]);
    }
    // entries left over after the last full chunk: one at a time, the segment always in bcur
    for (int32_t e = beg + nch * J; e < end; ++e) {
        const uint32_t ct = ctl[e];
        const float a = values[e];
        if (!REUSE || (ct & kHeadBit)) load_b<V>(Bl, ldb, cols[e], bcur);
        item_plain<P, V>(acc, ct, a, bcur);
    }

    // epilogue: each lane stores its V adjacent columns of every row of the group (coalesced
    // along N); rows beyond m (last group) and lanes beyond N are skipped.
    if (in) {
        const int64_t row0 = q * p;
        float* __restrict__ Cl = C + j0;
#pragma unroll
        for (int r = 0; r < P; ++r) {
            if (r < p && row0 + r < m) {
                float* dst = Cl + (row0 + r) * ldc;
                if constexpr (V == 4) {
                    f32x4 o = {acc_get(acc, acc_slot<P, V>(0, r)), acc_get(acc, acc_slot<P, V>(1, r)),
                               acc_get(acc, acc_slot<P, V>(2, r)), acc_get(acc, acc_slot<P, V>(3, r))};
                    *reinterpret_cast<f32x4*>(dst) = o;
                } else if constexpr (V == 2) {
                    f32x2 o = {acc_get(acc, acc_slot<P, V>(0, r)), acc_get(acc, acc_slot<P, V>(1, r))};
                    *reinterpret_cast<f32x2*>(dst) = o;
                } else {
                    *dst = acc_get(acc, acc_slot<P, V>(0, r));
                }
            }
        }
    }
}

template <int P, int V, bool REUSE>
hipError_t launch_spdm_reg_instance(const SpdmArgs& a, hipStream_t s)
{
    constexpr int J = 8;
    const int64_t tiles = (a.N + 64 * V - 1) / (64 * V);
    const int64_t total = a.g * tiles;
    const int64_t grid = (total + 7) / 8 * 8;          // whole rounds over the 8 XCDs
    if (grid <= 0 || grid > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    if (a.ldb > 0x3fffffffLL) return hipErrorInvalidValue;   // row pitch in bytes is kept in 32 bits
    spdm_reg<P, V, J, REUSE><<<dim3((unsigned)grid), dim3(64), 0, s>>>(a.values, a.cols, a.ctl, a.gIdxes, a.m, a.p, a.g, a.B,
                                                                     a.ldb, a.N, a.C, a.ldc, total);
    return hipGetLastError();
}

}  // namespace gcoo
