// Stand-alone micro-benchmarks behind the ceilings that the design notes quote for the SpDM kernels on MI355X.
// They measure what the machine delivers for the three things the kernels do per entry and per band, with
// nothing else in the way:
//   1. lds      ds_read_b128 bandwidth of a compute unit (the B values of the workgroup-shared kernel come from LDS)
//   2. issue    the workgroup-shared kernel's own instruction sequence for a block of 16 singles / 4 quads
//               (the macros of gcoo_spdm_share_kernel.hpp, so it is the same text), looped with no band
//               bookkeeping, no fills and no barrier: the rate at which a compute unit issues it
//   3. fill     48-row bands of a B tile fetched straight to LDS by eight waves, three buffers, one barrier per
//               band with the loads of the band after next still in flight: the kernel's fetch pattern alone
//   4. sweep    the register kernel's fetch pattern alone: every wave walks the rows of its B tile in ascending
//               order and loads a random share of them, 1 KB per row, four loads per step, three steps in flight
// Each line gives the time that the headline workload (8000 x 8000, 0.5 % density, N = 8000: 10.24 M entries x
// column tiles) would need at the measured rate.
// Build and run: python -m paper_2005_14469_amd.microbench
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <vector>

#include "gcoo_spdm_share_kernel.hpp"

#define CK(x)                                                                          \
    do {                                                                               \
        hipError_t e_ = (x);                                                           \
        if (e_ != hipSuccess) {                                                        \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);      \
            exit(1);                                                                   \
        }                                                                              \
    } while (0)

typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr double kEntryTiles = 320000.0 * 32.0;      // headline workload: entries x column tiles of 256
constexpr int kCUs = 256;

// ---------------------------------------------------------------- 1. LDS read bandwidth
__global__ __launch_bounds__(512) void lds_read(int iters, unsigned* sink)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int lane = threadIdx.x & 63;
    for (int i = threadIdx.x; i < 32768; i += 512) lds[i] = (float)i;
    __syncthreads();
    const unsigned base = lane * 16 + ((threadIdx.x >> 6) * 7 % 16) * 4096;
    unsigned acc = 0;
    for (int it = 0; it < iters; ++it) {
        f32x4 r0, r1, r2, r3, r4, r5, r6, r7;
        const unsigned a = (base + (it * 37 % 13) * 8192u) % 122880u;      // + 7168 + 16 stays below 131072
        asm volatile("ds_read_b128 %0, %8\n\tds_read_b128 %1, %8 offset:1024\n\tds_read_b128 %2, %8 offset:3072\n\t"
                     "ds_read_b128 %3, %8 offset:2048\n\tds_read_b128 %4, %8 offset:5120\n\tds_read_b128 %5, %8 offset:4096\n\t"
                     "ds_read_b128 %6, %8 offset:7168\n\tds_read_b128 %7, %8 offset:6144\n\ts_waitcnt lgkmcnt(0)"
                     : "=&v"(r0), "=&v"(r1), "=&v"(r2), "=&v"(r3), "=&v"(r4), "=&v"(r5), "=&v"(r6), "=&v"(r7)
                     : "v"(a));
        acc += __float_as_uint(r0.x) ^ __float_as_uint(r7.x);
    }
    if (acc == 0x12345u) sink[0] = acc;
}

// ---------------------------------------------------------------- 2. issue rate of the per-entry sequence
// MODE 0: sixteen singles (SH_GROUP x 4), 1: four quads, 2: the multiply-adds of sixteen entries with their
// index-mode switches and nothing else, 3: 64 plain v_fmac_f32 (no index mode, no LDS), 4: sixteen singles the
// way the kernel did them before (four sets of B values, a wait before every entry)
template <int MODE>
__global__ __launch_bounds__(512) void issue(int iters, float* out)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int lane = threadIdx.x & 63;
    for (int i = threadIdx.x; i < 3 * 12288; i += 512) lds[i] = 1.0f + (float)(i & 7);
    __syncthreads();
    gcoo::ShareAcc acc;
    acc.t0 = 0.0f; acc.t1 = 0.0f; acc.t2 = 0.0f; acc.t3 = 0.0f; acc.t4 = 0.0f; acc.t5 = 0.0f; acc.t6 = 0.0f;
    const unsigned rec = lane & 15;
    const float value = 0.5f;
    // rows of the four records of a group of four, one byte each (all below 48); slot of the record's B row
    const unsigned g4 = rec & ~3u;
    const unsigned rows = ((g4 * 3) % 48) | (((g4 * 3 + 7) % 48) << 8) | (((g4 * 3 + 19) % 48) << 16) | (((g4 * 3 + 31) % 48) << 24);
    const unsigned off = ((rec * 11) % 48) * 1024u;
    const unsigned l16 = lane * 16u;
    if constexpr (MODE == 0) {
        // the kernel's own macros: eight sets of B values, the reads of a group of four issued a whole group ahead
        asm volatile(
            "v_mov_b32 v40, %[val]\n\t"
            "v_mov_b32 v41, %[rows]\n\t"
            "v_mov_b32 v42, %[off]\n\t"
            "v_mov_b32 v46, %[off]\n\t"
            "v_mov_b32 v48, %[l16]\n\t"
            "s_mov_b32 s74, %[iters]\n\t"
            SH_ADDR(v36, v42, 0) SH_ADDR(v37, v42, 1) SH_ADDR(v38, v42, 2) SH_ADDR(v39, v42, 3)
            SH_READ_SET0 SH_READ_SET1 SH_READ_SET2 SH_READ_SET3
            ".Lq_loop_%=:\n\t"
            "s_mov_b32 s73, 1000\n\t"
            SH_ROWS(s70, 0)
            SH_GROUP(v42, 4, 5, 6, 7, SH_READ_SET4, SH_READ_SET5, SH_READ_SET6, SH_READ_SET7, SH_ROWS(s86, 4),
                     SH_FMAC_SET0(0, s70), SH_FMAC_SET1(1, s70), SH_FMAC_SET2(2, s70), SH_FMACL_SET3(3, s70))
            SH_GROUP(v42, 8, 9, 10, 11, SH_READ_SET0, SH_READ_SET1, SH_READ_SET2, SH_READ_SET3, SH_ROWS(s70, 8),
                     SH_FMAC_SET4(4, s86), SH_FMAC_SET5(5, s86), SH_FMAC_SET6(6, s86), SH_FMACL_SET7(7, s86))
            SH_GROUP(v42, 12, 13, 14, 15, SH_READ_SET4, SH_READ_SET5, SH_READ_SET6, SH_READ_SET7, SH_ROWS(s86, 12),
                     SH_FMAC_SET0(8, s70), SH_FMAC_SET1(9, s70), SH_FMAC_SET2(10, s70), SH_FMACL_SET3(11, s70))
            SH_GROUP(v46, 0, 1, 2, 3, SH_READ_SET0, SH_READ_SET1, SH_READ_SET2, SH_READ_SET3, "",
                     SH_FMAC_SET4(12, s86), SH_FMAC_SET5(13, s86), SH_FMAC_SET6(14, s86), SH_FMACL_SET7(15, s86))
            "s_sub_u32 s74, s74, 1\n\t"
            "s_cmp_lg_u32 s74, 0\n\t"
            "s_cbranch_scc1 .Lq_loop_%=\n"
            ".Lsh_send_%=:\n\t"
            "s_waitcnt lgkmcnt(0)\n\t"
            : "+{v[60:63]}"(acc.t0), "+{v[64:95]}"(acc.t1), "+{v[96:127]}"(acc.t2), "+{v[128:159]}"(acc.t3),
              "+{v[160:191]}"(acc.t4), "+{v[192:223]}"(acc.t5), "+{v[224:255]}"(acc.t6)
            : [iters] "s"(iters), [val] "v"(value), [rows] "v"(rows), [off] "v"(off), [l16] "v"(l16)
            : "m0", "scc", "memory", "v4", "v5", "v6", "v7", "v8", "v9", "v10", "v11", "v12", "v13", "v14", "v15", "v16", "v17", "v18", "v19",
              "v20", "v21", "v22", "v23", "v24", "v25", "v26", "v27", "v28", "v29", "v30", "v31", "v32", "v33",
              "v34", "v35", "v36", "v37", "v38", "v39", "v40", "v41", "v42", "v46", "v48", "s70", "s73", "s74", "s86");
    } else if constexpr (MODE == 1) {
        asm volatile(
            "v_mov_b32 v40, %[val]\n\t"
            "v_mov_b32 v41, %[rows]\n\t"
            "v_mov_b32 v42, %[off]\n\t"
            "v_mov_b32 v46, %[off]\n\t"
            "v_mov_b32 v48, %[l16]\n\t"
            "s_mov_b32 s74, %[iters]\n"
            ".Lq_loop_%=:\n\t"
            SH_ROWS(s70, 0)
            SH_ROWS(s86, 4)
            SH_ADDR(v36, v42, 0) SH_ADDR(v37, v42, 4) SH_ADDR(v38, v42, 8) SH_ADDR(v39, v42, 12)
            SH_READ_SET0 SH_READ_SET1 SH_READ_SET2 SH_READ_SET3
            SH_WAIT3
            SH_FMAC_SET0(0, s70) SH_FMAC_SET0(1, s70) SH_FMAC_SET0(2, s70) SH_FMACL_SET0(3, s70)
            SH_OFF
            SH_ROWS(s70, 8)
            "s_waitcnt lgkmcnt(2)\n\t"
            SH_FMAC_SET1(4, s86) SH_FMAC_SET1(5, s86) SH_FMAC_SET1(6, s86) SH_FMACL_SET1(7, s86)
            SH_OFF
            SH_ROWS(s86, 12)
            "s_waitcnt lgkmcnt(1)\n\t"
            SH_FMAC_SET2(8, s70) SH_FMAC_SET2(9, s70) SH_FMAC_SET2(10, s70) SH_FMACL_SET2(11, s70)
            SH_OFF
            "s_waitcnt lgkmcnt(0)\n\t"
            SH_FMAC_SET3(12, s86) SH_FMAC_SET3(13, s86) SH_FMAC_SET3(14, s86) SH_FMACL_SET3(15, s86)
            SH_OFF
            "s_sub_u32 s74, s74, 1\n\t"
            "s_cmp_lg_u32 s74, 0\n\t"
            "s_cbranch_scc1 .Lq_loop_%=\n\t"
            : "+{v[60:63]}"(acc.t0), "+{v[64:95]}"(acc.t1), "+{v[96:127]}"(acc.t2), "+{v[128:159]}"(acc.t3),
              "+{v[160:191]}"(acc.t4), "+{v[192:223]}"(acc.t5), "+{v[224:255]}"(acc.t6)
            : [iters] "s"(iters), [val] "v"(value), [rows] "v"(rows), [off] "v"(off), [l16] "v"(l16)
            : "m0", "scc", "memory", "v20", "v21", "v22", "v23", "v24", "v25", "v26", "v27", "v28", "v29", "v30", "v31", "v32", "v33",
              "v34", "v35", "v36", "v37", "v38", "v39", "v40", "v41", "v42", "v46", "v48", "s70", "s73", "s74", "s86");
    } else if constexpr (MODE == 4) {
        // the sequence the kernel used before: four sets of B values, each read issued right after the multiply-adds
        // that free its set (three entries ahead), a wait before every entry
#define OLD_GROUP(src, n0, n1, n2, n3, nextrows, i0, i1, i2, i3, rows)                    \
            "s_sub_u32 s73, s73, 1\n\t"                                               \
            "s_cbranch_scc1 .Lsh_send_%=\n\t"                                         \
            SH_ADDR(v36, src, n0) SH_ADDR(v37, src, n1) SH_ADDR(v38, src, n2) SH_ADDR(v39, src, n3) \
            nextrows                                                                  \
            SH_WAIT3 SH_FMAC_SET0(i0, rows) SH_READ_SET0                              \
            SH_WAIT3 SH_FMAC_SET1(i1, rows) SH_READ_SET1                              \
            SH_WAIT3 SH_FMAC_SET2(i2, rows) SH_READ_SET2                              \
            SH_WAIT3 SH_FMAC_SET3(i3, rows) SH_READ_SET3                              \
            SH_OFF
        asm volatile(
            "v_mov_b32 v40, %[val]\n\t"
            "v_mov_b32 v41, %[rows]\n\t"
            "v_mov_b32 v42, %[off]\n\t"
            "v_mov_b32 v46, %[off]\n\t"
            "v_mov_b32 v48, %[l16]\n\t"
            "s_mov_b32 s74, %[iters]\n"
            ".Lq_loop_%=:\n\t"
            "s_mov_b32 s73, 1000\n\t"
            SH_ROWS(s70, 0)
            SH_ADDR(v36, v42, 0) SH_ADDR(v37, v42, 1) SH_ADDR(v38, v42, 2) SH_ADDR(v39, v42, 3)
            SH_READ_SET0 SH_READ_SET1 SH_READ_SET2 SH_READ_SET3
            OLD_GROUP(v42, 4, 5, 6, 7, SH_ROWS(s86, 4), 0, 1, 2, 3, s70)
            OLD_GROUP(v42, 8, 9, 10, 11, SH_ROWS(s70, 8), 4, 5, 6, 7, s86)
            OLD_GROUP(v42, 12, 13, 14, 15, SH_ROWS(s86, 12), 8, 9, 10, 11, s70)
            OLD_GROUP(v46, 0, 1, 2, 3, "", 12, 13, 14, 15, s86)
            "s_waitcnt lgkmcnt(0)\n\t"
            "s_sub_u32 s74, s74, 1\n\t"
            "s_cmp_lg_u32 s74, 0\n\t"
            "s_cbranch_scc1 .Lq_loop_%=\n"
            ".Lsh_send_%=:\n\t"
            "s_waitcnt lgkmcnt(0)\n\t"
            : "+{v[60:63]}"(acc.t0), "+{v[64:95]}"(acc.t1), "+{v[96:127]}"(acc.t2), "+{v[128:159]}"(acc.t3),
              "+{v[160:191]}"(acc.t4), "+{v[192:223]}"(acc.t5), "+{v[224:255]}"(acc.t6)
            : [iters] "s"(iters), [val] "v"(value), [rows] "v"(rows), [off] "v"(off), [l16] "v"(l16)
            : "m0", "scc", "memory", "v20", "v21", "v22", "v23", "v24", "v25", "v26", "v27", "v28", "v29", "v30", "v31", "v32", "v33",
              "v34", "v35", "v36", "v37", "v38", "v39", "v40", "v41", "v42", "v46", "v48", "s70", "s73", "s74", "s86");
#undef OLD_GROUP
    } else if constexpr (MODE == 2) {
        asm volatile(
            "v_mov_b32 v40, %[val]\n\t"
            "v_mov_b32 v41, %[rows]\n\t"
            "v_mov_b32 v42, %[off]\n\t"
            "v_mov_b32 v46, %[off]\n\t"
            "v_mov_b32 v48, %[l16]\n\t"
            "v_mov_b32 v20, 1.0\n\tv_mov_b32 v21, 1.0\n\tv_mov_b32 v22, 1.0\n\tv_mov_b32 v23, 1.0\n\t"
            "s_mov_b32 s74, %[iters]\n"
            ".Lq_loop_%=:\n\t"
            SH_ROWS(s70, 0)
            SH_FMAC_SET0(0, s70) SH_FMAC_SET0(1, s70) SH_FMAC_SET0(2, s70) SH_FMAC_SET0(3, s70)
            SH_OFF
            SH_ROWS(s70, 4)
            SH_FMAC_SET0(4, s70) SH_FMAC_SET0(5, s70) SH_FMAC_SET0(6, s70) SH_FMAC_SET0(7, s70)
            SH_OFF
            SH_ROWS(s70, 8)
            SH_FMAC_SET0(8, s70) SH_FMAC_SET0(9, s70) SH_FMAC_SET0(10, s70) SH_FMAC_SET0(11, s70)
            SH_OFF
            SH_ROWS(s70, 12)
            SH_FMAC_SET0(12, s70) SH_FMAC_SET0(13, s70) SH_FMAC_SET0(14, s70) SH_FMAC_SET0(15, s70)
            SH_OFF
            "s_sub_u32 s74, s74, 1\n\t"
            "s_cmp_lg_u32 s74, 0\n\t"
            "s_cbranch_scc1 .Lq_loop_%=\n\t"
            : "+{v[60:63]}"(acc.t0), "+{v[64:95]}"(acc.t1), "+{v[96:127]}"(acc.t2), "+{v[128:159]}"(acc.t3),
              "+{v[160:191]}"(acc.t4), "+{v[192:223]}"(acc.t5), "+{v[224:255]}"(acc.t6)
            : [iters] "s"(iters), [val] "v"(value), [rows] "v"(rows), [off] "v"(off), [l16] "v"(l16)
            : "m0", "scc", "memory", "v20", "v21", "v22", "v23", "v40", "v41", "v42", "v46", "v48", "s70", "s73", "s74", "s86");
    } else {
        asm volatile(
            "v_mov_b32 v40, %[val]\n\t"
            "v_mov_b32 v20, 1.0\n\tv_mov_b32 v21, 1.0\n\tv_mov_b32 v22, 1.0\n\tv_mov_b32 v23, 1.0\n\t"
            "s_mov_b32 s74, %[iters]\n"
            ".Lq_loop_%=:\n\t"
            "v_fmac_f32 v60, v40, v20\n\tv_fmac_f32 v109, v40, v21\n\tv_fmac_f32 v158, v40, v22\n\tv_fmac_f32 v207, v40, v23\n\t"
            "v_fmac_f32 v61, v40, v20\n\tv_fmac_f32 v110, v40, v21\n\tv_fmac_f32 v159, v40, v22\n\tv_fmac_f32 v208, v40, v23\n\t"
            "v_fmac_f32 v62, v40, v20\n\tv_fmac_f32 v111, v40, v21\n\tv_fmac_f32 v160, v40, v22\n\tv_fmac_f32 v209, v40, v23\n\t"
            "v_fmac_f32 v63, v40, v20\n\tv_fmac_f32 v112, v40, v21\n\tv_fmac_f32 v161, v40, v22\n\tv_fmac_f32 v210, v40, v23\n\t"
            "v_fmac_f32 v64, v40, v20\n\tv_fmac_f32 v113, v40, v21\n\tv_fmac_f32 v162, v40, v22\n\tv_fmac_f32 v211, v40, v23\n\t"
            "v_fmac_f32 v65, v40, v20\n\tv_fmac_f32 v114, v40, v21\n\tv_fmac_f32 v163, v40, v22\n\tv_fmac_f32 v212, v40, v23\n\t"
            "v_fmac_f32 v66, v40, v20\n\tv_fmac_f32 v115, v40, v21\n\tv_fmac_f32 v164, v40, v22\n\tv_fmac_f32 v213, v40, v23\n\t"
            "v_fmac_f32 v67, v40, v20\n\tv_fmac_f32 v116, v40, v21\n\tv_fmac_f32 v165, v40, v22\n\tv_fmac_f32 v214, v40, v23\n\t"
            "v_fmac_f32 v68, v40, v20\n\tv_fmac_f32 v117, v40, v21\n\tv_fmac_f32 v166, v40, v22\n\tv_fmac_f32 v215, v40, v23\n\t"
            "v_fmac_f32 v69, v40, v20\n\tv_fmac_f32 v118, v40, v21\n\tv_fmac_f32 v167, v40, v22\n\tv_fmac_f32 v216, v40, v23\n\t"
            "v_fmac_f32 v70, v40, v20\n\tv_fmac_f32 v119, v40, v21\n\tv_fmac_f32 v168, v40, v22\n\tv_fmac_f32 v217, v40, v23\n\t"
            "v_fmac_f32 v71, v40, v20\n\tv_fmac_f32 v120, v40, v21\n\tv_fmac_f32 v169, v40, v22\n\tv_fmac_f32 v218, v40, v23\n\t"
            "v_fmac_f32 v72, v40, v20\n\tv_fmac_f32 v121, v40, v21\n\tv_fmac_f32 v170, v40, v22\n\tv_fmac_f32 v219, v40, v23\n\t"
            "v_fmac_f32 v73, v40, v20\n\tv_fmac_f32 v122, v40, v21\n\tv_fmac_f32 v171, v40, v22\n\tv_fmac_f32 v220, v40, v23\n\t"
            "v_fmac_f32 v74, v40, v20\n\tv_fmac_f32 v123, v40, v21\n\tv_fmac_f32 v172, v40, v22\n\tv_fmac_f32 v221, v40, v23\n\t"
            "v_fmac_f32 v75, v40, v20\n\tv_fmac_f32 v124, v40, v21\n\tv_fmac_f32 v173, v40, v22\n\tv_fmac_f32 v222, v40, v23\n\t"
            "s_sub_u32 s74, s74, 1\n\t"
            "s_cmp_lg_u32 s74, 0\n\t"
            "s_cbranch_scc1 .Lq_loop_%=\n\t"
            : "+{v[60:63]}"(acc.t0), "+{v[64:95]}"(acc.t1), "+{v[96:127]}"(acc.t2), "+{v[128:159]}"(acc.t3),
              "+{v[160:191]}"(acc.t4), "+{v[192:223]}"(acc.t5), "+{v[224:255]}"(acc.t6)
            : [iters] "s"(iters), [val] "v"(value)
            : "scc", "memory", "v20", "v21", "v22", "v23", "v40", "s74");
    }
    float s = 0.0f;
    for (int r = 0; r < 4; ++r) s += gcoo::share_acc_get(acc, gcoo::kShareAccFirst + r);
    if (s == 123.456f) out[0] = s;
}

// ---------------------------------------------------------------- 2a. the singles sequence with 128 registers per wave
// The same per-entry instructions as issue<0>, with the partial sums of 20 rows (+ the sink row) x 4 columns in
// v[44:127] and the working registers below them, so that four waves fit a SIMD (workgroups of 8 waves, two per compute
// unit, or one): does the sequence issue faster when a SIMD has four waves to choose from instead of two?
#define S16_DPP(i) " row_newbcast:" #i " row_mask:0xf bank_mask:0xf\n\t"
#define S16_ADDR(dst, src, i) "v_add_u32_dpp " #dst ", " #src ", v28" S16_DPP(i)
#define S16_ROWS(reg, i) "v_readlane_b32 " #reg ", v25, " #i "\n\t"
#define S16_FMAC(i, rows, b0, b1, b2, b3)                   \
    "s_set_gpr_idx_on " #rows ", gpr_idx(SRC2,DST)\n\t"      \
    "v_fmac_f32_dpp v44, v24, " #b0 S16_DPP(i)               \
    "v_fmac_f32_dpp v65, v24, " #b1 S16_DPP(i)               \
    "v_fmac_f32_dpp v86, v24, " #b2 S16_DPP(i)               \
    "v_fmac_f32_dpp v107, v24, " #b3 S16_DPP(i)              \
    "s_lshr_b32 " #rows ", " #rows ", 8\n\t"
#define S16_STEP(i, rows, set, b0, b1, b2, b3, ad)           \
    "s_waitcnt lgkmcnt(3)\n\t" S16_FMAC(i, rows, b0, b1, b2, b3) "ds_read_b128 v[" #b0 ":" #b3 "], " #ad "\n\t"
#define S16_GROUP(src, n0, n1, n2, n3, nextrows, i0, i1, i2, i3, rows)                                        \
    S16_ADDR(v20, src, n0) S16_ADDR(v21, src, n1) S16_ADDR(v22, src, n2) S16_ADDR(v23, src, n3) nextrows      \
    "s_waitcnt lgkmcnt(3)\n\t" S16_FMAC(i0, rows, v4, v5, v6, v7) "ds_read_b128 v[4:7], v20\n\t"             \
    "s_waitcnt lgkmcnt(3)\n\t" S16_FMAC(i1, rows, v8, v9, v10, v11) "ds_read_b128 v[8:11], v21\n\t"          \
    "s_waitcnt lgkmcnt(3)\n\t" S16_FMAC(i2, rows, v12, v13, v14, v15) "ds_read_b128 v[12:15], v22\n\t"       \
    "s_waitcnt lgkmcnt(3)\n\t" S16_FMAC(i3, rows, v16, v17, v18, v19) "ds_read_b128 v[16:19], v23\n\t"       \
    "s_set_gpr_idx_off\n\t"
__global__ __launch_bounds__(512) void issue128(int iters, float* out)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int lane = threadIdx.x & 63;
    for (int i = threadIdx.x; i < 12288; i += 512) lds[i] = 1.0f + (float)(i & 7);
    __syncthreads();
    const unsigned rec = lane & 15;
    const float value = 0.5f;
    const unsigned g4 = rec & ~3u;
    const unsigned rows = ((g4 * 3) % 20) | (((g4 * 3 + 7) % 20) << 8) | (((g4 * 3 + 11) % 20) << 16) | (((g4 * 3 + 17) % 20) << 24);
    const unsigned off = ((rec * 11) % 48) * 1024u;
    const unsigned l16 = lane * 16u;
    float r = 0.0f;
    asm volatile(
        "v_mov_b32 v24, %[val]\n\t"
        "v_mov_b32 v25, %[rows]\n\t"
        "v_mov_b32 v26, %[off]\n\t"
        "v_mov_b32 v27, %[off]\n\t"
        "v_mov_b32 v28, %[l16]\n\t"
        "s_mov_b32 s74, %[iters]\n"
        ".Lq_loop_%=:\n\t"
        S16_ROWS(s70, 0)
        S16_ADDR(v20, v26, 0) S16_ADDR(v21, v26, 1) S16_ADDR(v22, v26, 2) S16_ADDR(v23, v26, 3)
        "ds_read_b128 v[4:7], v20\n\tds_read_b128 v[8:11], v21\n\tds_read_b128 v[12:15], v22\n\tds_read_b128 v[16:19], v23\n\t"
        "s_sub_u32 s73, s73, 1\n\ts_nop 0\n\t"
        S16_GROUP(v26, 4, 5, 6, 7, S16_ROWS(s86, 4), 0, 1, 2, 3, s70)
        "s_sub_u32 s73, s73, 1\n\ts_nop 0\n\t"
        S16_GROUP(v26, 8, 9, 10, 11, S16_ROWS(s70, 8), 4, 5, 6, 7, s86)
        "s_sub_u32 s73, s73, 1\n\ts_nop 0\n\t"
        S16_GROUP(v26, 12, 13, 14, 15, S16_ROWS(s86, 12), 8, 9, 10, 11, s70)
        "s_sub_u32 s73, s73, 1\n\ts_nop 0\n\t"
        S16_GROUP(v27, 0, 1, 2, 3, "", 12, 13, 14, 15, s86)
        "s_waitcnt lgkmcnt(0)\n\t"
        "s_sub_u32 s74, s74, 1\n\t"
        "s_cmp_lg_u32 s74, 0\n\t"
        "s_cbranch_scc1 .Lq_loop_%=\n\t"
        "v_mov_b32 %[r], v44\n\t"
        : [r] "=v"(r)
        : [iters] "s"(iters), [val] "v"(value), [rows] "v"(rows), [off] "v"(off), [l16] "v"(l16)
        : "m0", "scc", "memory", "s70", "s73", "s74", "s86", "v4", "v5", "v6", "v7", "v8", "v9", "v10", "v11", "v12", "v13", "v14", "v15", "v16", "v17", "v18", "v19", "v20", "v21", "v22", "v23", "v24", "v25", "v26", "v27", "v28", "v29", "v30", "v31", "v32", "v33", "v34", "v35", "v36", "v37", "v38", "v39", "v40", "v41", "v42", "v43", "v44", "v45", "v46", "v47", "v48", "v49", "v50", "v51", "v52", "v53", "v54", "v55", "v56", "v57", "v58", "v59", "v60", "v61", "v62", "v63", "v64", "v65", "v66", "v67", "v68", "v69", "v70", "v71", "v72", "v73", "v74", "v75", "v76", "v77", "v78", "v79", "v80", "v81", "v82", "v83", "v84", "v85", "v86", "v87", "v88", "v89", "v90", "v91", "v92", "v93", "v94", "v95", "v96", "v97", "v98", "v99", "v100", "v101", "v102", "v103", "v104", "v105", "v106", "v107", "v108", "v109", "v110", "v111", "v112", "v113", "v114", "v115", "v116", "v117", "v118", "v119", "v120", "v121", "v122", "v123", "v124", "v125", "v126", "v127");
    if (r == 123.456f) out[0] = r;
}

#define VALU_BODY_0 \
        "v_fmac_f32 v8, v5, v2\n\tv_fmac_f32 v9, v6, v3\n\tv_fmac_f32 v10, v7, v0\n\tv_fmac_f32 v11, v4, v1\n\t" \
        "v_fmac_f32 v12, v5, v2\n\tv_fmac_f32 v13, v6, v3\n\tv_fmac_f32 v14, v7, v0\n\tv_fmac_f32 v15, v4, v1\n\t" \
        "v_fmac_f32 v16, v5, v2\n\tv_fmac_f32 v17, v6, v3\n\tv_fmac_f32 v18, v7, v0\n\tv_fmac_f32 v19, v4, v1\n\t" \
        "v_fmac_f32 v20, v5, v2\n\tv_fmac_f32 v21, v6, v3\n\tv_fmac_f32 v22, v7, v0\n\tv_fmac_f32 v23, v4, v1\n\t" \
        "v_fmac_f32 v24, v5, v2\n\tv_fmac_f32 v25, v6, v3\n\tv_fmac_f32 v26, v7, v0\n\tv_fmac_f32 v27, v4, v1\n\t" \
        "v_fmac_f32 v28, v5, v2\n\tv_fmac_f32 v29, v6, v3\n\tv_fmac_f32 v30, v7, v0\n\tv_fmac_f32 v31, v4, v1\n\t" \
        "v_fmac_f32 v32, v5, v2\n\tv_fmac_f32 v33, v6, v3\n\tv_fmac_f32 v34, v7, v0\n\tv_fmac_f32 v35, v4, v1\n\t" \
        "v_fmac_f32 v36, v5, v2\n\tv_fmac_f32 v37, v6, v3\n\tv_fmac_f32 v38, v7, v0\n\tv_fmac_f32 v39, v4, v1\n\t" \
        "v_fmac_f32 v40, v5, v2\n\tv_fmac_f32 v41, v6, v3\n\tv_fmac_f32 v42, v7, v0\n\tv_fmac_f32 v43, v4, v1\n\t" \
        "v_fmac_f32 v44, v5, v2\n\tv_fmac_f32 v45, v6, v3\n\tv_fmac_f32 v46, v7, v0\n\tv_fmac_f32 v47, v4, v1\n\t" \
        "v_fmac_f32 v48, v5, v2\n\tv_fmac_f32 v49, v6, v3\n\tv_fmac_f32 v50, v7, v0\n\tv_fmac_f32 v51, v4, v1\n\t" \
        "v_fmac_f32 v52, v5, v2\n\tv_fmac_f32 v53, v6, v3\n\tv_fmac_f32 v54, v7, v0\n\tv_fmac_f32 v55, v4, v1\n\t" \
        "v_fmac_f32 v56, v5, v2\n\tv_fmac_f32 v57, v6, v3\n\tv_fmac_f32 v58, v7, v0\n\tv_fmac_f32 v59, v4, v1\n\t" \
        "v_fmac_f32 v60, v5, v2\n\tv_fmac_f32 v61, v6, v3\n\tv_fmac_f32 v62, v7, v0\n\tv_fmac_f32 v63, v4, v1\n\t" \
        "v_fmac_f32 v64, v5, v2\n\tv_fmac_f32 v65, v6, v3\n\tv_fmac_f32 v66, v7, v0\n\tv_fmac_f32 v67, v4, v1\n\t" \
        "v_fmac_f32 v68, v5, v2\n\tv_fmac_f32 v69, v6, v3\n\tv_fmac_f32 v70, v7, v0\n\tv_fmac_f32 v71, v4, v1\n\t"
#define VALU_BODY_1 \
        "v_fmac_f32 v8, v4, v0\n\tv_fmac_f32 v9, v5, v1\n\tv_fmac_f32 v10, v6, v2\n\tv_fmac_f32 v11, v7, v3\n\t" \
        "v_fmac_f32 v12, v4, v0\n\tv_fmac_f32 v13, v5, v1\n\tv_fmac_f32 v14, v6, v2\n\tv_fmac_f32 v15, v7, v3\n\t" \
        "v_fmac_f32 v16, v4, v0\n\tv_fmac_f32 v17, v5, v1\n\tv_fmac_f32 v18, v6, v2\n\tv_fmac_f32 v19, v7, v3\n\t" \
        "v_fmac_f32 v20, v4, v0\n\tv_fmac_f32 v21, v5, v1\n\tv_fmac_f32 v22, v6, v2\n\tv_fmac_f32 v23, v7, v3\n\t" \
        "v_fmac_f32 v24, v4, v0\n\tv_fmac_f32 v25, v5, v1\n\tv_fmac_f32 v26, v6, v2\n\tv_fmac_f32 v27, v7, v3\n\t" \
        "v_fmac_f32 v28, v4, v0\n\tv_fmac_f32 v29, v5, v1\n\tv_fmac_f32 v30, v6, v2\n\tv_fmac_f32 v31, v7, v3\n\t" \
        "v_fmac_f32 v32, v4, v0\n\tv_fmac_f32 v33, v5, v1\n\tv_fmac_f32 v34, v6, v2\n\tv_fmac_f32 v35, v7, v3\n\t" \
        "v_fmac_f32 v36, v4, v0\n\tv_fmac_f32 v37, v5, v1\n\tv_fmac_f32 v38, v6, v2\n\tv_fmac_f32 v39, v7, v3\n\t" \
        "v_fmac_f32 v40, v4, v0\n\tv_fmac_f32 v41, v5, v1\n\tv_fmac_f32 v42, v6, v2\n\tv_fmac_f32 v43, v7, v3\n\t" \
        "v_fmac_f32 v44, v4, v0\n\tv_fmac_f32 v45, v5, v1\n\tv_fmac_f32 v46, v6, v2\n\tv_fmac_f32 v47, v7, v3\n\t" \
        "v_fmac_f32 v48, v4, v0\n\tv_fmac_f32 v49, v5, v1\n\tv_fmac_f32 v50, v6, v2\n\tv_fmac_f32 v51, v7, v3\n\t" \
        "v_fmac_f32 v52, v4, v0\n\tv_fmac_f32 v53, v5, v1\n\tv_fmac_f32 v54, v6, v2\n\tv_fmac_f32 v55, v7, v3\n\t" \
        "v_fmac_f32 v56, v4, v0\n\tv_fmac_f32 v57, v5, v1\n\tv_fmac_f32 v58, v6, v2\n\tv_fmac_f32 v59, v7, v3\n\t" \
        "v_fmac_f32 v60, v4, v0\n\tv_fmac_f32 v61, v5, v1\n\tv_fmac_f32 v62, v6, v2\n\tv_fmac_f32 v63, v7, v3\n\t" \
        "v_fmac_f32 v64, v4, v0\n\tv_fmac_f32 v65, v5, v1\n\tv_fmac_f32 v66, v6, v2\n\tv_fmac_f32 v67, v7, v3\n\t" \
        "v_fmac_f32 v68, v4, v0\n\tv_fmac_f32 v69, v5, v1\n\tv_fmac_f32 v70, v6, v2\n\tv_fmac_f32 v71, v7, v3\n\t"
#define VALU_BODY_2 \
        "v_fmac_f32 v8, v5, v1\n\tv_fmac_f32 v9, v6, v2\n\tv_fmac_f32 v10, v7, v3\n\tv_fmac_f32 v11, v4, v0\n\t" \
        "v_fmac_f32 v12, v5, v1\n\tv_fmac_f32 v13, v6, v2\n\tv_fmac_f32 v14, v7, v3\n\tv_fmac_f32 v15, v4, v0\n\t" \
        "v_fmac_f32 v16, v5, v1\n\tv_fmac_f32 v17, v6, v2\n\tv_fmac_f32 v18, v7, v3\n\tv_fmac_f32 v19, v4, v0\n\t" \
        "v_fmac_f32 v20, v5, v1\n\tv_fmac_f32 v21, v6, v2\n\tv_fmac_f32 v22, v7, v3\n\tv_fmac_f32 v23, v4, v0\n\t" \
        "v_fmac_f32 v24, v5, v1\n\tv_fmac_f32 v25, v6, v2\n\tv_fmac_f32 v26, v7, v3\n\tv_fmac_f32 v27, v4, v0\n\t" \
        "v_fmac_f32 v28, v5, v1\n\tv_fmac_f32 v29, v6, v2\n\tv_fmac_f32 v30, v7, v3\n\tv_fmac_f32 v31, v4, v0\n\t" \
        "v_fmac_f32 v32, v5, v1\n\tv_fmac_f32 v33, v6, v2\n\tv_fmac_f32 v34, v7, v3\n\tv_fmac_f32 v35, v4, v0\n\t" \
        "v_fmac_f32 v36, v5, v1\n\tv_fmac_f32 v37, v6, v2\n\tv_fmac_f32 v38, v7, v3\n\tv_fmac_f32 v39, v4, v0\n\t" \
        "v_fmac_f32 v40, v5, v1\n\tv_fmac_f32 v41, v6, v2\n\tv_fmac_f32 v42, v7, v3\n\tv_fmac_f32 v43, v4, v0\n\t" \
        "v_fmac_f32 v44, v5, v1\n\tv_fmac_f32 v45, v6, v2\n\tv_fmac_f32 v46, v7, v3\n\tv_fmac_f32 v47, v4, v0\n\t" \
        "v_fmac_f32 v48, v5, v1\n\tv_fmac_f32 v49, v6, v2\n\tv_fmac_f32 v50, v7, v3\n\tv_fmac_f32 v51, v4, v0\n\t" \
        "v_fmac_f32 v52, v5, v1\n\tv_fmac_f32 v53, v6, v2\n\tv_fmac_f32 v54, v7, v3\n\tv_fmac_f32 v55, v4, v0\n\t" \
        "v_fmac_f32 v56, v5, v1\n\tv_fmac_f32 v57, v6, v2\n\tv_fmac_f32 v58, v7, v3\n\tv_fmac_f32 v59, v4, v0\n\t" \
        "v_fmac_f32 v60, v5, v1\n\tv_fmac_f32 v61, v6, v2\n\tv_fmac_f32 v62, v7, v3\n\tv_fmac_f32 v63, v4, v0\n\t" \
        "v_fmac_f32 v64, v5, v1\n\tv_fmac_f32 v65, v6, v2\n\tv_fmac_f32 v66, v7, v3\n\tv_fmac_f32 v67, v4, v0\n\t" \
        "v_fmac_f32 v68, v5, v1\n\tv_fmac_f32 v69, v6, v2\n\tv_fmac_f32 v70, v7, v3\n\tv_fmac_f32 v71, v4, v0\n\t"
// ---------------------------------------------------------------- 2b. VALU issue rate against waves per SIMD and register banks
// 64 independent v_fmac_f32 per turn in 72 registers; workgroups of four waves (one per SIMD), W of them per compute
// unit (the launch asks for 1/W of the LDS), so W waves share a SIMD.  The vector registers sit in four banks
// (register number mod 4).  KIND 0: the three operands of every instruction in three banks; 1: all in one bank;
// 2: the two sources in one bank, the destination in another.
#define VALU_KERNEL(KIND)                                                                                       \
    __global__ __launch_bounds__(256) void valu##KIND(int iters, float* out)                                    \
    {                                                                                                           \
        float r = 0.0f;                                                                                         \
        asm volatile(                                                                                           \
            "v_mov_b32 v0, 1.0\n\tv_mov_b32 v1, 1.0\n\tv_mov_b32 v2, 1.0\n\tv_mov_b32 v3, 1.0\n\t"                   \
            "v_mov_b32 v4, 0.5\n\tv_mov_b32 v5, 0.5\n\tv_mov_b32 v6, 0.5\n\tv_mov_b32 v7, 0.5\n\t"                   \
            "s_mov_b32 s20, %[iters]\n"                                                                         \
            ".Lv_loop_%=:\n\t" VALU_BODY_##KIND                                                                 \
            "s_sub_u32 s20, s20, 1\n\t"                                                                         \
            "s_cmp_lg_u32 s20, 0\n\t"                                                                           \
            "s_cbranch_scc1 .Lv_loop_%=\n\t"                                                                    \
            "v_mov_b32 %[r], v8\n\t"                                                                            \
            : [r] "=v"(r)                                                                                       \
            : [iters] "s"(iters)                                                                                \
            : "scc", "s20", "v0", "v1", "v2", "v3", "v4", "v5", "v6", "v7", "v8", "v9", "v10", "v11", "v12", "v13", "v14", "v15", "v16", "v17", "v18", "v19", "v20", "v21", "v22", "v23", "v24", "v25", "v26", "v27", "v28", "v29", "v30", "v31", "v32", "v33", "v34", "v35", "v36", "v37", "v38", "v39", "v40", "v41", "v42", "v43", "v44", "v45", "v46", "v47", "v48", "v49", "v50", "v51", "v52", "v53", "v54", "v55", "v56", "v57", "v58", "v59", "v60", "v61", "v62", "v63", "v64", "v65", "v66", "v67", "v68", "v69", "v70", "v71");                                                   \
        if (r == 123.456f) out[0] = r;                                                                          \
    }
VALU_KERNEL(0)
VALU_KERNEL(1)
VALU_KERNEL(2)

// ---------------------------------------------------------------- 2c. what scalar instructions and branches cost a wave
// 8 waves per workgroup, one workgroup per compute unit (two waves per SIMD, as in the kernels).  One turn of the
// loop is 16 instructions of one kind: 0 independent s_add_u32; 1 eight compare-and-branch pairs, never taken;
// 2 eight pairs, always taken (to the next instruction); 3 eight pairs of a v_readlane_b32 and a scalar add that
// uses its result; 4 sixteen dependent v_add_u32.
#define REP8(x) x x x x x x x x
template <int KIND>
__global__ __launch_bounds__(512) void scalar_cost(int iters, unsigned* sink)
{
    unsigned v = threadIdx.x, r = 0;
    if constexpr (KIND == 0) {
        asm volatile("s_mov_b32 s74, %[iters]\n"
                     ".Lsc_loop_%=:\n\t"
                     REP8("s_add_u32 s70, s70, 1\n\ts_add_u32 s71, s71, 3\n\t")
                     "s_sub_u32 s74, s74, 1\n\ts_cmp_lg_u32 s74, 0\n\ts_cbranch_scc1 .Lsc_loop_%=\n\t"
                     "v_mov_b32 %[r], s70\n\t"
                     : [r] "=v"(r) : [iters] "s"(iters) : "scc", "s70", "s71", "s74");
    } else if constexpr (KIND == 1) {
        asm volatile("s_mov_b32 s74, %[iters]\n\ts_mov_b32 s70, 0\n"
                     ".Lsc_loop_%=:\n\t"
                     REP8("s_cmp_eq_u32 s70, 12345\n\ts_cbranch_scc1 .Lsc_out_%=\n\t")
                     "s_sub_u32 s74, s74, 1\n\ts_cmp_lg_u32 s74, 0\n\ts_cbranch_scc1 .Lsc_loop_%=\n"
                     ".Lsc_out_%=:\n\t"
                     "v_mov_b32 %[r], s70\n\t"
                     : [r] "=v"(r) : [iters] "s"(iters) : "scc", "s70", "s71", "s74");
    } else if constexpr (KIND == 2) {
        asm volatile("s_mov_b32 s74, %[iters]\n\ts_mov_b32 s70, 0\n"
                     ".Lsc_loop_%=:\n\t"
                     "s_cmp_eq_u32 s70, 0\n\ts_cbranch_scc1 .Lsc_a_%=\n.Lsc_a_%=:\n\t"
                     "s_cmp_eq_u32 s70, 0\n\ts_cbranch_scc1 .Lsc_b_%=\n.Lsc_b_%=:\n\t"
                     "s_cmp_eq_u32 s70, 0\n\ts_cbranch_scc1 .Lsc_c_%=\n.Lsc_c_%=:\n\t"
                     "s_cmp_eq_u32 s70, 0\n\ts_cbranch_scc1 .Lsc_d_%=\n.Lsc_d_%=:\n\t"
                     "s_cmp_eq_u32 s70, 0\n\ts_cbranch_scc1 .Lsc_e_%=\n.Lsc_e_%=:\n\t"
                     "s_cmp_eq_u32 s70, 0\n\ts_cbranch_scc1 .Lsc_f_%=\n.Lsc_f_%=:\n\t"
                     "s_cmp_eq_u32 s70, 0\n\ts_cbranch_scc1 .Lsc_g_%=\n.Lsc_g_%=:\n\t"
                     "s_cmp_eq_u32 s70, 0\n\ts_cbranch_scc1 .Lsc_h_%=\n.Lsc_h_%=:\n\t"
                     "s_sub_u32 s74, s74, 1\n\ts_cmp_lg_u32 s74, 0\n\ts_cbranch_scc1 .Lsc_loop_%=\n\t"
                     "v_mov_b32 %[r], s70\n\t"
                     : [r] "=v"(r) : [iters] "s"(iters) : "scc", "s70", "s71", "s74");
    } else if constexpr (KIND == 3) {
        asm volatile("s_mov_b32 s74, %[iters]\n\ts_mov_b32 s72, 0\n"
                     ".Lsc_loop_%=:\n\t"
                     REP8("v_readlane_b32 s71, %[v], 3\n\ts_add_u32 s72, s72, s71\n\t")
                     "s_sub_u32 s74, s74, 1\n\ts_cmp_lg_u32 s74, 0\n\ts_cbranch_scc1 .Lsc_loop_%=\n\t"
                     "v_mov_b32 %[r], s72\n\t"
                     : [r] "=v"(r) : [iters] "s"(iters), [v] "v"(v) : "scc", "s70", "s71", "s72", "s74");
    } else {
        asm volatile("s_mov_b32 s74, %[iters]\n"
                     ".Lsc_loop_%=:\n\t"
                     REP8("v_add_u32 %[v], 1, %[v]\n\tv_add_u32 %[v], 3, %[v]\n\t")
                     "s_sub_u32 s74, s74, 1\n\ts_cmp_lg_u32 s74, 0\n\ts_cbranch_scc1 .Lsc_loop_%=\n\t"
                     "v_mov_b32 %[r], %[v]\n\t"
                     : [r] "=v"(r), [v] "+v"(v) : [iters] "s"(iters) : "scc", "s74");
    }
    if (r == 0x7fffffffu) sink[0] = r;
}

// ---------------------------------------------------------------- 3. bands of a B tile straight to LDS
// Workgroup = 8 waves; band b = 48 rows picked in ascending order from the tile's k rows (stride `gap` on
// average), six rows per wave, to buffer b % 3; one barrier per band in front of which the loads of the band
// after next may still be in flight.
__global__ __launch_bounds__(512) void fill(const float* __restrict__ B, int k, int ldb, int bands, int gap, int nq, float* out)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const unsigned bid = blockIdx.x, per = gridDim.x >> 3;
    const unsigned item = (bid & 7u) * per + (bid >> 3);
    const unsigned tile = item / nq;                       // tile-major, like the kernel (the last tile reaches into the row pitch)
    const float* bt = B + (size_t)tile * 256 + lane * 4;
    unsigned seed = item * 2654435761u + 99u;
    auto request = [&](int band) {
        for (int t = 0; t < 6; ++t) {
            seed = seed * 1664525u + 1013904223u;
            long row = ((long)band * 48 + wv * 6 + t) * gap + (seed >> 10) % gap;
            if (row >= k) row = row % k;
            __builtin_amdgcn_global_load_lds((__attribute__((address_space(1))) const void*)(bt + row * ldb),
                                             (__attribute__((address_space(3))) void*)(lds + (band % 3) * 12288 + (wv * 6 + t) * 256), 16, 0, 0);
        }
    };
    request(0);
    request(1);
    for (int b = 0; b < bands; ++b) {
        if (b + 2 < bands) {
            request(b + 2);
            asm volatile("s_waitcnt vmcnt(6)\n\ts_barrier" ::: "memory");
        } else {
            asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
        }
    }
    if (lds[threadIdx.x] == 123.456f) out[0] = 1.0f;
}

// ---------------------------------------------------------------- 4. the register kernel's fetch pattern
__device__ __forceinline__ void ld16(f32x4& t, unsigned off, const char* base)
{
    asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(t) : "v"(off), "s"(base));
}
__global__ __launch_bounds__(64) void sweep(const char* __restrict__ B, unsigned rows, unsigned pitch, unsigned gap, float* out, int groups)
{
    const int lane = threadIdx.x;
    const unsigned bid = blockIdx.x, per = gridDim.x >> 3;
    const unsigned w = (bid & 7u) * per + (bid >> 3);
    const unsigned tile = w / groups;
    unsigned s = __builtin_amdgcn_readfirstlane(w * 2654435761u + 12345u);
    const char* base = B + (size_t)tile * 1024;
    const unsigned off = lane * 16;
    f32x4 bq[4][4];
    f32x4 acc = {0, 0, 0, 0};
    unsigned row = 0;
    auto issue4 = [&](f32x4(&d)[4]) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            s = s * 1664525u + 1013904223u;
            row += 1 + (s >> 8) % gap;
            const unsigned r = row < rows ? row : rows - 1;
            ld16(d[j], off, base + (size_t)r * pitch);
        }
    };
    issue4(bq[0]);
    issue4(bq[1]);
    issue4(bq[2]);
    while (row < rows) {
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            issue4(bq[(st + 3) % 4]);
            asm volatile("s_waitcnt vmcnt(12)");
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                asm volatile("v_add_f32 %0, %0, %1" : "+v"(acc.x) : "v"(bq[st][j].x));
                asm volatile("v_add_f32 %0, %0, %1" : "+v"(acc.y) : "v"(bq[st][j].w));
            }
        }
    }
    asm volatile("s_waitcnt vmcnt(0)");
    if (acc.x == 123.456f) out[0] = acc.y;
}

template <typename F>
static float timed(F launch, int reps)
{
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    launch();
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    for (int r = 0; r < reps; ++r) launch();
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    float ms;
    CK(hipEventElapsedTime(&ms, e0, e1));
    CK(hipGetLastError());
    return ms / reps;
}

int main()
{
    CK(hipSetDevice(0));
    float* out;
    CK(hipMalloc(&out, 4096));
    unsigned* sink = reinterpret_cast<unsigned*>(out);

    // 1
    CK(hipFuncSetAttribute((const void*)lds_read, hipFuncAttributeMaxDynamicSharedMemorySize, 131072));
    {
        const int iters = 4000;
        const float ms = timed([&] { lds_read<<<kCUs, 512, 131072>>>(iters, sink); }, 3);
        const double bytes = (double)kCUs * 8 * 64 * 16 * 8.0 * iters;
        printf("lds    ds_read_b128, 8 waves per CU: %.3f ms, %.1f TB/s chip; one 1 KB row per entry and tile -> %.0f us for the headline workload\n",
               ms, bytes / ms * 1e-9, kEntryTiles * 1024.0 / (bytes / ms * 1e3) * 1e6);
        fflush(stdout);
    }
    // 2
    CK(hipFuncSetAttribute((const void*)issue<0>, hipFuncAttributeMaxDynamicSharedMemorySize, 3 * 49152));
    CK(hipFuncSetAttribute((const void*)issue<1>, hipFuncAttributeMaxDynamicSharedMemorySize, 3 * 49152));
    CK(hipFuncSetAttribute((const void*)issue<2>, hipFuncAttributeMaxDynamicSharedMemorySize, 3 * 49152));
    CK(hipFuncSetAttribute((const void*)issue<3>, hipFuncAttributeMaxDynamicSharedMemorySize, 3 * 49152));
    CK(hipFuncSetAttribute((const void*)issue<4>, hipFuncAttributeMaxDynamicSharedMemorySize, 3 * 49152));
    {
        const int iters = 4000;
        const char* names[5] = {"16 singles (address, LDS read, index mode, 4 multiply-adds each)  ", "4 quads (one LDS read per four entries)",
                                "multiply-adds and index mode only", "plain v_fmac_f32 only",
                                "16 singles the former way: four sets of B values, a wait per entry"};
        const double instr[5] = {4 * (2 + 8 + 1 + 1 + 23 + 1) - 1 + 4, 115, 107, 67, 172};      // instructions of one turn of each loop (16 entries)
        for (int mode = 0; mode < 5; ++mode) {
            const float ms = timed([&] {
                if (mode == 0) issue<0><<<kCUs, 512, 3 * 49152>>>(iters, out);
                else if (mode == 1) issue<1><<<kCUs, 512, 3 * 49152>>>(iters, out);
                else if (mode == 2) issue<2><<<kCUs, 512, 3 * 49152>>>(iters, out);
                else if (mode == 3) issue<3><<<kCUs, 512, 3 * 49152>>>(iters, out);
                else issue<4><<<kCUs, 512, 3 * 49152>>>(iters, out);
            }, 3);
            const double entries = (double)kCUs * 8 * 16.0 * iters;       // 16 entries per wave and turn
            const double per_entry_ns = ms * 1e6 / ((double)16 * iters);   // per wave
            printf("issue  %-66s %.3f ms: %.2f ns per entry and wave, about %.1f instructions per entry -> %.0f us for the headline workload\n",
                   names[mode], ms, per_entry_ns, instr[mode] / 16.0, kEntryTiles / (entries / ms) * 1e3);
            fflush(stdout);
        }
    }
    // 2a
    CK(hipFuncSetAttribute((const void*)issue128, hipFuncAttributeMaxDynamicSharedMemorySize, 156 * 1024));
    for (int wgs : {1, 2}) {
        const int iters = 4000;
        const size_t lds = (size_t)(156 * 1024) / wgs;
        const float ms = timed([&] { issue128<<<kCUs * wgs, 512, lds>>>(iters, out); }, 3);
        const double entries = (double)kCUs * wgs * 8 * 16.0 * iters;
        printf("issue  16 singles with 128 registers per wave, %d waves per SIMD: %.3f ms, %.2f ns per entry and wave -> %.0f us for the headline workload\n",
               2 * wgs, ms, ms * 1e6 / (16.0 * iters), kEntryTiles / (entries / ms) * 1e3);
        fflush(stdout);
    }
    // 2c
    {
        const int iters = 20000;
        const char* names[5] = {"16 independent s_add_u32", "8 x (s_cmp, s_cbranch not taken)", "8 x (s_cmp, s_cbranch taken)",
                                "8 x (v_readlane_b32, s_add_u32 of its result)", "16 dependent v_add_u32"};
        for (int kind = 0; kind < 5; ++kind) {
            const float ms = timed([&] {
                if (kind == 0) scalar_cost<0><<<kCUs, 512>>>(iters, sink);
                else if (kind == 1) scalar_cost<1><<<kCUs, 512>>>(iters, sink);
                else if (kind == 2) scalar_cost<2><<<kCUs, 512>>>(iters, sink);
                else if (kind == 3) scalar_cost<3><<<kCUs, 512>>>(iters, sink);
                else scalar_cost<4><<<kCUs, 512>>>(iters, sink);
            }, 3);
            printf("scalar %-48s %.3f ms: %.2f ns per instruction and wave (two waves per SIMD, 19 instructions a turn)\n", names[kind], ms,
                   ms * 1e6 / (19.0 * iters));
            fflush(stdout);
        }
    }
    // 2b
    CK(hipFuncSetAttribute((const void*)valu0, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
    CK(hipFuncSetAttribute((const void*)valu1, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
    CK(hipFuncSetAttribute((const void*)valu2, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
    for (int kind = 0; kind < 3; ++kind)
        for (int waves : {1, 2, 4}) {
            const int iters = 4000;
            const size_t lds = (size_t)(156 * 1024) / waves;        // so that exactly `waves` workgroups fit a compute unit
            const float ms = timed([&] {
                if (kind == 0) valu0<<<kCUs * waves, 256, lds>>>(iters, out);
                else if (kind == 1) valu1<<<kCUs * waves, 256, lds>>>(iters, out);
                else valu2<<<kCUs * waves, 256, lds>>>(iters, out);
            }, 3);
            const double per_simd = (double)waves * 64.0 * iters / (ms * 1e6);       // v_fmac_f32 per ns and SIMD
            const char* names[3] = {"operands in three register banks", "all three operands in one bank", "both sources in one bank"};
            printf("valu   %d waves per SIMD, independent v_fmac_f32, %s: %.3f ms, %.2f instructions per ns and SIMD, %.1f TFLOP/s for the chip\n",
                   waves, names[kind], ms, per_simd, per_simd * 1024 * 128.0 * 1e-3);
            fflush(stdout);
        }
    // 3 and 4 read a B of 8000 x 8000 floats
    const int k = 8000, ldb = 8000;
    float* B;
    CK(hipMalloc(&B, (size_t)k * ldb * 4 + 65536));
    CK(hipMemset(B, 0, (size_t)k * ldb * 4 + 65536));
    CK(hipFuncSetAttribute((const void*)fill, hipFuncAttributeMaxDynamicSharedMemorySize, 3 * 49152));
    {
        // the headline workload at 42 rows per group: 24 super-groups x 32 tiles, 136 bands each (6515 distinct columns of 8000)
        const int grid = 24 * 32, bands = 136;
        const float ms = timed([&] { fill<<<grid, 512, 3 * 49152>>>(B, k, ldb, bands, 1, 24, out); }, 5);
        const double bytes = (double)grid * bands * 48 * 1024.0;
        printf("fill   %d workgroups x %d bands x 48 rows of 1 KB straight to LDS, one barrier per band: %.3f ms, %.1f TB/s (%.1f GB: what the "
               "workgroup-shared kernel fetches for the headline workload at 42 rows per group)\n", grid, bands, ms, bytes / ms * 1e-9, bytes * 1e-9);
        fflush(stdout);
    }
    {
        // the headline workload at 32 rows per group: 250 groups x 32 tiles, each wave loads about 1/7 of the 8000 rows
        const int groups = 250, tiles = 32, grid = groups * tiles;
        for (unsigned gap : {13u, 1u}) {
            const float ms = timed([&] { sweep<<<grid, 64>>>(reinterpret_cast<const char*>(B), (unsigned)k, (unsigned)ldb * 4u, gap, out, groups); }, 5);
            const double loads = (double)grid * (k / ((gap + 1) / 2.0));
            printf("sweep  %d waves, every %s row of a tile, 1 KB per load, 12 loads in flight: %.3f ms, %.1f TB/s through the vector cache (%.1f GB%s)\n",
                   grid, gap == 1 ? "" : "7th (on average)", ms, loads * 1024.0 / ms * 1e-9, loads * 1024.0 * 1e-9,
                   gap == 1 ? "" : ": what the register kernel fetches for the headline workload");
            fflush(stdout);
        }
    }
    return 0;
}
