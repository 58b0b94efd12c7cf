// Host-side launch interface of the register SpDM kernel.  Each V (columns per lane) is compiled
// in a translation unit of its own (spdm_sched_v*.hip) so that the instances build in parallel.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <limits.h>

namespace gcoo {

struct SchedClass;

struct SpdmArgs {
    const SchedClass* hdr;     // [g][nw][kMaxRun]
    const uint32_t* stream;    // run schedule
    const int32_t* gIdxes;     // [g+1]
    int64_t m;
    int32_t p;
    int64_t g;
    int32_t nw;                // column windows of the schedule
    const float* B;
    int64_t ldb;
    int64_t N;
    float* C;
    int64_t ldc;
    int64_t nnz;
    // statistics of the conversion on the device ([1] = entries of the largest group), from which the
    // kernel derives the entry count from which a group is split over the waves of a workgroup; nullptr: the
    // launch has too many items for that to pay
    const unsigned long long* stats;
    // order[0..g): the groups by falling size; order[g..2g): those sizes.  nullptr: not built (more than
    // kOrderMaxGroups groups)
    const int32_t* order;
};

// V = 4 needs p <= 32, V = 38 (four columns per lane, tall accumulator file) p <= 38, V = 2 needs
// p <= 64; N, ldb, ldc and both base addresses must be multiples of the columns per lane.
// Anything else returns hipErrorInvalidValue.
hipError_t launch_spdm_sched(int V, const SpdmArgs& a, hipStream_t s);

hipError_t launch_spdm_sched_v4(const SpdmArgs& a, hipStream_t s);
hipError_t launch_spdm_sched_v4_tall(const SpdmArgs& a, hipStream_t s);
hipError_t launch_spdm_sched_v2(const SpdmArgs& a, hipStream_t s);

// The workgroup-shared kernel that reads the share schedule: p <= 48; N, ldb, ldc multiples of 4; B and C
// 16-byte aligned; every row offset of B in bytes below 2^32.
struct ShareArgs {
    const uint32_t* hdr;       // headers
    const uint32_t* blocks;    // streams
    const int32_t* sbase;      // [8 * nq] first block of every stream
    const int32_t* ucols;      // distinct columns per super-group, the list of Q starting at gIdxes[8Q]
    const int32_t* ucount;     // [nq]
    const int32_t* gIdxes;     // [g + 1]
    int64_t m;
    int32_t p;
    int64_t g;
    int64_t nq;                // super-groups
    const float* B;
    int64_t ldb;
    int64_t N;
    float* C;
    int64_t ldc;
};
hipError_t launch_spdm_share(const ShareArgs& a, hipStream_t s);

}  // namespace gcoo
