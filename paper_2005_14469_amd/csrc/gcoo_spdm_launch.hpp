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
    int32_t heavy_min;         // groups with this many entries or more go to the workgroup-shared kernel (INT32_MAX: none)
};

// V = 4 needs p <= 32, V = 38 (four columns per lane, tall accumulator file) p <= 38, V = 2 needs
// p <= 64, V = 1 needs p <= 128; N, ldb, ldc and both base addresses must be multiples of the
// columns per lane.  Anything else returns hipErrorInvalidValue.
hipError_t launch_spdm_sched(int V, const SpdmArgs& a, hipStream_t s);

hipError_t launch_spdm_sched_v4(const SpdmArgs& a, hipStream_t s);
hipError_t launch_spdm_sched_v4_tall(const SpdmArgs& a, hipStream_t s);
hipError_t launch_spdm_sched_v2(const SpdmArgs& a, hipStream_t s);
hipError_t launch_spdm_sched_v1(const SpdmArgs& a, hipStream_t s);

// The workgroup-shared kernel (band schedule): p <= 32; N, ldb, ldc multiples of 4; B and C 16-byte aligned.
struct BandArgs {
    const uint32_t* stream;    // band schedule
    const int32_t* gIdxes;     // [g+1]
    const int32_t* ucount;     // [nq] distinct columns per super-group
    int64_t m;
    int32_t p;
    int64_t g;
    int64_t k;
    int64_t nq;                // super-groups
    const float* B;
    int64_t ldb;
    int64_t N;
    float* C;
    int64_t ldc;
};
hipError_t launch_spdm_band(const BandArgs& a, hipStream_t s);

}  // namespace gcoo
