// Host-side launch interface of the register SpDM kernels.  Each (P, V) instance is compiled in
// a translation unit of its own (spdm_reg_p*_v*.hip) so that the instances build in parallel.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gcoo {

// One control word per stored entry, built after the sort:
//   bit 31      first entry of a run of equal columns inside its group
//   bits 0..7   row inside the group (row - q*p)
//   bits 8..11  only in the first entry of every chunk of kChunk entries of a group (counted
//               from the group's start): number of run heads in that chunk
constexpr uint32_t kHeadBit = 0x80000000u;
constexpr int kChunk = 8;
constexpr int kCountShift = 8;

struct SpdmArgs {
    const float* values;
    const int32_t* cols;
    const uint32_t* ctl;
    const int32_t* gIdxes;
    int64_t m;
    int32_t p;
    int64_t g;
    const float* B;
    int64_t ldb;
    int64_t N;
    float* C;
    int64_t ldc;
};

// Launch spdm_reg<P, V, *, reuse> for one of the built (P, V) pairs:
// (8,4) (16,4) (32,4) (64,2) (128,1).  Any other pair returns hipErrorInvalidValue.
hipError_t launch_spdm_reg(int P, int V, bool reuse, const SpdmArgs& a, hipStream_t s);

hipError_t launch_spdm_reg_p8_v4(bool reuse, const SpdmArgs& a, hipStream_t s);
hipError_t launch_spdm_reg_p16_v4(bool reuse, const SpdmArgs& a, hipStream_t s);
hipError_t launch_spdm_reg_p32_v4(bool reuse, const SpdmArgs& a, hipStream_t s);
hipError_t launch_spdm_reg_p64_v2(bool reuse, const SpdmArgs& a, hipStream_t s);
hipError_t launch_spdm_reg_p128_v1(bool reuse, const SpdmArgs& a, hipStream_t s);

}  // namespace gcoo
