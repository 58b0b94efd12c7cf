// Instance of the register SpDM kernel with V = 4 columns per lane and the tall accumulator file
// (groups of 33 .. 38 rows).
#define GCOO_ACC_TALL 1
#include "gcoo_spdm_kernels.hpp"

namespace gcoo {
hipError_t launch_spdm_sched_v4_tall(const SpdmArgs& a, hipStream_t s) { return launch_spdm_sched_instance<4>(a, s); }
}  // namespace gcoo
