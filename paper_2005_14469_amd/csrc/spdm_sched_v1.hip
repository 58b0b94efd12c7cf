// Instance of the register SpDM kernel with V = 1 columns per lane.
#include "gcoo_spdm_kernels.hpp"

namespace gcoo {
hipError_t launch_spdm_sched_v1(const SpdmArgs& a, hipStream_t s) { return launch_spdm_sched_instance<1>(a, s); }
}  // namespace gcoo
