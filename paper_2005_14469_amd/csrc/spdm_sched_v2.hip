// Instance of the register SpDM kernel with V = 2 columns per lane.
#include "gcoo_spdm_kernels.hpp"

namespace gcoo {
hipError_t launch_spdm_sched_v2(const SpdmArgs& a, hipStream_t s) { return launch_spdm_sched_instance<2>(a, s); }
}  // namespace gcoo
