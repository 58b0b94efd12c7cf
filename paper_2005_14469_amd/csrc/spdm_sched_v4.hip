// Instance of the register SpDM kernel with V = 4 columns per lane.
#include "gcoo_spdm_kernels.hpp"

namespace gcoo {
hipError_t launch_spdm_sched_v4(const SpdmArgs& a, hipStream_t s) { return launch_spdm_sched_instance<4>(a, s); }
}  // namespace gcoo
