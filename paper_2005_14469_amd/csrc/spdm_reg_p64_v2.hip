// Instance P = 64 rows of partial sums, V = 2 columns per lane of the register SpDM kernel.
#include "gcoo_spdm_kernels.hpp"

namespace gcoo {
hipError_t launch_spdm_reg_p64_v2(bool reuse, const SpdmArgs& a, hipStream_t s)
{
    return reuse ? launch_spdm_reg_instance<64, 2, true>(a, s) : launch_spdm_reg_instance<64, 2, false>(a, s);
}
}  // namespace gcoo
