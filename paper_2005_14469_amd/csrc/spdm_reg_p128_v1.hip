// Instance P = 128 rows of partial sums, V = 1 columns per lane of the register SpDM kernel.
#include "gcoo_spdm_kernels.hpp"

namespace gcoo {
hipError_t launch_spdm_reg_p128_v1(bool reuse, const SpdmArgs& a, hipStream_t s)
{
    return reuse ? launch_spdm_reg_instance<128, 1, true>(a, s) : launch_spdm_reg_instance<128, 1, false>(a, s);
}
}  // namespace gcoo
