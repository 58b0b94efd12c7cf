// Instance P = 8 rows of partial sums, V = 4 columns per lane of the register SpDM kernel.
#include "gcoo_spdm_kernels.hpp"

namespace gcoo {
hipError_t launch_spdm_reg_p8_v4(bool reuse, const SpdmArgs& a, hipStream_t s)
{
    return reuse ? launch_spdm_reg_instance<8, 4, true>(a, s) : launch_spdm_reg_instance<8, 4, false>(a, s);
}
}  // namespace gcoo
