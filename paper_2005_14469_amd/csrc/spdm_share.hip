// The workgroup-shared SpDM kernel that reads the share schedule, and its launcher.
#include "gcoo_spdm_share_kernel.hpp"
#include "gcoo_spdm_launch.hpp"

namespace gcoo {

hipError_t launch_spdm_share(const ShareArgs& a, hipStream_t s)
{
    const int64_t tiles = (a.N + 255) / 256;
    const int64_t total = a.nq * tiles;
    const int64_t grid = (total + 7) / 8 * 8;              // whole rounds over the 8 XCDs
    if (grid <= 0 || grid > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    if (a.p < 1 || a.p > kShareMaxP || a.N % 4 != 0 || a.ldb % 4 != 0 || a.ldc % 4 != 0) return hipErrorInvalidValue;
    if (a.nq != share_super_groups(a.g)) return hipErrorInvalidValue;
    // more LDS than the default limit of a workgroup: ask for it once per device
    static thread_local int asked_on = -1;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (asked_on != dev) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&spdm_share), hipFuncAttributeMaxDynamicSharedMemorySize, kShareLdsBytes);
        if (e != hipSuccess) return e;
        asked_on = dev;
    }
    spdm_share<<<dim3((unsigned)grid), dim3(64 * kShareW), kShareLdsBytes, s>>>(a, total);
    return hipGetLastError();
}

}  // namespace gcoo
