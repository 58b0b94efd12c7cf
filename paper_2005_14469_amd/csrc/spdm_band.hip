// The workgroup-shared SpDM kernel (4 columns per lane), its two instances and their launcher.
#include "gcoo_spdm_band_kernel.hpp"

namespace gcoo {

template <class S>
static hipError_t launch_band_instance(const BandArgs& a, int64_t grid, int64_t total, hipStream_t s)
{
    // more LDS than the default limit of a workgroup: ask for it once per device
    static thread_local int asked_on = -1;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (asked_on != dev) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&spdm_band<S>), hipFuncAttributeMaxDynamicSharedMemorySize, kBandLdsBytes);
        if (e != hipSuccess) return e;
        asked_on = dev;
    }
    spdm_band<S><<<dim3((unsigned)grid), dim3(64 * S::W), kBandLdsBytes, s>>>(a.stream, a.gIdxes, a.ucount, a.m, a.p, a.g, a.k, a.nq, a.B,
                                                                           a.ldb, a.N, a.C, a.ldc, total);
    return hipGetLastError();
}

hipError_t launch_spdm_band(const BandArgs& a, hipStream_t s)
{
    const int64_t tiles = (a.N + 255) / 256;
    const int64_t total = a.nq * tiles;
    const int64_t grid = (total + 7) / 8 * 8;              // whole rounds over the 8 XCDs
    if (grid <= 0 || grid > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    if (a.p < 1 || a.p > kBandMaxP || a.N % 4 != 0 || a.ldb % 4 != 0 || a.ldc % 4 != 0) return hipErrorInvalidValue;
    if (a.ldb > 0x3fffffffLL) return hipErrorInvalidValue;   // row pitch in bytes is kept in 32 bits
    if (a.nq != (a.g + band_waves(a.p) - 1) / band_waves(a.p)) return hipErrorInvalidValue;
    return band_waves(a.p) == 16 ? launch_band_instance<BandShape16>(a, grid, total, s) : launch_band_instance<BandShape8>(a, grid, total, s);
}

}  // namespace gcoo
