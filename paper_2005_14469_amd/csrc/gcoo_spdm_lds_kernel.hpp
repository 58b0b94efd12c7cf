// The LDS variant of the SpDM kernel: Algorithm 2 of the paper with the partial sums in LDS.
// It reads the five GCOO arrays as they are and serves every shape.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>


namespace gcoo {


// ---------------------------------------------------------------------------------------------
// Variant LDS: the p x 64 partial sums of a wave live in LDS (one column per lane, so no bank
// conflicts and no cross-lane hazards).  Works for every p <= 256, every N and leading
// dimension.  The fallback for shapes the register kernels do not take.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void spdm_lds(const float* __restrict__ values, const int32_t* __restrict__ rows,
                                               const int32_t* __restrict__ cols, const int32_t* __restrict__ gIdxes,
                                               int64_t m, int32_t p, const float* __restrict__ B, int64_t ldb, int64_t N,
                                               float* __restrict__ C, int64_t ldc, int64_t g)
{
    extern __shared__ float acc[];                       // p * 64
    const int lane = threadIdx.x;
    const int64_t w = blockIdx.x;
    const int64_t tile = w / g, q = w - tile * g;
    const int64_t j = tile * 64 + lane;
    const bool in = j < N;
    const int32_t beg = gIdxes[q], end = gIdxes[q + 1];
    const int64_t row0 = q * p;
    for (int i = 0; i < p; ++i) acc[i * 64 + lane] = 0.0f;
    int32_t prev = -1;
    float bv = 0.0f;
    for (int32_t e = beg; e < end; ++e) {
        const int32_t col = cols[e];
        const int32_t r = rows[e] - (int32_t)row0;
        const float av = values[e];
        if (col != prev) {                                // new run: fetch the B value once
            bv = in ? B[(int64_t)col * ldb + j] : 0.0f;
            prev = col;
        }
        acc[r * 64 + lane] += av * bv;
    }
    if (in) {
        for (int i = 0; i < p && row0 + i < m; ++i) C[(row0 + i) * ldc + j] = acc[i * 64 + lane];
    }
}


}  // namespace gcoo
