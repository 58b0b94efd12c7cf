// A plain CSR row-split SpMM, the kind of kernel the paper measures GCOOSpDM against
// (Section 4: the vendor CSR routine).  It is here for context in the benchmark only and is
// deliberately simple: one wave64 per (row of A, 256 columns of B), the row's entries are read one
// after the other (they are wave-uniform), each one fetches its 1 KB segment of a B row, and the
// wave keeps four sums per lane.  No staging, no reuse of B across rows.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gcoo_baseline.h"

namespace gcoo {

template <int V>
__global__ __launch_bounds__(64) void csr_spmm_rowsplit(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
                                                        const float* __restrict__ vals, int64_t m, const float* __restrict__ B,
                                                        int64_t ldb, int64_t N, float* __restrict__ C, int64_t ldc, int64_t tiles)
{
    const int64_t w = blockIdx.x;
    const int64_t row = w / tiles, tile = w - row * tiles;     // tiles of one row are neighbours: they share the row's entries in cache
    if (row >= m) return;
    const int64_t j0 = tile * (64 * V) + (int64_t)threadIdx.x * V;
    if (j0 >= N) return;
    float acc[V];
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = 0.0f;
    const int32_t e0 = row_ptr[row], e1 = row_ptr[row + 1];
    for (int32_t e = e0; e < e1; ++e) {
        const float a = vals[e];
        const float* b = B + (int64_t)col_idx[e] * ldb + j0;
        if constexpr (V == 4) {
            const float4 t = *reinterpret_cast<const float4*>(b);
            acc[0] = fmaf(a, t.x, acc[0]); acc[1] = fmaf(a, t.y, acc[1]); acc[2] = fmaf(a, t.z, acc[2]); acc[3] = fmaf(a, t.w, acc[3]);
        } else {
            acc[0] = fmaf(a, b[0], acc[0]);
        }
    }
    float* c = C + row * ldc + j0;
    if constexpr (V == 4) *reinterpret_cast<float4*>(c) = make_float4(acc[0], acc[1], acc[2], acc[3]);
    else c[0] = acc[0];
}

}  // namespace gcoo

extern "C" int gcoo_csr_spmm_baseline(int64_t m, int64_t k, const int32_t* row_ptr_dev, const int32_t* col_idx_dev,
                                      const float* vals_dev, const float* B_dev, int64_t ldb, int64_t N, float* C_dev,
                                      int64_t ldc, void* stream)
{
    if (m < 0 || k < 0 || N < 0 || ldb < N || ldc < N || !row_ptr_dev) return -1;
    if (m == 0 || N == 0) return 0;
    if (!C_dev || !B_dev) return -1;
    const uintptr_t pb = reinterpret_cast<uintptr_t>(B_dev), pc = reinterpret_cast<uintptr_t>(C_dev);
    const bool v4 = (N % 4 == 0) && (ldb % 4 == 0) && (ldc % 4 == 0) && (pb % 16 == 0) && (pc % 16 == 0);
    const int V = v4 ? 4 : 1;
    const int64_t tiles = (N + 64 * V - 1) / (64 * V);
    if (m > 0x7fffffffLL / tiles) return -1;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)(m * tiles)), block(64);
    if (v4) gcoo::csr_spmm_rowsplit<4><<<grid, block, 0, s>>>(row_ptr_dev, col_idx_dev, vals_dev, m, B_dev, ldb, N, C_dev, ldc, tiles);
    else gcoo::csr_spmm_rowsplit<1><<<grid, block, 0, s>>>(row_ptr_dev, col_idx_dev, vals_dev, m, B_dev, ldb, N, C_dev, ldc, tiles);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}
