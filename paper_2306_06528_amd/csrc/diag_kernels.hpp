// Diagnostic yardsticks (not part of the SVGD path): plain memory kernels of known traffic, used
// to scale hardware byte counters and to measure what this part's HBM gives a kernel that does
// nothing but the update's memory accesses.
#pragma once
#include "common.hpp"

namespace svgd {

// Plain copy of known size: reads and writes exactly n16 * 16 bytes.
__global__ __launch_bounds__(256) void diag_copy_kernel(const f32x4 *__restrict__ src,
                                                        f32x4 *__restrict__ dst, int64_t n16)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (int64_t)gridDim.x * 256)
        dst[i] = src[i];
}

// The traffic shape of the fused update and nothing else: x_i <- x_i + s * g_i in place for n rows
// of D floats, ld floats apart - per element one read of X, one read of G, one write of X, over
// the same 2n row streams, with 16-byte accesses.  No kernel matrix, no contraction.
//   PAT 0: the matrix-core update's access pattern - a wave instruction covers 4 rows x 256 bytes
//          (lane (q, c) takes row r0 + q of a 64-column tile), 8 such loads per array in flight;
//   PAT 1: the vector-ALU update's pattern - a wave instruction covers 1 KiB of one row (256-column
//          tile), 8 rows per array in flight.
// The waves of a workgroup take adjacent tiles; workgroups stride over the tiles.  Stores carry
// the streaming hint, as the update's do.
template <int PAT>
__global__ __launch_bounds__(256) void diag_axpy_rows_kernel(float *__restrict__ X, const float *__restrict__ G,
                                                             int n, int64_t D, int64_t ld, float s)
{
    constexpr int TC = PAT == 0 ? 64 : 256;      // columns per wave tile
    constexpr int RPI = PAT == 0 ? 4 : 1;        // rows per wave instruction
    constexpr int U = 8;                         // loads per array in flight
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int q = lane >> 4, c16 = lane & 15;
    const int64_t ntile = (D + TC - 1) / TC;
    for (int64_t tile = (int64_t)blockIdx.x * 4 + wave; tile < ntile; tile += (int64_t)gridDim.x * 4) {
        const int64_t col = tile * TC + (PAT == 0 ? 4 * c16 : 4 * lane);
        const bool full = (col + 4 <= D);
        for (int r0 = 0; r0 < n; r0 += U * RPI) {
            f32x4 x[U], g[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int row = r0 + u * RPI + (PAT == 0 ? q : 0);
                if (row < n) {
                    x[u] = load4(X + (int64_t)row * ld, col, D, full);
                    g[u] = load4(G + (int64_t)row * ld, col, D, full);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int row = r0 + u * RPI + (PAT == 0 ? q : 0);
                if (row < n) store4(X + (int64_t)row * ld, col, D, full, x[u] + s * g[u]);
            }
        }
    }
}

} // namespace svgd
