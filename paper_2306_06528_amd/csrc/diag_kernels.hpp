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
//          (lane (q, c) takes row r0 + q of a 64-column tile);
//   PAT 1: the vector-ALU update's pattern - a wave instruction covers 1 KiB of one row (256-column
//          tile).
// U loads per array are in flight per lane (U * RPI rows); rows beyond n are clamped for the loads
// and masked for the stores, so the steady state has no divergent branch.  The waves of a
// workgroup take adjacent tiles; workgroups stride over the full tiles (reverse: from the last
// tile down, so that a caller alternating the direction starts each pass on what the previous one
// left in the memory-side cache); the columns after the last full tile are done element-wise by
// the last workgroup.  Stores carry the streaming hint, as the update's do; NT = 1: so do all
// loads, NT = 2: so do the loads of G while X is loaded plainly, the update's policy (streaming
// loads are only sensible when no cache line is shared between rows, i.e. rows that start on
// 128-byte boundaries).
template <int PAT, int U, int NT>
__global__ __launch_bounds__(256) void diag_axpy_rows_kernel(float *__restrict__ X, const float *__restrict__ G,
                                                             int n, int64_t D, int64_t ld, float s, int reverse)
{
    constexpr int TC = PAT == 0 ? 64 : 256;      // columns per wave tile
    constexpr int RPI = PAT == 0 ? 4 : 1;        // rows per wave instruction
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int q = lane >> 4, c16 = lane & 15;
    const int64_t nfull = D / TC;
    const int lrow = PAT == 0 ? q : 0;
    const int64_t lcol = PAT == 0 ? 4 * c16 : 4 * lane;
    const int64_t first = (int64_t)blockIdx.x * 4 + wave, stride = (int64_t)gridDim.x * 4;
    const int64_t cnt = first < nfull ? (nfull - 1 - first) / stride + 1 : 0;
    for (int64_t k = 0; k < cnt; ++k) {
        const int64_t tile = first + (reverse ? cnt - 1 - k : k) * stride;
        const int64_t col = tile * TC + lcol;
        for (int r0 = 0; r0 < n; r0 += U * RPI) {
            f32x4 x[U], g[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int row = r0 + u * RPI + lrow;
                const int64_t off = (int64_t)(row < n ? row : n - 1) * ld + col;
                if constexpr (NT == 1) x[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4u *>(X + off));
                else x[u] = *reinterpret_cast<const f32x4u *>(X + off);
                if constexpr (NT != 0) g[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4u *>(G + off));
                else g[u] = *reinterpret_cast<const f32x4u *>(G + off);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int row = r0 + u * RPI + lrow;
                if (row < n)
                    __builtin_nontemporal_store(x[u] + s * g[u], reinterpret_cast<f32x4u *>(X + (int64_t)row * ld + col));
            }
        }
    }
    if (blockIdx.x == gridDim.x - 1) {
        const int64_t c0 = nfull * TC, ntail = D - c0;
        for (int64_t e = threadIdx.x; e < ntail * n; e += 256) {
            const int64_t row = e / ntail, col = c0 + e % ntail;
            X[row * ld + col] += s * G[row * ld + col];
        }
    }
}

// The traffic shape of the pairwise pass and nothing else: every element of n rows of D floats,
// ld floats apart, is read once with 16-byte loads and added up (so that the loads cannot be
// dropped); one float per workgroup goes to sink[blockIdx.x].  PAT and NT as above (NT = 1: the
// loads carry the streaming hint), eight loads in flight per lane, workgroups stride over the
// full tiles with their waves on adjacent tiles, the columns after the last full tile are read
// element-wise by the last workgroup.
template <int PAT, int NT>
__global__ __launch_bounds__(256) void diag_read_rows_kernel(const float *__restrict__ X, int n, int64_t D, int64_t ld,
                                                             float *__restrict__ sink)
{
    constexpr int TC = PAT == 0 ? 64 : 256;
    constexpr int RPI = PAT == 0 ? 4 : 1;
    constexpr int U = 8;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int q = lane >> 4, c16 = lane & 15;
    const int64_t nfull = D / TC;
    const int lrow = PAT == 0 ? q : 0;
    const int64_t lcol = PAT == 0 ? 4 * c16 : 4 * lane;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int64_t tile = (int64_t)blockIdx.x * 4 + wave; tile < nfull; tile += (int64_t)gridDim.x * 4) {
        const int64_t col = tile * TC + lcol;
        for (int r0 = 0; r0 < n; r0 += U * RPI) {
            f32x4 x[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int row = r0 + u * RPI + lrow;
                const int64_t off = (int64_t)(row < n ? row : n - 1) * ld + col;
                if constexpr (NT == 1) x[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4u *>(X + off));
                else x[u] = *reinterpret_cast<const f32x4u *>(X + off);
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (r0 + u * RPI + lrow < n) acc += x[u];
        }
    }
    float t = (acc.x + acc.y) + (acc.z + acc.w);
    if (blockIdx.x == gridDim.x - 1) {
        const int64_t c0 = nfull * TC, ntail = D - c0;
        for (int64_t e = threadIdx.x; e < ntail * n; e += 256) t += X[(e / ntail) * ld + c0 + e % ntail];
    }
    __shared__ float part[4];
    t = wave_sum(t);
    if (lane == 0) part[wave] = t;
    __syncthreads();
    if (threadIdx.x == 0) sink[blockIdx.x] = (part[0] + part[1]) + (part[2] + part[3]);
}

} // namespace svgd
