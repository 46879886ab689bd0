// Pass 3: the fused all-particle update.  For every column k independently
//
//     z_jk   = g_jk - (2/h) x_jk
//     phi_ik = sum_j C_ij z_jk + rho_i x_ik,      C_ij = K_ij / n,  rho_i = (2/h) (sum_j K_ij) / n
//     x_ik  <- x_ik + eps * phi_ik
//
// which is phi_i = (1/n) sum_j [K_ij g_j + (2/h) K_ij (x_i - x_j)] with the sum over j of the
// x_j terms folded into a single n x n product (paper App. B.2: `update.add_(p_j_grad, alpha=k)`,
// `update.add_(diff)`, `update / n`, then the followers' `p.add_(update, alpha=lr)`).
// X and G are read once and X is written once, in place: a column's outputs depend only on that
// column's inputs, and every thread/wave loads all n rows of its columns before storing any, so
// every phi_i is computed from the pre-step X.
#pragma once
#include "common.hpp"

namespace svgd {

// ---------------------------------------------------------------------------------------------
// n <= 16: vector ALU, lanes = columns, 4 consecutive columns per thread (16-byte loads, 1 KiB
// contiguous per row per wave).  C and rho are wave-uniform and read through scalar loads.
// ---------------------------------------------------------------------------------------------
template <int N, bool EMIT>
__global__ __launch_bounds__(256) void update_valu_kernel(float *__restrict__ X,
                                                          const float *__restrict__ G,
                                                          float *__restrict__ PHI,
                                                          const float *__restrict__ coef,
                                                          const DevState *__restrict__ st,
                                                          int64_t D, float eps)
{
    const float c2h = st->two_over_h;
    const float *__restrict__ C = coef + kOffC;
    const float *__restrict__ rho = coef + kOffRho;
    const int64_t ngroups = (D + 3) >> 2;
    const int64_t nthreads = (int64_t)gridDim.x * 256;
    for (int64_t grp = (int64_t)blockIdx.x * 256 + threadIdx.x; grp < ngroups; grp += nthreads) {
        const int64_t col = grp << 2;
        const bool full = (col + 4 <= D);
        f32x4 x[N], z[N];
#pragma unroll
        for (int j = 0; j < N; ++j) {
            x[j] = load4(X + (int64_t)j * D, col, D, full);
            z[j] = load4(G + (int64_t)j * D, col, D, full);
        }
#pragma unroll
        for (int j = 0; j < N; ++j) z[j] -= c2h * x[j];
#pragma unroll
        for (int i = 0; i < N; ++i) {
            f32x4 acc = rho[i] * x[i];
#pragma unroll
            for (int j = 0; j < N; ++j) acc += C[i * N + j] * z[j];
            if constexpr (EMIT)
                store4(PHI + (int64_t)i * D, col, D, full, acc);
            else
                store4(X + (int64_t)i * D, col, D, full, x[i] + eps * acc);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// 16 < n <= 64: matrix cores, v_mfma_f32_16x16x4_f32 with M = output particle i, K = input
// particle j, N = column.  A wave owns 16*NB rows x 64 columns per iteration:
//   lane (q = lane/16, c = lane%16) loads, for b < NB and r < 4, row 16b + 4q + r at columns
//   4c..4c+3 of the tile (256 B contiguous per row per quarter-wave).  Step s = 4b + r of the
//   contraction feeds k-slot q with row 16b + 4q + r; the 4 components of the 16-byte load are
//   4 independent N-tiles (tile t = columns {4c + t}).  The 16x16 result of output block bi puts
//   row 16bi + 4q + r, column c in register r of lane (q, c) - exactly the rows this lane
//   loaded, so x_old is already in place for the epilogue and nothing crosses lanes.
// The A operands (C re-ordered, 4*NB*NB registers) are loaded once per wave; the grid is
// persistent.  Rows >= n (n not a multiple of 16) are neither loaded nor stored; their A entries
// are zero.
// ---------------------------------------------------------------------------------------------
template <int NB, bool EMIT>
__global__ __launch_bounds__(256) void update_mfma_kernel(float *__restrict__ X,
                                                          const float *__restrict__ G,
                                                          float *__restrict__ PHI,
                                                          const float *__restrict__ coef,
                                                          const DevState *__restrict__ st, int n,
                                                          int64_t D, float eps)
{
    constexpr int NS = 4 * NB; // contraction steps = rows per lane
    const int lane = threadIdx.x & 63;
    const int q = lane >> 4, c16 = lane & 15;
    const float c2h = st->two_over_h;

    float A[NB][NS];
#pragma unroll
    for (int bi = 0; bi < NB; ++bi)
#pragma unroll
        for (int s = 0; s < NS; ++s) A[bi][s] = coef[kOffAT + (bi * NS + s) * kWave + lane];
    float rho[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        const int row = 16 * (s >> 2) + 4 * q + (s & 3);
        rho[s] = (row < n) ? coef[kOffRho + row] : 0.f;
    }

    const int64_t ntile = (D + 63) >> 6;
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    for (int64_t tile = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); tile < ntile; tile += nwaves) {
        const int64_t col = (tile << 6) + 4 * c16;
        const bool full = ((tile << 6) + 64 <= D);
        f32x4 x[NS], z[NS];
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const int row = 16 * (s >> 2) + 4 * q + (s & 3);
            if (row < n) {
                x[s] = load4(X + (int64_t)row * D, col, D, full);
                z[s] = load4(G + (int64_t)row * D, col, D, full);
            } else {
                x[s] = f32x4{0.f, 0.f, 0.f, 0.f};
                z[s] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
        }
#pragma unroll
        for (int s = 0; s < NS; ++s) z[s] -= c2h * x[s];

#pragma unroll
        for (int t = 0; t < 4; ++t) {
            f32x4 acc[NB];
#pragma unroll
            for (int bi = 0; bi < NB; ++bi) acc[bi] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < NS; ++s)
#pragma unroll
                for (int bi = 0; bi < NB; ++bi)
                    acc[bi] = __builtin_amdgcn_mfma_f32_16x16x4f32(A[bi][s], z[s][t], acc[bi], 0, 0, 0);
#pragma unroll
            for (int bi = 0; bi < NB; ++bi)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int s = 4 * bi + r;
                    const float phi = fmaf(rho[s], x[s][t], acc[bi][r]);
                    x[s][t] = EMIT ? phi : fmaf(eps, phi, x[s][t]);
                }
        }
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const int row = 16 * (s >> 2) + 4 * q + (s & 3);
            if (row < n) store4((EMIT ? PHI : X) + (int64_t)row * D, col, D, full, x[s]);
        }
    }
}

} // namespace svgd
