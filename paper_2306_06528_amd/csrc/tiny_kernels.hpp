// The whole step in one launch, for problems so small that three dependent launches cost more
// than the work: a single workgroup computes the pair sums, the bandwidth, K and the update
// (passes 1 to 3 of the larger path, same arithmetic) with barriers in between instead of kernel
// boundaries.  Worth it only while one compute unit can stream X and G in about the time a launch
// takes, hence the size limit.  512 threads: at most two 4-column groups per thread, and 256
// registers per lane for the accumulators.
#pragma once
#include "bandwidth_kernels.hpp"
#include "gram_kernels.hpp"

namespace svgd {

constexpr int kTinyMaxN = 8; // the direct-difference format; larger n start to spill registers
constexpr int64_t kTinyMaxElems = 16384; // n * D
constexpr int kTinyThreads = 512;

enum TinyWhat : int {
    kTinyStep = 0,     // X updated in place
    kTinyPhi = 1,      // phi written to PHI, X untouched
    kTinyBandwidth = 2 // passes 1 and 2 only: h, K and the tables (same sums, hence the same h)
};

template <int N, int WHAT>
__global__ __launch_bounds__(kTinyThreads) void step_tiny_kernel(float *__restrict__ X,
                                                               const float *__restrict__ G,
                                                               float *__restrict__ PHI, int64_t D, int64_t ld,
                                                               float eps, double h_fixed,
                                                               DevState *__restrict__ st,
                                                               float *__restrict__ coef)
{
    static_assert(N <= kTinyMaxN, "direct differences only");
    constexpr int P = N * (N + 1) / 2;
    __shared__ BwShared sh;
    __shared__ float cl[N * N + N]; // C, then rho
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int64_t ngroups = (D + 3) >> 2;

    // pass 1: pair sums over the columns in the format of gram_valu_kernel<N>, lanes = 4-column groups
    float acc[P];
#pragma unroll
    for (int p = 0; p < P; ++p) acc[p] = 0.f;
    for (int64_t grp = tid; grp < ngroups; grp += kTinyThreads) {
        const int64_t col = grp << 2;
        const bool full = (col + 4 <= D);
        f32x4 x[N];
#pragma unroll
        for (int j = 0; j < N; ++j) x[j] = load4(X + (int64_t)j * ld, col, D, full);
        pair_accumulate<N>(x, acc);
    }
    double *red = sh.pr; // [kTinyThreads / 64][P], free until the bandwidth computation's first barrier
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const float v = wave_sum(acc[p]);
        if (lane == 0) red[wave * P + p] = (double)v;
    }
    __syncthreads();
    if (tid < P) {
        double s = 0.0;
        for (int w = 0; w < kTinyThreads / 64; ++w) s += red[w * P + tid];
        sh.S[tid] = s;
    }

    // pass 2
    const double h = bandwidth_from_sums<kTinyThreads>(sh, N, kModeDiff, h_fixed, st, coef, cl);
    __syncthreads();
    const float c2h = (N == 1) ? 0.f : (float)(2.0 / h);

    if constexpr (WHAT == kTinyBandwidth) return;

    // pass 3: every thread re-reads the columns it summed (cache hits) and updates them; all
    // reads of pass 1 lie before the barriers above, so in place is safe
    for (int64_t grp = tid; grp < ngroups; grp += kTinyThreads) {
        const int64_t col = grp << 2;
        const bool full = (col + 4 <= D);
        f32x4 x[N], z[N];
#pragma unroll
        for (int j = 0; j < N; ++j) {
            x[j] = load4(X + (int64_t)j * ld, col, D, full);
            z[j] = load4(G + (int64_t)j * ld, col, D, full);
        }
#pragma unroll
        for (int j = 0; j < N; ++j) z[j] -= c2h * x[j];
#pragma unroll
        for (int i = 0; i < N; ++i) {
            f32x4 a = cl[N * N + i] * x[i];
#pragma unroll
            for (int j = 0; j < N; ++j) a += cl[i * N + j] * z[j];
            if constexpr (WHAT == kTinyPhi)
                store4(PHI + (int64_t)i * ld, col, D, full, a);
            else
                store4(X + (int64_t)i * ld, col, D, full, x[i] + eps * a);
        }
    }
}

} // namespace svgd
