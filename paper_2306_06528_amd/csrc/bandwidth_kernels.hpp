// Pass 2: from the reduced pair sums to d2, the median-heuristic bandwidth h, the RBF kernel
// matrix K, its row sums, and the coefficient tables of the update kernels.  One workgroup,
// fp64 throughout (at most 2016 pairs: the cost is nil and none of the 1e-5 budget on h and K
// is spent here).  Nothing returns to the host: the paper's routine (App. B.2) reads each kernel
// value back with `.item()`; here K stays on the device.
#pragma once
#include "common.hpp"

namespace svgd {

constexpr int kBwThreads = 1024;
constexpr int kSlices = 32; // slices of the partial reduction (see reduce_partials_kernel)

__device__ inline int pair_index(int i, int j, int n) { return i * n - (i * (i + 1)) / 2 + (j - i - 1); } // i < j

__global__ __launch_bounds__(kBwThreads) void bandwidth_kernel(const double *__restrict__ part2,
                                                               int n, int mode,
                                                               double h_fixed,
                                                               DevState *__restrict__ st,
                                                               float *__restrict__ coef)
{
    __shared__ double S[kMaxPairsFull];              // reduced sums, later K per pair
    __shared__ double pr[kMaxN * (kMaxN - 1) / 2];   // d2 per unordered pair i < j
    __shared__ double sel[2];
    __shared__ double h_sh;

    const int tid = threadIdx.x;
    const int P = n * (n + 1) / 2;
    const int Pp = n * (n - 1) / 2;

    // part2 always holds kSlices slices (empty ones are zero): a fixed trip count lets all the
    // loads of one entry issue together instead of one latency after the other
    for (int p = tid; p < P; p += kBwThreads) {
        double v[kSlices];
#pragma unroll
        for (int k = 0; k < kSlices; ++k) v[k] = part2[(int64_t)k * P + p];
        double s = 0.0;
#pragma unroll
        for (int k = 0; k < kSlices; ++k) s += v[k];
        S[p] = s;
    }
    if (tid < 2) sel[tid] = 0.0;
    __syncthreads();

    // d2 per pair: direct sums, or S_ii + S_jj - 2 S_ij (clamped at 0) from the centred Gram
    for (int i = tid >> 6; i < n; i += kBwThreads / 64) {   // wave -> row, lane -> column
        for (int j = i + 1 + (tid & 63); j < n; j += 64) {
            double d;
            if (mode == kModeDiff) {
                d = S[tri(i, j, n)];
            } else {
                d = S[tri(i, i, n)] + S[tri(j, j, n)] - 2.0 * S[tri(i, j, n)];
            }
            if (!(d > 0.0)) d = 0.0; // clamps rounding negatives (and -0.0)
            pr[pair_index(i, j, n)] = d;
        }
    }
    __syncthreads();

    // Median of the multiset of all n*n entries of d2: n diagonal zeros plus every pair value
    // twice.  Sorted position t of the full list is 0 for t < n and the ((t-n)/2)-th smallest
    // pair value otherwise; an even count averages positions n*n/2 - 1 and n*n/2.  The pair
    // values are sorted by a bitonic network in LDS (S is free by now and serves as the buffer;
    // padded with +inf to a power of two).
    if (h_fixed <= 0.0 && Pp > 0) {
        int M = 1;
        while (M < Pp) M <<= 1;
        for (int e = tid; e < M; e += kBwThreads) S[e] = (e < Pp) ? pr[e] : __builtin_huge_val();
        __syncthreads();
        for (int k = 2; k <= M; k <<= 1) {
            for (int j = k >> 1; j > 0; j >>= 1) {
                for (int e = tid; e < (M >> 1); e += kBwThreads) {
                    const int a = ((e & ~(j - 1)) << 1) | (e & (j - 1)); // bit j clear
                    const int b2 = a | j;
                    const double va = S[a], vb = S[b2];
                    const bool up = ((a & k) == 0);
                    if ((va > vb) == up) {
                        S[a] = vb;
                        S[b2] = va;
                    }
                }
                // M/2 <= kBwThreads, so a thread owns one pair per stage and a wave's 64 pairs at
                // distance j < 64 lie in its own 128-element block: such stages exchange data
                // only inside the wave (whose LDS operations execute in order) and need no barrier
                // unless a wider stage precedes or follows.
                const int next_j = (j > 1) ? (j >> 1) : k;
                if (j >= 64 || next_j >= 64) __syncthreads();
            }
        }
        if (tid == 0) {
            const int n2 = n * n;
            const int t_lo = (n2 - 1) / 2, t_hi = n2 / 2;
            sel[0] = (t_lo >= n) ? S[(t_lo - n) / 2] : 0.0;
            sel[1] = (t_hi >= n) ? S[(t_hi - n) / 2] : 0.0;
        }
    }
    __syncthreads();
    if (tid == 0) {
        double med = 0.5 * (sel[0] + sel[1]);
        double h = (h_fixed > 0.0) ? h_fixed : med / log((double)n + 1.0);
        if (!(h > 0.0)) h = 1.0;
        h_sh = h;
        st->h = h;
        st->med = med;
        // a single particle has no repulsive term at all: make that exact (phi = g)
        st->two_over_h = (n == 1) ? 0.f : (float)(2.0 / h);
        st->n = n;
    }
    __syncthreads();
    const double h = h_sh;
    const double c2h = (n == 1) ? 0.0 : 2.0 / h;
    const double inv_n = 1.0 / (double)n;

    for (int e = tid; e < Pp; e += kBwThreads) S[e] = exp(-pr[e] / h); // K per pair, reusing S
    __syncthreads();
    if (tid < n) {
        double r = 1.0;
        for (int j = 0; j < n; ++j)
            if (j != tid) r += S[tid < j ? pair_index(tid, j, n) : pair_index(j, tid, n)];
        coef[kOffRho + tid] = (float)(c2h * r * inv_n);
    }
    for (int i = tid >> 6; i < n; i += kBwThreads / 64) {   // wave -> row, lane -> column
        for (int j = tid & 63; j < n; j += 64) {
            const double k = (i == j) ? 1.0 : S[i < j ? pair_index(i, j, n) : pair_index(j, i, n)];
            coef[kOffK + i * n + j] = (float)k;
            coef[kOffC + i * n + j] = (float)(k * inv_n);
        }
    }
    // A operands of v_mfma_f32_16x16x4_f32 for the matrix-core update kernel: for output block
    // bi and step s = 4b + r, lane (q = lane/16, m = lane%16) holds C[16bi + m][16b + 4q + r].
    if (n > kValuMaxN) {
        const int NB = (n + 15) / 16;
        const int total = NB * 4 * NB * kWave;
        for (int e = tid; e < total; e += kBwThreads) {
            const int lane = e & 63;
            const int s = (e >> 6) % (4 * NB);
            const int bi = (e >> 6) / (4 * NB);
            const int i = 16 * bi + (lane & 15);
            const int j = 16 * (s >> 2) + 4 * (lane >> 4) + (s & 3);
            double c = 0.0;
            if (i < n && j < n)
                c = ((i == j) ? 1.0 : S[i < j ? pair_index(i, j, n) : pair_index(j, i, n)]) * inv_n;
            coef[kOffAT + e] = (float)c;
        }
    }
}

} // namespace svgd
