// Pass 2: from the reduced pair sums to d2, the median-heuristic bandwidth h, the RBF kernel
// matrix K, its row sums, and the coefficient tables of the update kernels.  One workgroup,
// fp64 throughout (at most 2016 pairs: the cost is nil and none of the 1e-5 budget on h and K
// is spent here).  Nothing returns to the host: the paper's routine (App. B.2) reads each kernel
// value back to the host, one synchronisation per pair; here K stays on the device.
#pragma once
#include "common.hpp"

namespace svgd {

constexpr int kBwThreads = 1024;
constexpr int kSlices = 8; // slices of the partial reduction (see reduce_partials_kernel)

__device__ inline int pair_index(int i, int j, int n) { return i * n - (i * (i + 1)) / 2 + (j - i - 1); } // i < j

// LDS of the bandwidth computation.
struct BwShared {
    double S[kMaxPairsFull];            // reduced sums, sort exchange, K per pair
    double pr[kMaxN * (kMaxN - 1) / 2]; // d2 per unordered pair i < j (free for other use before)
    double sel[2];
    double h;
};

// From the reduced pair sums in sh.S[0 .. n(n+1)/2) to h, K and the coefficient tables.  Called by
// all THREADS threads of a workgroup (2 * THREADS >= n(n-1)/2 rounded up to a power of two), which
// have written sh.S before (no barrier needed in between).  coef_lds, if not null, receives C [n*n] and rho [n] as well (LDS of the caller);
// on return the writes to it still need a barrier.
template <int THREADS>
__device__ inline void bandwidth_from_sums(BwShared &sh, int n, int mode, double h_fixed,
                                           DevState *__restrict__ st, float *__restrict__ coef,
                                           float *coef_lds)
{
    static_assert(THREADS % 64 == 0 && 2 * THREADS <= kMaxPairsFull, "the sort exchanges 2 * THREADS values through S");
    const int tid = threadIdx.x;
    const int Pp = n * (n - 1) / 2;
    if (tid < 2) sh.sel[tid] = 0.0;
    __syncthreads();

    // d2 per pair: direct sums, or S_ii + S_jj - 2 S_ij (clamped at 0) from the centred Gram
    for (int i = tid >> 6; i < n; i += THREADS / 64) {   // wave -> row, lane -> column
        for (int j = i + 1 + (tid & 63); j < n; j += 64) {
            double d;
            if (mode == kModeDiff) {
                d = sh.S[tri(i, j, n)];
            } else {
                d = sh.S[tri(i, i, n)] + sh.S[tri(j, j, n)] - 2.0 * sh.S[tri(i, j, n)];
            }
            if (!(d > 0.0)) d = 0.0; // clamps rounding negatives (and -0.0)
            sh.pr[pair_index(i, j, n)] = d;
        }
    }
    __syncthreads();

    // Median of the multiset of all n*n entries of d2: n diagonal zeros plus every pair value
    // twice.  Sorted position t of the full list is 0 for t < n and the ((t-n)/2)-th smallest
    // pair value otherwise; an even count averages positions n*n/2 - 1 and n*n/2.  S is free by
    // now and serves as the exchange buffer of the sort.
    if (h_fixed <= 0.0 && Pp > 0) {
        // Bitonic sort of the pair values, two per thread in registers (padded with +inf to a
        // power of two M <= 2 * THREADS).  Thread t owns elements 2t and 2t+1; a stage at
        // distance j pairs element i with i^j: inside the thread for j = 1, in lane t ^ (j/2) of
        // the same wave for j <= 64 (shuffles), through LDS for wider stages (10 of the 66
        // stages at M = 2048).  (Eight values per thread with every stage inside a thread and
        // LDS re-deals in between was measured slower: too few waves to hide the latencies.)
        int M = 2;
        while (M < Pp) M <<= 1;
        double e0 = (2 * tid < Pp) ? sh.pr[2 * tid] : __builtin_huge_val();
        double e1 = (2 * tid + 1 < Pp) ? sh.pr[2 * tid + 1] : __builtin_huge_val();
        // waves that hold nothing but padding sit the stages out (they still meet the barriers)
        const bool act = 2 * (tid & ~63) < M;
        for (int k = 2; k <= M; k <<= 1) {
            const bool up = (((2 * tid) & k) == 0); // same for both elements (k >= 2)
            for (int j = k >> 1; j > 0; j >>= 1) {
                const int half = j >> 1;
                double p0 = e1, p1 = e0; // j == 1: the partner is the thread's other element
                if (half >= 64) {
                    if (act) {
                        sh.S[2 * tid] = e0;
                        sh.S[2 * tid + 1] = e1;
                    }
                    __syncthreads();
                    if (act) {
                        const int tp = tid ^ half;
                        p0 = sh.S[2 * tp];
                        p1 = sh.S[2 * tp + 1];
                    }
                    __syncthreads();
                } else if (act && half > 0) {
                    p0 = __shfl_xor(e0, half, kWave);
                    p1 = __shfl_xor(e1, half, kWave);
                }
                if (act) {
                    // the lower element of an ascending pair keeps the minimum
                    const bool low0 = (j == 1) ? true : ((tid & half) == 0);
                    const bool low1 = (j == 1) ? false : low0;
                    e0 = (low0 == up) ? fmin(e0, p0) : fmax(e0, p0);
                    e1 = (low1 == up) ? fmin(e1, p1) : fmax(e1, p1);
                }
            }
        }
        sh.S[2 * tid] = e0;
        sh.S[2 * tid + 1] = e1;
        __syncthreads();
        if (tid == 0) {
            const int n2 = n * n;
            const int t_lo = (n2 - 1) / 2, t_hi = n2 / 2;
            sh.sel[0] = (t_lo >= n) ? sh.S[(t_lo - n) / 2] : 0.0;
            sh.sel[1] = (t_hi >= n) ? sh.S[(t_hi - n) / 2] : 0.0;
        }
    }
    __syncthreads();
    if (tid == 0) {
        double med = 0.5 * (sh.sel[0] + sh.sel[1]);
        double h = (h_fixed > 0.0) ? h_fixed : med / log((double)n + 1.0);
        if (!(h > 0.0)) h = 1.0;
        sh.h = h;
        st->h = h;
        st->med = med;
        // a single particle has no repulsive term at all: make that exact (phi = g)
        st->two_over_h = (n == 1) ? 0.f : (float)(2.0 / h);
        st->n = n;
    }
    __syncthreads();
    const double h = sh.h;
    const double c2h = (n == 1) ? 0.0 : 2.0 / h;
    const double inv_n = 1.0 / (double)n;

    for (int e = tid; e < Pp; e += THREADS) sh.S[e] = exp(-sh.pr[e] / h); // K per pair, reusing S
    __syncthreads();
    for (int i = tid >> 6; i < n; i += THREADS / 64) {   // wave -> row, lane -> column
        double r = 0.0;
        for (int j = tid & 63; j < n; j += 64) {
            const double k = (i == j) ? 1.0 : sh.S[i < j ? pair_index(i, j, n) : pair_index(j, i, n)];
            r += k;
            coef[kOffK + i * n + j] = (float)k;
            coef[kOffC + i * n + j] = (float)(k * inv_n);
            if (coef_lds) coef_lds[i * n + j] = (float)(k * inv_n);
        }
#pragma unroll
        for (int d = 32; d > 0; d >>= 1) r += __shfl_xor(r, d, kWave); // row sum of K
        if ((tid & 63) == 0) {
            const float rho = (float)(c2h * r * inv_n);
            coef[kOffRho + i] = rho;
            if (coef_lds) coef_lds[n * n + i] = rho;
        }
    }
    // A operands of v_mfma_f32_16x16x4_f32 for the matrix-core update kernel: for output block
    // bi and step s = 4b + r, lane (q = lane/16, m = lane%16) holds C[16bi + m][16b + 4q + r].
    if (n > kValuMaxN) {
        const int NB = (n + 15) / 16;
        const int total = NB * 4 * NB * kWave;
        for (int e = tid; e < total; e += THREADS) {
            const int lane = e & 63;
            const int s = (e >> 6) % (4 * NB);
            const int bi = (e >> 6) / (4 * NB);
            const int i = 16 * bi + (lane & 15);
            const int j = 16 * (s >> 2) + 4 * (lane >> 4) + (s & 3);
            double c = 0.0;
            if (i < n && j < n)
                c = ((i == j) ? 1.0 : sh.S[i < j ? pair_index(i, j, n) : pair_index(j, i, n)]) * inv_n;
            coef[kOffAT + e] = (float)c;
        }
    }
}

// A short list of partials (at most kDirectMaxFloats values, P <= kBwThreads) is summed by this
// kernel itself, straight from the fp32 partials, which saves the launch of the reduction kernel;
// `partials` is null otherwise and the sums come from part2.
constexpr int kDirectMaxFloats = 96 * 1024;

__global__ __launch_bounds__(kBwThreads) void bandwidth_kernel(const double *__restrict__ part2,
                                                               const float *__restrict__ partials,
                                                               int nparts, int n, int mode,
                                                               double h_fixed,
                                                               DevState *__restrict__ st,
                                                               float *__restrict__ coef)
{
    __shared__ BwShared sh;

    const int tid = threadIdx.x;
    const int P = n * (n + 1) / 2;

    if (partials != nullptr) {
        // Thread tid = kk * P + pp (kk < KL <= threads / P) sums the partials kk, kk + KL, ... of
        // entry pp: consecutive threads read consecutive floats, 16 loads in flight each; the KL
        // sums of an entry meet in LDS (sh.pr is not in use yet).
        const int KL = kBwThreads / P < 32 ? kBwThreads / P : 32; // capped: the KL sums are added serially
        const int kk = tid / P, pp = tid - kk * P;
        double s = 0.0;
        if (kk < KL) {
            constexpr int U = 16;
            const float *src = partials + tid; // element (kk, pp); partial k + KL is KL * P floats on
            const int64_t stride = (int64_t)KL * P;
            int k = kk;
            for (; k + (U - 1) * KL < nparts; k += U * KL) {
                float v[U];
#pragma unroll
                for (int u = 0; u < U; ++u) v[u] = src[(int64_t)u * stride];
#pragma unroll
                for (int u = 0; u < U; ++u) s += (double)v[u];
                src += U * stride;
            }
            if (k < nparts) { // the last, partly filled batch: loads clamped to the last partial
                float v[U];
                const int left = (nparts - 1 - k) / KL; // index of the last valid load
#pragma unroll
                for (int u = 0; u < U; ++u) v[u] = src[(int64_t)(u < left ? u : left) * stride];
#pragma unroll
                for (int u = 0; u < U; ++u) s += (u <= left) ? (double)v[u] : 0.0;
            }
        }
        sh.pr[tid] = s;
        __syncthreads();
        if (tid < P) {
            double t = 0.0;
            for (int q = 0; q < KL; ++q) t += sh.pr[q * P + tid];
            sh.S[tid] = t;
        }
    } else {
        // part2 always holds kSlices slices (empty ones are zero): a fixed trip count lets all
        // the loads of one entry issue together instead of one latency after the other
        for (int p = tid; p < P; p += kBwThreads) {
            double v[kSlices];
#pragma unroll
            for (int k = 0; k < kSlices; ++k) v[k] = part2[(int64_t)k * P + p];
            double s = 0.0;
#pragma unroll
            for (int k = 0; k < kSlices; ++k) s += v[k];
            sh.S[p] = s;
        }
    }
    bandwidth_from_sums<kBwThreads>(sh, n, mode, h_fixed, st, coef, nullptr);
}

} // namespace svgd
