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
constexpr int kSelDirect = 128; // a set of at most this many values is ranked directly

struct BwShared {
    double S[kMaxPairsFull];            // reduced pair sums, later K per pair
    double pr[kMaxN * (kMaxN - 1) / 2]; // d2 per unordered pair i < j (free for other use before)
    double sel[2];
    double h;
    // scratch of the median selection (select_two_ranks)
    unsigned long long mm[4];           // min / max bit patterns, two alternating slots
    double list[kSelDirect];            // the final short list
    unsigned hist[1024];                // bucket counts, one bucket per thread
    unsigned counters[kSelDirect];      // partial ranks of the list elements
    unsigned misc[16];                  // 0: list length, 1: bucket of r_lo, 2: bucket of r_hi, 3: values below it, 4: its count
    unsigned wsum[16];                  // wave totals of the bucket counts
};

// A double moved across lanes by a DPP control word (both halves).
template <int CTRL>
__device__ inline double dpp_f64(double v)
{
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __builtin_amdgcn_update_dpp(0, lo, CTRL, 0xF, 0xF, false);
    hi = __builtin_amdgcn_update_dpp(0, hi, CTRL, 0xF, 0xF, false);
    return __hiloint2double(hi, lo);
}

__device__ inline double readlane_f64(double v, int lane)
{
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), lane),
                            __builtin_amdgcn_readlane(__double2loint(v), lane));
}

// Minimum and maximum over the 64 lanes of a wave, returned in every lane (four DPP steps inside
// each row of 16 lanes, then the four rows; no LDS traffic).
__device__ inline void wave_minmax(double &mn, double &mx)
{
#define SVGD_MM_STEP(C)                                                                            \
    mn = fmin(mn, dpp_f64<C>(mn));                                                                 \
    mx = fmax(mx, dpp_f64<C>(mx));
    SVGD_MM_STEP(0xB1)  // quad_perm [1,0,3,2]
    SVGD_MM_STEP(0x4E)  // quad_perm [2,3,0,1]
    SVGD_MM_STEP(0x141) // row_half_mirror
    SVGD_MM_STEP(0x140) // row_mirror
#undef SVGD_MM_STEP
    mn = fmin(fmin(readlane_f64(mn, 0), readlane_f64(mn, 16)), fmin(readlane_f64(mn, 32), readlane_f64(mn, 48)));
    mx = fmax(fmax(readlane_f64(mx, 0), readlane_f64(mx, 16)), fmax(readlane_f64(mx, 32), readlane_f64(mx, 48)));
}

// Sum over the 64 lanes of a wave, returned in every lane (same steps as wave_minmax).
__device__ inline double wave_sum_f64(double v)
{
    v += dpp_f64<0xB1>(v);
    v += dpp_f64<0x4E>(v);
    v += dpp_f64<0x141>(v);
    v += dpp_f64<0x140>(v);
    return (readlane_f64(v, 0) + readlane_f64(v, 16)) + (readlane_f64(v, 32) + readlane_f64(v, 48));
}

// Inclusive prefix sum over the 64 lanes of a wave: four DPP shift-adds inside each row of 16
// lanes, then the totals of the lower rows (read from lanes 15, 31, 47) are added to the upper ones.
__device__ inline unsigned wave_inclusive_scan(unsigned x)
{
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xF, 0xF, true); // row_shr:1, 0 shifted in
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xF, 0xF, true); // row_shr:2
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xF, 0xF, true); // row_shr:4
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xF, 0xF, true); // row_shr:8
    const unsigned t0 = (unsigned)__builtin_amdgcn_readlane((int)x, 15);
    const unsigned t1 = (unsigned)__builtin_amdgcn_readlane((int)x, 31);
    const unsigned t2 = (unsigned)__builtin_amdgcn_readlane((int)x, 47);
    const int row = (threadIdx.x & 63) >> 4;
    return x + (row >= 1 ? t0 : 0u) + (row >= 2 ? t1 : 0u) + (row >= 3 ? t2 : 0u);
}

// The pair values of rank r_lo and r_hi (0-based, r_hi = r_lo or r_lo + 1) among sh.pr[0 .. Pp),
// written to sh.sel[0] and sh.sel[1].  Exact selection without sorting:
//   - a small set (<= kSelDirect values) is ranked directly: every element counts how many others
//     precede it (ties by position), and the elements of the wanted ranks announce themselves;
//   - a larger one is spread over THREADS buckets by value, bucket(v) = floor((v - a) * THREADS /
//     (b - a)) clamped, [a, b] = minimum and maximum of the set - monotone in v, so all of bucket
//     k lies below all of bucket k + 1; the bucket counts are prefix-summed, and the bucket that
//     holds the wanted ranks becomes the active set (gathered into a list once it is small).
//     a and b fall into the first and the last bucket, so the set shrinks at every level.  Ranks
//     that fall into two different buckets are the maximum of the one and the minimum of the other.
// With n = 64 (2016 values) this takes one level and a short list; the bitonic sort it replaces
// cost 66 exchange stages.  Everything that crosses waves goes through LDS atomics and a barrier
// (four barriers on the usual path); inside a wave only DPP moves are used - cross-lane reads
// through LDS cost as much as a barrier here.
// Contract: called by all THREADS threads with kSelDirect < Pp <= 2 * THREADS (smaller sets go to
// rank_directly), after a barrier behind which
//   - sh.pr holds the values (thread t wrote pr[t] and pr[t + THREADS]),
//   - sh.mm[0] / mm[1] hold the bit patterns of their minimum / maximum, mm[2] = ~0, mm[3] = 0,
//   - sh.hist and sh.counters are zero, sh.misc[0] = 0, sh.misc[1..] = ~0
// (bandwidth_from_sums prepares all of this on its way).  Values that are negative or not finite
// cannot be ranked consistently: the loop is bounded and then returns some value of the set.

// Non-negative doubles (and +inf) order like their bit patterns read as unsigned integers.
__device__ inline unsigned long long f64_key(double v) { return (unsigned long long)__double_as_longlong(v); }
__device__ inline double key_f64(unsigned long long k) { return __longlong_as_double((long long)k); }

// minimum and maximum of the calling waves' values into two LDS words: DPP inside the wave, one
// atomic per wave on the bit patterns (mx >= 0)
__device__ inline void minmax_to_lds(double mn, double mx, unsigned long long *slot)
{
    wave_minmax(mn, mx);
    if ((threadIdx.x & 63) == 0) {
        atomicMin(&slot[0], f64_key(mn));
        atomicMax(&slot[1], f64_key(mx));
    }
}

// Rank (position in sorted order, ties by index) of every element of a short list (len <=
// kSelDirect); the elements of the wanted ranks are stored to sel.  THREADS / kSelDirect threads
// share one element, each comparing it with a slice of the list (a single thread walking the
// whole list would wait for one LDS round trip after the other); the partial ranks meet in
// `counters`, which must be zero on entry.  list_visible: a barrier already lies between the
// writes of the list and this call.
// Workgroup barrier.  LO ("LDS only"): for code whose barriers order nothing but LDS traffic -
// it waits for this wave's LDS operations and not for its outstanding global loads, which
// __syncthreads() would (the fused step has its first tile's loads in flight during pass 2).
template <bool LO>
__device__ inline void block_sync()
{
    if constexpr (LO) asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    else __syncthreads();
}

template <int THREADS, bool LO = false>
__device__ inline void rank_directly(const double *list, int len, int below, int r_lo, int r_hi, double *sel,
                                     unsigned *counters, bool list_visible)
{
    constexpr int PARTS = THREADS / kSelDirect;             // threads per element
    constexpr int SLICE = (kSelDirect + PARTS - 1) / PARTS; // list entries per thread
    static_assert(PARTS >= 1 && PARTS * kSelDirect == THREADS, "THREADS is a multiple of kSelDirect");
    const int tid = threadIdx.x;
    const int e = tid % kSelDirect, part = tid / kSelDirect;
    if (!list_visible) block_sync<LO>();
    double v = 0.0;
    if (e < len) {
        v = list[e];
        unsigned cnt = 0;
        const int u0 = part * SLICE;
#pragma unroll
        for (int k = 0; k < SLICE; ++k) {
            const int u = u0 + k;
            if (u < len) {
                const double w = list[u];
                cnt += (w < v || (w == v && u < e)) ? 1u : 0u;
            }
        }
        if (cnt) atomicAdd(&counters[e], cnt);
    }
    block_sync<LO>();
    if (part == 0 && e < len) {
        const int rank = below + (int)counters[e];
        if (rank == r_lo) sel[0] = v;
        if (rank == r_hi) sel[1] = v;
    }
}

template <int THREADS, bool LO = false>
__device__ inline void select_two_ranks(BwShared &sh, int Pp, int r_lo, int r_hi)
{
    static_assert(THREADS % 64 == 0 && THREADS >= 256 && THREADS <= 1024, "one bucket per thread, at most 16 waves");
    constexpr int NW = THREADS / 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const unsigned long long kmax = ~0ull;
    const double inf = __builtin_huge_val();

    // every thread owns up to two values
    const double e0 = (tid < Pp) ? sh.pr[tid] : 0.0;
    const double e1 = (tid + THREADS < Pp) ? sh.pr[tid + THREADS] : 0.0;
    bool act0 = tid < Pp, act1 = tid + THREADS < Pp;
    int below = 0; // values known to be smaller than the whole active set
    int cnt = Pp;  // size of the active set

    for (int level = 0; level < 12; ++level) {
        const int slot = (level & 1) * 2;
        if (level > 0) {
            // refine: clear what the previous level used (its last reads lie behind the barrier at
            // its end), find the range of the narrowed set
            sh.hist[tid] = 0;
            if (tid < 16) sh.misc[tid] = (tid == 0) ? 0u : 0xFFFFFFFFu;
            if (tid == 0) { // the other slot, for the level after this one
                sh.mm[2 - slot] = kmax;
                sh.mm[3 - slot] = 0ull;
            }
            minmax_to_lds(fmin(act0 ? e0 : inf, act1 ? e1 : inf), fmax(act0 ? e0 : 0.0, act1 ? e1 : 0.0), &sh.mm[slot]);
            block_sync<LO>();
        }
        const double a = key_f64(sh.mm[slot]), b = key_f64(sh.mm[slot + 1]);
        if (!(a < b)) { // all active values equal (or nothing rankable): both ranks are a
            if (tid == 0) {
                sh.sel[0] = a;
                sh.sel[1] = a;
            }
            return;
        }
        // spread the active values over THREADS buckets
        const double scale = (double)THREADS / (b - a);
        auto bucket = [&](double v) {
            const int k = (int)((v - a) * scale);
            return k < 0 ? 0 : (k > THREADS - 1 ? THREADS - 1 : k);
        };
        const int k0 = act0 ? bucket(e0) : 0, k1 = act1 ? bucket(e1) : 0;
        if (act0) atomicAdd(&sh.hist[k0], 1u);
        if (act1) atomicAdd(&sh.hist[k1], 1u);
        block_sync<LO>();
        // inclusive prefix sum of the bucket counts: DPP inside the wave, wave totals through LDS
        const unsigned mine = sh.hist[tid];
        unsigned incl = wave_inclusive_scan(mine);
        if (lane == 63) sh.wsum[wave] = incl;
        block_sync<LO>();
        unsigned before = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) before += (w < wave) ? sh.wsum[w] : 0u;
        incl += before;
        const unsigned excl = incl - mine;
        // the buckets holding the wanted ranks (ranks relative to the active set)
        const unsigned q_lo = (unsigned)(r_lo - below), q_hi = (unsigned)(r_hi - below);
        if (mine > 0 && excl <= q_lo && q_lo < incl) {
            sh.misc[1] = (unsigned)tid;
            sh.misc[3] = excl;
            sh.misc[4] = mine;
        }
        if (mine > 0 && excl <= q_hi && q_hi < incl) sh.misc[2] = (unsigned)tid;
        block_sync<LO>();
        const unsigned b_lo = sh.misc[1], b_hi = sh.misc[2];
        if (b_lo == 0xFFFFFFFFu || b_hi == 0xFFFFFFFFu) break; // unrankable input
        if (b_lo != b_hi) {
            // adjacent ranks in different buckets: the largest value of the one, the smallest of the
            // other (the other min/max slot is prepared and unused at this point)
            double mx = 0.0, mn = inf;
            if (act0 && (unsigned)k0 == b_lo) mx = fmax(mx, e0);
            if (act1 && (unsigned)k1 == b_lo) mx = fmax(mx, e1);
            if (act0 && (unsigned)k0 == b_hi) mn = fmin(mn, e0);
            if (act1 && (unsigned)k1 == b_hi) mn = fmin(mn, e1);
            minmax_to_lds(mn, mx, &sh.mm[2 - slot]);
            block_sync<LO>();
            if (tid == 0) {
                sh.sel[0] = key_f64(sh.mm[3 - slot]);
                sh.sel[1] = key_f64(sh.mm[2 - slot]);
            }
            return;
        }
        below += (int)sh.misc[3];
        cnt = (int)sh.misc[4];
        act0 = act0 && (unsigned)k0 == b_lo;
        act1 = act1 && (unsigned)k1 == b_lo;
        if (cnt <= kSelDirect) { // gather the bucket into a list and rank it
            if (act0) sh.list[atomicAdd(&sh.misc[0], 1u)] = e0;
            if (act1) sh.list[atomicAdd(&sh.misc[0], 1u)] = e1;
            rank_directly<THREADS, LO>(sh.list, cnt, below, r_lo, r_hi, sh.sel, sh.counters, false);
            return;
        }
        block_sync<LO>(); // all reads of misc, hist and wsum are done before the next level clears them
    }
    if (tid == 0) {
        sh.sel[0] = sh.pr[0];
        sh.sel[1] = sh.pr[0];
    }
}

// From the reduced pair sums in sh.S[0 .. n(n+1)/2) to h, K and the coefficient tables.  Called by
// all THREADS threads of a workgroup (n(n-1)/2 <= 2 * THREADS), which have written sh.S before (no
// barrier needed in between).  coef_lds, if not null, receives C [n*n] and rho [n] as well (LDS of
// the caller); on return the writes to it still need a barrier.  write_global = false: st and coef
// (device memory) are left alone - for workgroups that repeat the computation of another one.
// Returns h (in every thread).
template <int THREADS, bool LO = false>
__device__ inline double bandwidth_from_sums(BwShared &sh, int n, int mode, double h_fixed,
                                           DevState *__restrict__ st, float *__restrict__ coef,
                                           float *coef_lds, bool write_global = true)
{
    static_assert(THREADS % 64 == 0 && THREADS <= 1024, "whole waves, one histogram bucket per thread");
    const int tid = threadIdx.x;
    const int Pp = n * (n - 1) / 2;
    const bool select = h_fixed <= 0.0 && Pp > 0;
    const bool buckets = select && Pp > kSelDirect; // the selection will work with buckets
    // the selection's scratch in its initial state (see select_two_ranks)
    if (tid < 2) sh.sel[tid] = 0.0;
    if (tid < kSelDirect) sh.counters[tid] = 0;
    if (buckets) {
        sh.hist[tid] = 0;
        if (tid < 16) sh.misc[tid] = (tid == 0) ? 0u : 0xFFFFFFFFu;
        if (tid < 4) sh.mm[tid] = (tid & 1) ? 0ull : ~0ull;
    }
    block_sync<LO>();

    // d2 per pair: direct sums, or S_ii + S_jj - 2 S_ij (clamped at 0) from the centred Gram.
    // Thread p takes pair p: row i is the largest one whose first pair index, i (2n - i - 1) / 2,
    // does not exceed p (estimate from the quadratic, then corrected).
    double dmin = __builtin_huge_val(), dmax = 0.0;
    for (int p = tid; p < Pp; p += THREADS) {
        const float tn = (float)(2 * n - 1);
        int i = (int)(0.5f * (tn - sqrtf(fmaxf(tn * tn - 8.0f * (float)p, 0.0f))));
        i = i < 0 ? 0 : (i > n - 2 ? n - 2 : i);
        while (i > 0 && pair_index(i, i + 1, n) > p) --i;
        while (i < n - 2 && pair_index(i + 1, i + 2, n) <= p) ++i;
        const int j = i + 1 + (p - pair_index(i, i + 1, n));
        double d;
        if (mode == kModeDiff) {
            d = sh.S[tri(i, j, n)];
        } else {
            d = sh.S[tri(i, i, n)] + sh.S[tri(j, j, n)] - 2.0 * sh.S[tri(i, j, n)];
        }
        if (!(d > 0.0)) d = 0.0; // clamps rounding negatives (and -0.0, and NaN)
        sh.pr[p] = d;
        dmin = fmin(dmin, d);
        dmax = fmax(dmax, d);
    }
    if (buckets) minmax_to_lds(dmin, dmax, &sh.mm[0]); // the range of all values, for the first level
    block_sync<LO>();

    // Median of the multiset of all n*n entries of d2: n diagonal zeros plus every pair value
    // twice.  Sorted position t of the full list is 0 for t < n and the ((t-n)/2)-th smallest
    // pair value otherwise; an even count averages positions n*n/2 - 1 and n*n/2.  So what is
    // needed are the pair values of rank r_lo and r_hi (equal or adjacent), not a sorted list.
    const int t_lo = (n * n - 1) / 2, t_hi = (n * n) / 2; // t_hi >= n for every n >= 2
    if (select) {
        // n = 2: position t_lo is one of the diagonal zeros - the other rank is selected twice
        const int r_lo = (t_lo >= n) ? (t_lo - n) / 2 : (t_hi - n) / 2, r_hi = (t_hi - n) / 2;
        if (buckets) select_two_ranks<THREADS, LO>(sh, Pp, r_lo, r_hi);
        else rank_directly<THREADS, LO>(sh.pr, Pp, 0, r_lo, r_hi, sh.sel, sh.counters, true);
    }
    block_sync<LO>();
    if (tid == 0) { // one thread derives h (a logarithm and two divisions in fp64), LDS hands it on
        const double med = 0.5 * ((t_lo >= n ? sh.sel[0] : 0.0) + sh.sel[1]);
        double hh = (h_fixed > 0.0) ? h_fixed : med / log((double)n + 1.0);
        if (!(hh > 0.0)) hh = 1.0;
        sh.h = hh;
        if (write_global) {
            st->h = hh;
            st->med = med;
            // a single particle has no repulsive term at all: make that exact (phi = g)
            st->two_over_h = (n == 1) ? 0.f : (float)(2.0 / hh);
            st->n = n;
        }
    }
    block_sync<LO>();
    const double h = sh.h;
    const double c2h = (n == 1) ? 0.0 : 2.0 / h;
    const double inv_n = 1.0 / (double)n;
    const double neg_inv_h = -1.0 / h;

    for (int e = tid; e < Pp; e += THREADS) sh.S[e] = exp(sh.pr[e] * neg_inv_h); // K per pair, reusing S
    block_sync<LO>();
    // K, C, row sums: wave -> row, lane -> column.  K_ij and K_ji are the same LDS entry, so K is
    // exactly symmetric; the diagonal is exactly 1.
    for (int i = tid >> 6; i < n; i += THREADS / 64) {
        double r = 0.0;
        for (int j = tid & 63; j < n; j += 64) {
            const double k = (i == j) ? 1.0 : sh.S[i < j ? pair_index(i, j, n) : pair_index(j, i, n)];
            r += k;
            if (write_global) {
                coef[kOffK + i * n + j] = (float)k;
                coef[kOffC + i * n + j] = (float)(k * inv_n);
            }
            if (coef_lds) coef_lds[i * n + j] = (float)(k * inv_n);
        }
        r = wave_sum_f64(r); // row sum of K
        if ((tid & 63) == 0) {
            const float rho = (float)(c2h * r * inv_n);
            if (write_global) coef[kOffRho + i] = rho;
            if (coef_lds) coef_lds[n * n + i] = rho;
        }
    }
    return h;
}

// The whole of pass 2 as the prologue of an update kernel (fused step): every workgroup sums the
// short list of partials that the previous update left behind and derives h, K, C and rho for
// itself, C [n*n] and rho [n] into coef_lds (LDS of the caller, barrier included); the workgroup
// with write_global also records them in st and coef for svgd_get_last.  Returns h.  THREADS
// threads, n <= 32 (n(n-1)/2 <= 2 * THREADS).  A workgroup costs what the bandwidth kernel costs, but
// all of them run at once and the launch, with its gap, is gone.
// after_sums() is called once the list has been read and before the arithmetic that needs no
// memory: the place for the caller to send off loads of its own (issued earlier they would only
// make the list wait behind them - a wave's loads complete in order).
struct NoCall {
    __device__ void operator()() const {}
};
template <int THREADS, class AfterSums = NoCall>
__device__ inline double kernel_matrix_prologue(BwShared &sh, const float *__restrict__ partials, int nparts, int n,
                                                int mode, double h_fixed, DevState *__restrict__ st,
                                                float *__restrict__ coef, float *coef_lds, bool write_global,
                                                AfterSums after_sums = AfterSums{})
{
    const int P = n * (n + 1) / 2;
    constexpr int U = 16; // loads in flight per thread
    if (2 * P <= THREADS) {
        // few pairs: thread (kk, pp) = (tid / P, tid % P), kk < KL, sums the partials kk, kk + KL, ...
        // of entry pp (consecutive threads read consecutive floats); the KL sums of an entry meet
        // in LDS (sh.pr is not in use yet)
        const int KL = THREADS / P < 32 ? THREADS / P : 32;
        const int tid = threadIdx.x, kk = tid / P, pp = tid - kk * P;
        double s = 0.0;
        if (kk < KL) {
            for (int k = kk; k < nparts; k += U * KL) {
                float v[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int ku = k + u * KL;
                    v[u] = partials[(int64_t)(ku < nparts ? ku : nparts - 1) * P + pp];
                }
#pragma unroll
                for (int u = 0; u < U; ++u) s += (k + u * KL < nparts) ? (double)v[u] : 0.0;
            }
            sh.pr[tid] = s;
        }
        __syncthreads();
        if (tid < P) {
            double t = 0.0;
            for (int q = 0; q < KL; ++q) t += sh.pr[q * P + tid];
            sh.S[tid] = t;
        }
    } else {
        for (int pp = threadIdx.x; pp < P; pp += THREADS) { // consecutive threads read consecutive floats
            double s = 0.0;
            for (int k = 0; k < nparts; k += U) {
                float v[U];
#pragma unroll
                for (int u = 0; u < U; ++u) v[u] = partials[(int64_t)(k + u < nparts ? k + u : nparts - 1) * P + pp];
#pragma unroll
                for (int u = 0; u < U; ++u) s += (k + u < nparts) ? (double)v[u] : 0.0;
            }
            sh.S[pp] = s;
        }
    }
    after_sums();
    const double h = bandwidth_from_sums<THREADS, true>(sh, n, mode, h_fixed, st, coef, coef_lds, write_global);
    block_sync<true>();
    return h;
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
        const int kk = tid / P; // (pp = tid - kk * P)
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
