// Pairwise squared distances, pass 1: per-workgroup partial sums over a split of the D columns.
//
// Paper App. B.2 computes, per ordered pair, diff = (p_j - p_i)/l and radius^2 = dot(diff, diff).
// Here all pairs are accumulated in ONE pass over X: a thread (or a wave) holds all n values of
// a few columns on chip, adds their contribution to every pair, and moves on.
#pragma once
#include <type_traits>
#include "common.hpp"

namespace svgd {

// ---------------------------------------------------------------------------------------------
// n <= kValuMaxN (12): vector ALU, lanes = columns.  Each thread loads 4 consecutive columns of
// every row (one 16-byte load per row, 1 KiB contiguous per row per wave) and keeps one fp32
// accumulator per pair in registers.
//   N <= 8 : direct differences (x_i - x_j)^2 - no cancellation at all.
//   N  > 8 : Gram of the column-centred y = x - mean_i(x); d2 = S_ii + S_jj - 2 S_ij later.
// Chains are short (D / (4 * threads) terms per accumulator); lanes are combined by DPP adds,
// waves through LDS, workgroups in fp64 by the reduce kernel.
// ---------------------------------------------------------------------------------------------

// One 4-column group's contribution to every pair sum: acc[tri(i, j, N)] += sum over the 4
// columns of (x_i - x_j)^2 (N <= 8) or of y_i y_j, y = x - column mean (N > 8; x is overwritten
// by y).
template <int N>
__device__ __forceinline__ void pair_accumulate(f32x4 (&x)[N], float (&acc)[N * (N + 1) / 2])
{
    constexpr bool kDiff = (N <= 8);
    if constexpr (kDiff) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
#pragma unroll
            for (int j = i + 1; j < N; ++j) {
                const f32x4 d = x[i] - x[j];
                float a = acc[tri(i, j, N)];
                a = fmaf(d.x, d.x, a);
                a = fmaf(d.y, d.y, a);
                a = fmaf(d.z, d.z, a);
                a = fmaf(d.w, d.w, a);
                acc[tri(i, j, N)] = a;
            }
        }
    } else {
        f32x4 m = x[0];
#pragma unroll
        for (int j = 1; j < N; ++j) m += x[j];
        m *= (1.0f / N);
#pragma unroll
        for (int j = 0; j < N; ++j) x[j] -= m; // columns beyond D were loaded as 0 -> stay 0
#pragma unroll
        for (int i = 0; i < N; ++i) {
#pragma unroll
            for (int j = i; j < N; ++j) {
                float a = acc[tri(i, j, N)];
                a = fmaf(x[i].x, x[j].x, a);
                a = fmaf(x[i].y, x[j].y, a);
                a = fmaf(x[i].z, x[j].z, a);
                a = fmaf(x[i].w, x[j].w, a);
                acc[tri(i, j, N)] = a;
            }
        }
    }
}

// STREAM: loads with the streaming hint, see gram_mfma_kernel (here also for unaligned rows: a
// wave covers 1 KiB of a row, the one line it shares with its neighbour matters little).
template <int N, bool ROWS = false, bool STREAM = false>
__global__ __launch_bounds__(256) void gram_valu_kernel(const float *__restrict__ X, int64_t D, int64_t ld,
                                                        float *__restrict__ partials,
                                                        typename RowArg<ROWS>::type rt)
{
    constexpr int P = N * (N + 1) / 2;
    float acc[P];
#pragma unroll
    for (int p = 0; p < P; ++p) acc[p] = 0.f;

    const int64_t ngroups = (D + 3) >> 2;
    const int64_t nthreads = (int64_t)gridDim.x * 256;
    // two column groups per iteration when the registers allow: twice the loads in flight
    constexpr int U = (N <= 8) ? 2 : 1;
    // The columns are walked from the far end: the update that follows walks them from the near
    // end, so each pass starts on the part of X that the pass before it touched last and that the
    // memory-side cache still holds.
    const int64_t grp0 = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t cnt = (grp0 < ngroups) ? (ngroups - 1 - grp0) / (U * nthreads) + 1 : 0;
    for (int64_t k = cnt - 1; k >= 0; --k) {
        const int64_t grp = grp0 + k * U * nthreads;
        f32x4 x[U][N];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t col = (grp + u * nthreads) << 2; // past the end: every load is masked to 0
            const bool full = (col + 4 <= D);
#pragma unroll
            for (int j = 0; j < N; ++j) {
                const float *xr = X + (ROWS ? rt.x[ROWS ? j : 0] : (int64_t)j * ld);
                x[u][j] = STREAM ? load4_stream(xr, col, D, full) : load4(xr, col, D, full);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) pair_accumulate<N>(x[u], acc);
    }

    __shared__ float red[4][P];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const float v = wave_sum(acc[p]);
        if (lane == 0) red[wave][p] = v;
    }
    __syncthreads();
    for (int p = threadIdx.x; p < P; p += 256)
        partials[(int64_t)blockIdx.x * P + p] = (red[0][p] + red[1][p]) + (red[2][p] + red[3][p]);
}

// ---------------------------------------------------------------------------------------------
// kValuMaxN < n <= 64: matrix cores.  The Gram S = Y Y^T of the column-centred Y is a contraction over
// columns, so the MFMA A and B operands are both "lane = (particle row, column slot)".  Loading
// that shape straight from HBM would touch 16 rows per quarter-wave, so each wave instead
//   1. loads a 16*NB-row x 64-column slab with row-contiguous 16-byte loads (256 B per row per
//      quarter-wave), rows {4i + lane/16}, columns 4*(lane%16)..+3,
//   2. centres the columns (own rows in registers, two cross-lane adds for the other rows),
//   3. writes the slab to a wave-private LDS region with a 16-byte-granule XOR swizzle,
//   4. reads it back as v_mfma_f32_16x16x4_f32 operands: lane (q = lane/16, rr = lane%16) takes
//      row 16b+rr, 4 columns per read; the 4 k-slots of one MFMA are columns {16s+4q+c, q=0..3},
//      (the loads of the next slab are issued here, before the multiply phase),
//   5. issues one MFMA per unordered block pair (b <= b'), fp32 accumulators in registers:
//      lane (q, c), register r of pair (b, b') holds S[16b + 4q + r][16b' + c].
// Any assignment of columns to k-slots is valid because every column is summed exactly once.
// ---------------------------------------------------------------------------------------------
// Order of the slabs.  The update re-reads X right after this pass, every wave (or workgroup) of it
// walking a contiguous range of 64-column tiles from the left (tile_range).  What the memory-side
// cache holds of X when the update starts should therefore be the first `hot` tiles of each of
// those `nranges` ranges of `per` tiles, and this pass visits them last: its index space is
//     [0, I1)        the other ("cold") tiles, range after range,
//     [I1, I1 + I2)  the hot tiles, range after range,
//     I1 + I2        the partial slab after the last full tile, if D mod 64 != 0,
// with I1 = nranges * (per - hot), I2 = nranges * hot (indices that fall beyond a short last range
// are empty slabs), and wave w of workgroup b takes the indices 4 (b + k * gridDim.x) + w: the
// workgroups sweep the index space together, the four waves of one on adjacent slabs.
constexpr int kGramWaves = 4; // waves per workgroup, as in the update kernel

// (a wave's indices are `stride` = 4 * gridDim.x apart; its quotient and remainder by the lengths
// of a range's cold and hot parts come from the host, so that stepping from one index to the next
// needs no division; everything fits 32 bits, the host sees to that)
struct GramOrder {
    uint32_t nranges, per, hot;
    uint32_t q_cold, r_cold; // stride = q_cold * (per - hot) + r_cold   (0, 0 if per == hot)
    uint32_t q_hot, r_hot;   // stride = q_hot * hot + r_hot             (0, 0 if hot == 0)
};

// ORDER 0: plain order, index = tile (go is not looked at) - for an X that the memory-side cache
//   holds anyway, or nearly: there the bookkeeping of the order costs more than the order gains.
// ORDER 1: the order described above.
// ORDER 2: the same, and the cold tiles are loaded with the streaming hint (no allocation on the
//   way in) - for rows on 128-byte boundaries (nothing is shared between the slabs of neighbouring
//   waves).  The pass itself then runs 5 % (n = 64, D = 11.2 M) to 28 % (n = 16, same D) faster.
// The host takes ORDER 1 or 2 when X is larger than twice the memory-side cache.
template <int NB, bool ROWS = false, int ORDER = 0>
__global__ __launch_bounds__(64 * kGramWaves) void gram_mfma_kernel(const float *__restrict__ X, int n,
                                                                    int64_t D, int64_t ld, float *__restrict__ partials,
                                                                    typename RowArg<ROWS>::type rt, GramOrder go)
{
    constexpr int NROW = 16 * NB;
    constexpr int RPL = 4 * NB; // rows per lane while loading
    constexpr int NPAIR = NB * (NB + 1) / 2;
    __shared__ float lds[kGramWaves][NROW * 64];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int q = lane >> 4, c16 = lane & 15;
    float *my = lds[wave];
    const float inv_n = 1.0f / (float)n;

    f32x4 acc[NPAIR];
#pragma unroll
    for (int p = 0; p < NPAIR; ++p) acc[p] = f32x4{0.f, 0.f, 0.f, 0.f};

    constexpr bool ORDERED = ORDER != 0, STREAM = ORDER == 2;
    const int64_t nfull = D >> 6;
    const uint32_t uper = go.per, uhot = go.hot, ucold = uper - uhot, unfull = (uint32_t)nfull;
    const uint32_t I1 = ORDERED ? go.nranges * ucold : 0u, I2 = ORDERED ? go.nranges * uhot : unfull;
    const uint32_t nidx = I1 + I2 + (((nfull << 6) < D) ? 1u : 0u);
    const uint32_t lo = 4u * blockIdx.x + (uint32_t)__builtin_amdgcn_readfirstlane(wave), stride = 4u * gridDim.x;
    // the walk: index `at` is tile r * per + o (+ hot while cold), or the partial slab (phase 2)
    uint32_t at = lo, phase = 0, r = 0, o = 0;
    auto enter = [&]() { // state at index `at`, by division: once per wave and phase
        if (at < I1) {
            phase = 0;
            r = at / ucold;
            o = at - r * ucold;
        } else if (at < I1 + I2) {
            phase = 1;
            r = (at - I1) / uhot;
            o = (at - I1) - r * uhot;
        } else {
            phase = 2;
        }
    };
    auto advance = [&]() {
        at += stride;
        if constexpr (ORDERED) {
            if (phase == 0 && at < I1) {
                o += go.r_cold;
                r += go.q_cold;
                if (o >= ucold) { o -= ucold; ++r; }
            } else if (phase == 1 && at < I1 + I2) {
                o += go.r_hot;
                r += go.q_hot;
                if (o >= uhot) { o -= uhot; ++r; }
            } else if (phase < 2) {
                enter();
            }
        }
    };
    if constexpr (ORDERED) enter();
    f32x4 x[RPL];
    int64_t xro[ROWS ? RPL : 1]; // where this lane's rows start (separate rows only)
    if constexpr (ROWS) {
#pragma unroll
        for (int i = 0; i < RPL; ++i) xro[i] = (4 * i + q < n) ? rt.x[ROWS ? 4 * i + q : 0] : 0;
    }
    // The slab at `at` (then on to the next index): where it lies and how it is to be loaded -
    // 0: plain 16-byte loads, 1: streaming ones, 2: the partial slab, 3: an empty slab.  One
    // wave-uniform decision per slab, then sixteen loads in a row: decided per row, every load
    // sat behind its own little tree of branches, a hundred branches per slab during which the
    // matrix pipe had nothing from this wave.
    int64_t col = 0;
    auto next_slab = [&]() __attribute__((always_inline)) -> int {
        const bool is_cold = ORDERED && phase == 0;
        int64_t tile = ORDERED ? nfull : (int64_t)at; // ordered, phase 2: the partial slab
        if (ORDERED && phase < 2) {
            const uint32_t t = r * uper + (is_cold ? uhot : 0u) + o;
            const uint32_t end = ((uint64_t)(r + 1) * uper < unfull) ? (r + 1) * uper : unfull;
            tile = t < end ? (int64_t)t : -1; // beyond a short last range: an empty slab
        }
        advance();
        const int64_t wcol = tile << 6;
        col = wcol + 4 * c16;
        if (ORDERED && tile < 0) return 3;
        if (wcol + 64 > D) return 2;
        return (STREAM && is_cold) ? 1 : 0;
    };
    auto rows = [&](auto how) __attribute__((always_inline)) {
        constexpr int HOW = decltype(how)::value;
#pragma unroll
        for (int i = 0; i < RPL; ++i) {
            const int row = 4 * i + q;
            const float *xr = X + (ROWS ? xro[ROWS ? i : 0] : (int64_t)row * ld);
            f32x4 v = {0.f, 0.f, 0.f, 0.f}; // rows beyond n, and empty slabs, add nothing to any sum
            if (HOW != 3 && row < n) {
                if constexpr (HOW == 0) v = *reinterpret_cast<const f32x4u *>(xr + col);
                else if constexpr (HOW == 1) v = __builtin_nontemporal_load(reinterpret_cast<const f32x4u *>(xr + col));
                else v = load4(xr, col, D, false);
            }
            x[i] = v;
        }
    };
    // run `f` with the load mode as a compile-time constant
    auto with_mode = [&](int how, auto f) __attribute__((always_inline)) {
        if (how == 0) f(std::integral_constant<int, 0>{});
        else if (how == 1) f(std::integral_constant<int, 1>{});
        else if (how == 2) f(std::integral_constant<int, 2>{});
        else f(std::integral_constant<int, 3>{});
    };
    auto load_slab = [&]() __attribute__((always_inline)) { with_mode(next_slab(), rows); };
    // steps 2 and 3: the slab in x, centred, into `buf`
    auto centre_and_stage = [&](float *buf) __attribute__((always_inline)) {
        f32x4 s = x[0];
#pragma unroll
        for (int i = 1; i < RPL; ++i) s += x[i];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            s[c] = sum_over_rows(s[c]) * inv_n;
        }
        // The LDS region is private to this wave and a wave's LDS operations execute in order, so
        // no barrier is needed between consuming a slab and overwriting it.
#pragma unroll
        for (int i = 0; i < RPL; ++i) {
            const int row = 4 * i + q;
            // rows >= n hold -mean here; they only reach entries with i or j >= n, never stored
            *reinterpret_cast<f32x4 *>(&buf[row * 64 + ((c16 ^ (row & 15)) << 2)]) = x[i] - s;
        }
    };
    // steps 4 and 5 on the slab in `buf`
    auto multiply = [&](const float *buf) __attribute__((always_inline)) {
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            f32x4 a[NB];
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const int row = 16 * b + c16; // here c16 plays the role of rr (matrix row)
                a[b] = *reinterpret_cast<const f32x4 *>(&buf[row * 64 + (((4 * st + q) ^ c16) << 2)]);
            }
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                int p = 0;
#pragma unroll
                for (int b = 0; b < NB; ++b) {
#pragma unroll
                    for (int b2 = b; b2 < NB; ++b2) {
                        acc[p] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[b][c], a[b2][c], acc[p], 0, 0, 0);
                        ++p;
                    }
                }
            }
        }
    };
    // Two workgroups per CU, i.e. two waves per SIMD, take turns at the matrix pipe.  (One wave per
    // SIMD that overlaps the steps itself - two slabs in its LDS region; slab t multiplied while
    // slab t+1 is centred and staged and the loads of slab t+2 go out, all in one basic block -
    // was slower: 632 against 566 us at n = 64, D = 11.2 M.)
    if (lo < nidx) load_slab();
    for (uint32_t idx = lo; idx < nidx; idx += stride) {
        centre_and_stage(my);
        // the next slab's loads are in flight while this one is multiplied
        if (idx + stride < nidx) load_slab();
        multiply(my);
    }

    // combine the waves through LDS, then store the upper triangle in tri(i, j) order
    __syncthreads();
    float *xch = &lds[0][0]; // [wave-1][pair][r][lane], NPAIR*256 floats per wave (<= NROW*64)
    if (wave > 0) {
#pragma unroll
        for (int p = 0; p < NPAIR; ++p)
#pragma unroll
            for (int r = 0; r < 4; ++r) xch[((wave - 1) * NPAIR * 4 + p * 4 + r) * 64 + lane] = acc[p][r];
    }
    __syncthreads();
    if (wave == 0) {
        const int P = n * (n + 1) / 2;
        float *out = partials + (int64_t)blockIdx.x * P;
        int p = 0;
#pragma unroll
        for (int b = 0; b < NB; ++b) {
#pragma unroll
            for (int b2 = b; b2 < NB; ++b2) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int i = 16 * b + 4 * q + r;
                    const int j = 16 * b2 + c16;
                    float v = acc[p][r];
#pragma unroll
                    for (int w = 1; w < kGramWaves; ++w) v += xch[((w - 1) * NPAIR * 4 + p * 4 + r) * 64 + lane];
                    if (i <= j && j < n) out[tri(i, j, n)] = v;
                }
                ++p;
            }
        }
    }
}

// Sum the per-workgroup fp32 partials in fp64, split into gridDim.y interleaved slices so that
// many threads share the work: part2[slice][p] = sum_{k = slice (mod nslices)} partials[k][p]
// (zero for a slice with no partials).
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float *__restrict__ partials,
                                                              int nparts, int P,
                                                              double *__restrict__ part2)
{
    const int p = blockIdx.x * 256 + threadIdx.x;
    const int slice = blockIdx.y, nslices = gridDim.y;
    if (p >= P) return;
    double s = 0.0;
    constexpr int U = 16; // loads in flight per thread
    for (int k = slice; k < nparts; k += U * nslices) {
        float v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) { // unconditional loads (index clamped) issue together
            const int ku = k + u * nslices;
            v[u] = partials[(int64_t)(ku < nparts ? ku : nparts - 1) * P + p];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) s += (k + u * nslices < nparts) ? (double)v[u] : 0.0;
    }
    part2[(int64_t)slice * P + p] = s;
}

} // namespace svgd
