// Pass 3: the fused all-particle update.  For every column k independently
//
//     z_jk   = g_jk - (2/h) x_jk
//     phi_ik = sum_j C_ij z_jk + rho_i x_ik,      C_ij = K_ij / n,  rho_i = (2/h) (sum_j K_ij) / n
//     x_ik  <- x_ik + eps * phi_ik
//
// which is phi_i = (1/n) sum_j [K_ij g_j + (2/h) K_ij (x_i - x_j)] with the sum over j of the
// x_j terms folded into a single n x n product (paper App. B.2, SVGD routine: per-pair kernel value,
// accumulation of the kernel-weighted gradients and of the kernel gradient, division by n, then
// the followers' parameter update; here in the score/ascent convention, x += eps * phi).
// X and G are read once and X is written once, in place: a column's outputs depend only on that
// column's inputs, and every thread/wave loads all n rows of its columns before storing any, so
// every phi_i is computed from the pre-step X.
#pragma once
#include <type_traits>

#include "bandwidth_kernels.hpp"
#include "common.hpp"

namespace svgd {

// FUSED: the step in ONE launch.  The kernel starts with pass 2 (kernel_matrix_prologue: every
// workgroup derives h, C and rho for itself from the short list of pair-sum partials that the
// previous update left behind) and, being a CARRY kernel, ends by leaving the partials of the new
// X for the next one - in the other half of the scratch, because workgroups that are still in
// their prologue read the old list.  Used when that list is short (small problems, where two more
// launches would cost as much as the work).
struct FusedArgs {
    const float *partials_in; // [nparts_in][n (n + 1) / 2], format of the Gram kernels
    int nparts_in;
    double h_fixed;
    // Not about fusion, but every update kernel takes this struct: walk the columns from the far
    // end.  Which thread or wave owns which columns does not change, only the order in which it
    // visits them.  A caller that alternates the direction from step to step starts every pass
    // on the part of X that the previous pass touched last, i.e. on what the memory-side cache
    // still holds.
    int reverse;
    // ALIGNED matrix-core kernels: the four waves of a workgroup take adjacent tiles of one range
    // instead of a range each (see tile_range).
    int adjacent;
};

// ---------------------------------------------------------------------------------------------
// n <= kValuMaxN (12): vector ALU, lanes = columns, 4 consecutive columns per thread (16-byte
// loads, 1 KiB contiguous per row per wave).  C and rho are wave-uniform: LDS broadcasts.
// ---------------------------------------------------------------------------------------------
template <int N, bool EMIT, bool CARRY, bool ROWS = false, bool FUSED = false>
__global__ __launch_bounds__(256) void update_valu_kernel(float *__restrict__ X,
                                                          const float *__restrict__ G,
                                                          float *__restrict__ PHI,
                                                          float *__restrict__ coef,
                                                          DevState *__restrict__ st,
                                                          int64_t D, int64_t ld, float eps,
                                                          float *__restrict__ gram_out,
                                                          typename RowArg<ROWS>::type rt, FusedArgs fa)
{
    static_assert(!(ROWS && (EMIT || CARRY)), "separate rows: plain in-place step only");
    static_assert(!FUSED || (CARRY && !ROWS), "the fused step lives on carried pair sums");
    static_assert(!(CARRY && EMIT), "the pair sums are carried only when X is updated");
    // CARRY: the pair sums of the UPDATED columns, in the format of gram_valu_kernel<N>
    constexpr bool kDiff = (N <= 8);
    constexpr int P = N * (N + 1) / 2;
    float pacc[CARRY ? P : 1];
    if constexpr (CARRY) {
#pragma unroll
        for (int p = 0; p < P; ++p) pacc[p] = 0.f;
    }
    // C and rho are wave-uniform.  They are staged in LDS and read back as broadcasts: a chain of
    // dependent scalar loads from global memory costs microseconds per wave, which is all there
    // is to hide behind when D is small.
    __shared__ __attribute__((aligned(16))) float C[N * N + N];
    float *rho = C + N * N;
    const int64_t ngroups = (D + 3) >> 2;
    const int64_t nthreads = (int64_t)gridDim.x * 256;
    // PREFETCH (carried pair sums of 9 to 12 particles, where the registers allow a single wave per
    // SIMD anyway): the loads of a thread's next column group are issued as soon as this group's
    // results are stored, before its pair sums are accumulated, so that arithmetic runs while the
    // loads are in flight (88.6 instead of 94.3 us per step at n = 12, D = 3,000,000).  At n <= 8
    // the longer live ranges cost a resident wave and the kernel gets slower.
    constexpr bool PREFETCH = CARRY && N > 8;
    f32x4 x[N], z[N];
    auto load_group = [&](int64_t g) __attribute__((always_inline)) {
        const int64_t c = g << 2;
        const bool fl = (c + 4 <= D);
#pragma unroll
        for (int j = 0; j < N; ++j) {
            x[j] = load4(X + (ROWS ? rt.x[ROWS ? j : 0] : (int64_t)j * ld), c, D, fl);
            z[j] = load4_stream(G + (ROWS ? rt.g[ROWS ? j : 0] : (int64_t)j * ld), c, D, fl);
        }
    };
    // this thread's groups: grp0 + k * nthreads, k < cnt, visited upwards or (reverse) downwards
    const int64_t grp0 = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t cnt = (grp0 < ngroups) ? (ngroups - 1 - grp0) / nthreads + 1 : 0;
    const int64_t gstep = fa.reverse ? -nthreads : nthreads;
    int64_t grp = fa.reverse ? grp0 + (cnt - 1) * nthreads : grp0;
    // Fused step: the first column group's loads go out in the middle of the prologue, after the
    // list of partial sums has been read, so that they are in flight during the arithmetic on h and K.
    // (only a group that lies wholly inside the row: the masked loads of a ragged last group come
    // with branches and waits of their own and are left to the loop)
    const bool early = FUSED && cnt > 0 && ((grp << 2) + 4 <= D);
    float c2h;
    if constexpr (FUSED) {
        __shared__ BwShared sh;
        auto first_loads = [&]() __attribute__((always_inline)) {
            if (early) {
                const int64_t c = grp << 2;
#pragma unroll
                for (int j = 0; j < N; ++j) {
                    x[j] = *reinterpret_cast<const f32x4u *>(X + (int64_t)j * ld + c);
                    z[j] = __builtin_nontemporal_load(reinterpret_cast<const f32x4u *>(G + (int64_t)j * ld + c));
                }
            }
        };
        const double h = kernel_matrix_prologue<256>(sh, fa.partials_in, fa.nparts_in, N, kDiff ? kModeDiff : kModeGram,
                                                     fa.h_fixed, st, coef, C, blockIdx.x == 0, first_loads);
        c2h = (N == 1) ? 0.f : (float)(2.0 / h);
    } else {
        c2h = st->two_over_h;
        for (int e = threadIdx.x; e < N * N; e += 256) C[e] = coef[kOffC + e];
        if (threadIdx.x < N) rho[threadIdx.x] = coef[kOffRho + threadIdx.x];
        __syncthreads();
    }
    if constexpr (PREFETCH) {
        if (cnt > 0 && !early) load_group(grp);
    }
    for (int64_t k = 0; k < cnt; ++k, grp += gstep) {
        const int64_t col = grp << 2;
        const bool full = (col + 4 <= D);
        if constexpr (!PREFETCH) {
            if (k > 0 || !early) load_group(grp);
        }

        f32x4 m = f32x4{0.f, 0.f, 0.f, 0.f};
        if constexpr (CARRY && !kDiff) { // centre by the pre-update column mean
#pragma unroll
            for (int j = 0; j < N; ++j) m += x[j];
            m *= (1.0f / N);
        }
#pragma unroll
        for (int j = 0; j < N; ++j) z[j] -= c2h * x[j];
        f32x4 y[CARRY ? N : 1];
#pragma unroll
        for (int i = 0; i < N; ++i) {
            f32x4 acc = rho[i] * x[i];
#pragma unroll
            for (int j = 0; j < N; ++j) acc += C[i * N + j] * z[j];
            if constexpr (EMIT) {
                store4(PHI + (int64_t)i * ld, col, D, full, acc);
            } else {
                const f32x4 xn = x[i] + eps * acc;
                store4(X + (ROWS ? rt.x[ROWS ? i : 0] : (int64_t)i * ld), col, D, full, xn);
                if constexpr (CARRY) y[i] = xn - m; // columns beyond D: x = g = 0 -> xn = 0, m = 0
            }
        }
        if constexpr (CARRY) {
            if constexpr (PREFETCH) {
                if (k + 1 < cnt) load_group(grp + gstep);
            }
#pragma unroll
            for (int i = 0; i < N; ++i) {
#pragma unroll
                for (int j = kDiff ? i + 1 : i; j < N; ++j) {
                    const f32x4 u = kDiff ? y[i] - y[j] : y[i];
                    const f32x4 v = kDiff ? u : y[j];
                    float a = pacc[tri(i, j, N)];
                    a = fmaf(u.x, v.x, a);
                    a = fmaf(u.y, v.y, a);
                    a = fmaf(u.z, v.z, a);
                    a = fmaf(u.w, v.w, a);
                    pacc[tri(i, j, N)] = a;
                }
            }
        }
    }
    if constexpr (CARRY) {
        __shared__ float red[4][P];
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const float v = wave_sum(pacc[p]);
            if (lane == 0) red[wave][p] = v;
        }
        __syncthreads();
        for (int p = threadIdx.x; p < P; p += 256)
            gram_out[(int64_t)blockIdx.x * P + p] = (red[0][p] + red[1][p]) + (red[2][p] + red[3][p]);
    }
}

// ---------------------------------------------------------------------------------------------
// kValuMaxN < n <= 64: matrix cores, v_mfma_f32_16x16x4_f32 with M = output particle i, K = input
// particle j, N = column.
//
// Register tile.  A wave owns 16*NB rows x 64 columns at a time: lane (q = lane/16, c = lane%16)
// loads, for b < NB and r < 4, row 16b + 4q + r at columns 4c..4c+3 of the tile (256 B contiguous
// per row per quarter-wave).  Step s = 4b + r of the contraction feeds k-slot q with row
// 16b + 4q + r; the 4 components of the 16-byte load are 4 independent N-tiles (tile t = columns
// {4c + t}).  The 16x16 result of output block bi puts row 16bi + 4q + r, column c in register r
// of lane (q, c) - exactly the rows this lane loaded, so x_old is already in place for the
// epilogue and nothing crosses lanes.  The A operands (C re-ordered into the per-lane layout by
// the prologue) sit in LDS, shared by the workgroup's 4 waves, and are re-read per output block.
//
// Stores.  A row starts at i*ld floats, so in general the rows are not 128-byte aligned and a
// store of "the tile's columns" would cut cache lines in two for almost every row; partial-line
// writes cost far more HBM time than they carry bytes.  Loads do not care.  So each wave
//   - owns a CONTIGUOUS range of tiles and walks it left to right,
//   - stages each finished 16-row output block in LDS (cur, 16 x 64 floats),
//   - and for row i stores the 64-column window that ends r_i columns before the tile does,
//     r_i = (address of row i at the tile's first column, in floats) mod 32: that window starts
//     on a 128-byte boundary, and its first r_i columns are the previous tile's last ones, kept
//     in LDS (carry, 64 x 32 floats per wave).
// Every store instruction then writes whole cache lines.  Only the two ends of a wave's range
// see partial lines: the first tile masks what lies left of the range, and the carry is flushed
// element-wise after the last tile.
// ALIGNED: the caller guarantees that every row starts on a 128-byte boundary (ld a multiple of
// 32 floats, base pointer aligned).  Then r_i = 0 for all rows, the windows are the tiles, and
// the results are stored straight from the registers that computed them - no staging at all
// unless the Gram operands need it.
// Columns beyond the last full tile (D mod 64) are done by one extra workgroup with a plain
// loop.  Rows >= n (n not a multiple of 16) are neither loaded nor stored; their A entries are
// zero (their contraction steps still run: skipping them behind wave-uniform branches cost more
// than it saved, see below).  One to four rows beyond a multiple of 16 do not get a block of
// their own at all (REM, below).
// ---------------------------------------------------------------------------------------------
constexpr int kUpdCur = 16 * 64;    // floats per wave
constexpr int kUpdCarry = 64 * 32;  // floats per wave

template <bool EMIT, bool CARRY, bool ROWS>
__device__ inline void update_tail_columns(float *__restrict__ X, const float *__restrict__ G,
                                           float *__restrict__ OUT, const float *Cm, const float *rhov,
                                           float c2h, int n, int64_t D, int64_t ld, int64_t col0, float eps,
                                           float *__restrict__ lds, float *__restrict__ gram_out,
                                           const typename RowArg<ROWS>::type &rt)
{
    // plain per-column evaluation for the < 64 columns after the last full tile
    float *zs = lds, *xs = lds + 64 * 64, *yn = lds + 2 * 64 * 64;
    const int col = threadIdx.x & 63, part = threadIdx.x >> 6;
    const bool ok = (col0 + col < D);
    for (int j = part; j < n; j += 4) {
        float xv = 0.f, gv = 0.f;
        if (ok) {
            xv = X[(ROWS ? rt.x[ROWS ? j : 0] : (int64_t)j * ld) + col0 + col];
            gv = G[(ROWS ? rt.g[ROWS ? j : 0] : (int64_t)j * ld) + col0 + col];
        }
        xs[j * 64 + col] = xv;
        zs[j * 64 + col] = gv - c2h * xv;
    }
    __syncthreads();
    float m = 0.f;
    if constexpr (CARRY) {
        for (int j = 0; j < n; ++j) m += xs[j * 64 + col];
        m *= 1.0f / (float)n;
    }
    for (int i = part; i < n; i += 4) {
        float acc = 0.f;
        for (int j = 0; j < n; ++j) acc = fmaf(Cm[i * n + j], zs[j * 64 + col], acc);
        const float xv = xs[i * 64 + col];
        const float phi = fmaf(rhov[i], xv, acc);
        const float out = EMIT ? phi : fmaf(eps, phi, xv);
        if (ok) OUT[(ROWS ? rt.x[ROWS ? i : 0] : (int64_t)i * ld) + col0 + col] = out;
        if constexpr (CARRY) yn[i * 64 + col] = ok ? out - m : 0.f;
    }
    if constexpr (CARRY) {
        // Gram of the updated, column-centred tail columns, in tri(i, j) order
        __syncthreads();
        const int P = n * (n + 1) / 2;
        for (int p = threadIdx.x; p < P; p += 256) {
            int i = 0, rem = p;
            while (rem >= n - i) { rem -= n - i; ++i; }
            const int j = i + rem;
            float acc = 0.f;
            for (int c = 0; c < 64; ++c) acc = fmaf(yn[i * 64 + c], yn[j * 64 + c], acc);
            gram_out[p] = acc;
        }
    }
}

// keeps the compiler from turning per-row addresses into 2 x 16 loop-carried pointer pairs
// (an integer offset is laundered, not the pointer, so the accesses stay global_load/store)
__device__ inline void opaque(int64_t &v) { asm volatile("" : "+v"(v)); }

// CARRY: additionally accumulate the Gram of the UPDATED columns, centred by the pre-update column
// mean (any per-column shift common to all particles leaves every d2 unchanged), and write one
// partial per workgroup (the last one is the tail's) to gram_out in the format of
// gram_mfma_kernel.  The next step can then skip its own pass over X.
//
// Instruction mix.  One wave per SIMD has to keep the matrix pipe, the vector ALU, LDS and the
// memory pipe busy at once, so the work of a tile is ordered as
//     M(0) | M(1)+E(0)+G(0) | M(2)+E(1)+G(1) | ... | E(NB-1)+G(NB-1)
// with M(b) = the MFMAs and epilogue of output block b, E(b) = the aligned stores of block b
// (LDS reads, address arithmetic, global stores) and G(b) = the Gram MFMAs of block b (CARRY).
// The pieces of one group are written interleaved and sit in one basic block (no branches in the
// steady-state tile), which lets the scheduler fill the MFMA shadows; a handful of wave-uniform
// branches inside the tile made it 20-30 % slower when tried.  The first tile of a range, which
// has to mask its left edge, is a separate, branchy instance of the same code.
// ROWS: the particles are n separately allocated rows; row addresses (and store alignments) come
// from a RowTable instead of i * ld (plain in-place step only, re-aligned stores).
// REM: n = 16 NB + R with 1 <= R <= 4.  A whole further block of 16 rows for those few particles
// would cost a tile the instructions of 16 more rows while it moves the bytes of R; instead the R
// remainder rows ride along in one register per array - lane (q, c) holds row 16 NB + q, columns
// 4c..4c+3, exactly one contraction step of the matrix instruction.  Their contribution to the
// other rows' phi is that one extra step per output block; their own phi, R x n x 64 products,
// is summed on the vector ALU (each lane over its own rows, then across the wave's four rows of
// lanes); they are stored as one more store group, and their pair sums (CARRY) are accumulated
// like those of a further block whose rows R..15 are zero.
template <int NB, bool EMIT, bool FULLROWS, bool CARRY, bool ALIGNED = false, bool ROWS = false, bool FUSED = false,
          bool REV = false, bool REM = false>
__global__ __launch_bounds__(256)
__attribute__((amdgpu_waves_per_eu((NB <= 2 && !FULLROWS) ? 2 : 1, (NB <= 2 && !FULLROWS) ? 2 : 1)))
void update_mfma_kernel(float *__restrict__ X, const float *__restrict__ G, float *__restrict__ PHI,
                        float *__restrict__ coef, DevState *__restrict__ st, int n,
                        int64_t D, int64_t ld, float eps, float *__restrict__ gram_out,
                        typename RowArg<ROWS>::type rt, FusedArgs fa)
{
    static_assert(!FUSED || (CARRY && !ROWS && NB <= 2), "the fused step: carried pair sums, n <= 32");
    static_assert(!(CARRY && EMIT), "the Gram is carried only when X is updated");
    static_assert(!(ROWS && (EMIT || CARRY)), "separate rows: plain in-place step");
    static_assert(!REV || (CARRY && !ALIGNED && !FUSED), "the mirrored walk exists for re-aligned stores with carried sums");
    static_assert(!REM || (FULLROWS && NB <= 3), "remainder rows come after full blocks");
    constexpr int NS = 4 * NB; // contraction steps = rows per lane
    constexpr int NBG = NB + (REM ? 1 : 0); // blocks as the pair sums see them
    constexpr int NPAIR = NBG * (NBG + 1) / 2;
    const int R = REM ? n - 16 * NB : 0; // remainder rows
    // [A operands: NB*NB*64 float4][4 waves x (cur + carry)]
    __shared__ __attribute__((aligned(16))) float lds[NB * NB * 64 * 4 + 4 * (kUpdCur + kUpdCarry)];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int q = lane >> 4, c16 = lane & 15;
    float *__restrict__ OUT = EMIT ? PHI : X;
    // C (n x n) and rho (n): the handle's tables, or - fused step - this workgroup's own copies in
    // LDS, computed by the prologue in the (still unused) staging area
    __shared__ float cl[FUSED ? 32 * 32 + 32 : 1];
    const float *Cm = coef + kOffC, *rhov = coef + kOffRho;
    float c2h;
    if constexpr (FUSED) {
        static_assert(sizeof(BwShared) <= 4 * (kUpdCur + kUpdCarry) * sizeof(float), "pass 2 fits into the staging area");
        BwShared &sh = *reinterpret_cast<BwShared *>(lds + NB * NB * 64 * 4);
        const double h = kernel_matrix_prologue<256>(sh, fa.partials_in, fa.nparts_in, n, kModeGram, fa.h_fixed, st, coef,
                                                     cl, blockIdx.x == 0);
        c2h = (n == 1) ? 0.f : (float)(2.0 / h);
        Cm = cl;
        rhov = cl + n * n;
    } else {
        c2h = st->two_over_h;
    }

    const int64_t nfull = D >> 6; // full 64-column tiles
    if (blockIdx.x == gridDim.x - 1) { // the extra workgroup: ragged tail only
        float *tail_out = nullptr;
        if constexpr (CARRY) {
            const int P = n * (n + 1) / 2;
            tail_out = gram_out + (int64_t)(gridDim.x - 1) * P; // after the workers' partials
            if ((nfull << 6) >= D)
                for (int p = threadIdx.x; p < P; p += 256) tail_out[p] = 0.f;
        }
        if ((nfull << 6) < D)
            update_tail_columns<EMIT, CARRY, ROWS>(X, G, OUT, Cm, rhov, c2h, n, D, ld, nfull << 6, eps, lds, tail_out, rt);
        return;
    }

    // With CARRY the staging block doubles as the Gram operand source (lane = row reads), so its
    // 16-byte granules are XOR-swizzled by the row; without it the block is plain row-major.
    auto cur_index = [](int rloc, int col) {
        return CARRY ? rloc * 64 + ((((col >> 2) ^ rloc) & 15) << 2) + (col & 3) : rloc * 64 + col;
    };
    f32x4 accg[CARRY ? NPAIR : 1];
    if constexpr (CARRY) {
#pragma unroll
        for (int p = 0; p < NPAIR; ++p) accg[p] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const float inv_n = 1.0f / (float)n;

    f32x4 *As4 = reinterpret_cast<f32x4 *>(lds);
    float *cur = lds + NB * NB * 64 * 4 + wave * (kUpdCur + kUpdCarry);
    float *carry = cur + kUpdCur;
    // A operands of v_mfma_f32_16x16x4_f32 for output block bi, steps 4sg..4sg+3, as one float4
    // per lane: for step s = 4sg + k lane (q = l/16, m = l%16) holds C[16bi + m][16sg + 4q + k]
    // (zero beyond n: rows and columns of the padding take no part)
    for (int e = threadIdx.x; e < NB * NB * 64; e += 256) {
        const int l = e & 63, sg = (e >> 6) % NB, bi = (e >> 6) / NB;
        const int i = 16 * bi + (l & 15), j0 = 16 * sg + 4 * (l >> 4);
        f32x4 v;
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = (i < n && j0 + k < n) ? Cm[i * n + j0 + k] : 0.f;
        As4[e] = v;
    }
    float rho[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        const int row = 16 * (s >> 2) + 4 * q + (s & 3);
        rho[s] = (FULLROWS || row < n) ? rhov[row] : 0.f;
    }
    // remainder rows.  arem: the A operand of their one contraction step for output block bi -
    // lane (q, m) holds C[16bi + m][16NB + q].  crem: for remainder row r and lane row q the
    // coefficients C[16NB + r][.] of the rows that a lane of that q holds, in the order of its
    // registers (NS rows of the full blocks, then row 16NB + q), padded to a multiple of four.
    constexpr int CREM = NS + 4;
    __shared__ float arem[REM ? NB * 64 : 1];
    __shared__ __attribute__((aligned(16))) float crem[REM ? 16 * CREM : 4];
    float rho_r = 0.f;
    if constexpr (REM) {
        for (int e = threadIdx.x; e < NB * 64; e += 256) {
            const int l = e & 63, bi = e >> 6;
            arem[e] = ((l >> 4) < R) ? Cm[(16 * bi + (l & 15)) * n + 16 * NB + (l >> 4)] : 0.f;
        }
        for (int e = threadIdx.x; e < 16 * CREM; e += 256) {
            const int s = e % CREM, rq = e / CREM, r = rq >> 2, qq = rq & 3;
            float v = 0.f;
            if (r < R) {
                if (s < NS) v = Cm[(16 * NB + r) * n + 16 * (s >> 2) + 4 * qq + (s & 3)];
                else if (s == NS && qq < R) v = Cm[(16 * NB + r) * n + 16 * NB + qq];
            }
            crem[e] = v;
        }
        if (q < R) rho_r = rhov[16 * NB + q];
    }
    __syncthreads();

    // The tiles of this wave: t0, t0 + TS, ... < t1.  Re-aligned stores hand a row's tail from one
    // tile to the next through the wave's carry, so there each wave walks a contiguous range of
    // its own (TS = 1).  ALIGNED has nothing to hand over: on request (fa.adjacent, the host's
    // choice) the workgroup owns a contiguous range and its four waves take adjacent tiles
    // (TS = 4), which makes the workgroup's accesses 1 KiB contiguous per row.
    const int64_t TS = (ALIGNED && fa.adjacent != 0) ? 4 : 1;
    int64_t t0, t1;
    tile_range(nfull, gridDim.x - 1, blockIdx.x, wave, TS == 4, t0, t1);
    const int64_t c_begin = t0 << 6;
    // visiting order: tiles t_first + k * t_step, k < ntiles.  ALIGNED kernels take the direction
    // at run time; re-aligned stores hand a row's leftover from tile to tile, so their mirror
    // image, which walks right to left, is an instance of its own (REV).
    const int64_t ntiles = (t1 - t0 + TS - 1) / TS;
    const bool rev = REV || (ALIGNED && fa.reverse != 0);
    const int64_t t_step = rev ? -TS : TS;
    const int64_t t_first = rev ? t0 + (ntiles - 1) * TS : t0;

    // lane part of every load address: row 4q, column 4c; the rest is wave-uniform
    const int64_t in_lane = ROWS ? (int64_t)(4 * c16) : (int64_t)(4 * q) * ld + 4 * c16;
    // stores: lane (rl = q, p = c16) writes row urow + q; a row's misalignment in floats is
    // (a0 + row * dm) mod 32 because every tile starts at a multiple of 32 columns
    const int64_t out_lane = ROWS ? (int64_t)(4 * c16) : (int64_t)q * ld + 4 * c16;
    const uint32_t dm = (uint32_t)ld & 31u;
    const uint32_t a0 = (uint32_t)(reinterpret_cast<uintptr_t>(OUT) >> 2) & 31u;
    // separate rows: where this lane's rows of X and G start (loads), and for every row where it
    // starts and how it is aligned (stores; in LDS, read per store group)
    int64_t xro[ROWS ? NS : 1], gro[ROWS ? NS : 1];
    __shared__ int64_t srow[ROWS ? kMaxN : 1];
    __shared__ int sri[ROWS ? kMaxN : 1];
    if constexpr (ROWS) {
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const int row = 16 * (s >> 2) + (s & 3) + 4 * q;
            xro[s] = (row < n) ? rt.x[ROWS ? row : 0] : 0;
            gro[s] = (row < n) ? rt.g[ROWS ? row : 0] : 0;
        }
        if (threadIdx.x < kMaxN) {
            srow[threadIdx.x] = ((int)threadIdx.x < n) ? rt.x[ROWS ? threadIdx.x : 0] : 0;
            sri[threadIdx.x] = ((int)threadIdx.x < n) ? rt.ri[ROWS ? threadIdx.x : 0] : 0;
        }
        __syncthreads();
    }

    // Software pipeline across tiles: the loads of tile t+1 are issued while tile t is being
    // multiplied.  Schedules chosen by measurement:
    //   XBUF (NB <= 2): the x rows of tile t+1 are loaded at the top of tile t into a second set of
    //     registers - small tiles are short, and the loads need the whole tile time to come back;
    //     otherwise into the registers of tile t as they fall free, the rows of block bi after
    //     that block's epilogue (more requests in flight only added HBM contention at n = 64);
    //   GBUF (NB <= 2, or CARRY): the same for the g rows.  Without it they are fetched as the last
    //     output block consumes them, i.e. issued last and needed first by the next tile; the
    //     longer tile of the carried sums then waits for them at every tile start (1.75 -> 1.72 ms
    //     at n = 64), while the plain update, which waits on memory anyway, is not helped.
    // The last tile of the range "prefetches" itself again (a few KB that nobody uses) so that the
    // steady-state code has no branch.
    constexpr bool XBUF = (NB <= 2);
    constexpr bool GBUF = (NB <= 2) || CARRY;
    f32x4 x[NS], z[NS], xn[XBUF ? NS : 1], gn[GBUF ? NS : 1];
    // remainder rows: this tile's x and z, and the next tile's x and g (always fetched a tile ahead)
    f32x4 xr = {0.f, 0.f, 0.f, 0.f}, zr = xr, xrn = xr, grn = xr;
    int64_t rem_x, rem_g; // row 16NB + q relative to in_lane (which has 4q ld on one array)
    if constexpr (ROWS) {
        rem_x = (REM && q < R) ? rt.x[ROWS ? 16 * NB + q : 0] : 0;
        rem_g = (REM && q < R) ? rt.g[ROWS ? 16 * NB + q : 0] : 0;
    } else {
        rem_x = rem_g = (int64_t)(16 * NB - 3 * q) * ld;
    }
    // G is read exactly once per step.  When no cache line is shared between tiles or rows
    // (ALIGNED) it is loaded with the streaming hint, which does not allocate on the way in:
    // measurably faster (a plain read-read-write stream over these buffers runs at 5.25 instead of
    // 5.08 TB/s), and it leaves the memory-side cache to X, which this kernel reads again in the
    // next step - at n = 32, D = 2,000,000 (X is 256 MB) that alone takes the update from 154 to
    // 119 us.  X itself is therefore loaded plainly.  With unaligned rows the line that a row
    // segment shares with the next tile has to stay cached, so nothing streams.
    auto load16x = [](const float *p) __attribute__((always_inline)) -> f32x4 {
        return *reinterpret_cast<const f32x4u *>(p);
    };
    auto load16g = [](const float *p) __attribute__((always_inline)) -> f32x4 {
        if constexpr (ALIGNED) return __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p));
        else return *reinterpret_cast<const f32x4u *>(p);
    };
    auto load_x = [&](const float *xt, int s) __attribute__((always_inline)) {
        const int urow = 16 * (s >> 2) + (s & 3); // uniform part of the row index
        if (FULLROWS || urow + 4 * q < n) x[s] = load16x(xt + (ROWS ? xro[ROWS ? s : 0] : (int64_t)urow * ld));
    };
    auto load_g = [&](const float *gt, int s) __attribute__((always_inline)) {
        const int urow = 16 * (s >> 2) + (s & 3);
        if (FULLROWS || urow + 4 * q < n) z[s] = load16g(gt + (ROWS ? gro[ROWS ? s : 0] : (int64_t)urow * ld));
    };
    auto load_next_rem = [&](const float *xt, const float *gt) __attribute__((always_inline)) {
        if constexpr (REM) {
            if (q < R) {
                xrn = load16x(xt + rem_x);
                grn = load16g(gt + rem_g);
            }
        }
    };
    auto load_next = [&](const float *xt, const float *gt) __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const int urow = 16 * (s >> 2) + (s & 3);
            if (FULLROWS || urow + 4 * q < n) {
                if constexpr (XBUF) xn[s] = load16x(xt + (ROWS ? xro[ROWS ? s : 0] : (int64_t)urow * ld));
                if constexpr (GBUF) gn[s] = load16g(gt + (ROWS ? gro[ROWS ? s : 0] : (int64_t)urow * ld));
            }
        }
        load_next_rem(xt, gt);
    };
    if (t0 < t1) {
        int64_t in_off = in_lane + (t_first << 6);
        opaque(in_off);
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            x[s] = f32x4{0.f, 0.f, 0.f, 0.f};
            z[s] = f32x4{0.f, 0.f, 0.f, 0.f};
            if constexpr (XBUF) xn[s] = f32x4{0.f, 0.f, 0.f, 0.f};
            else load_x(X + in_off, s);
            if constexpr (GBUF) gn[s] = f32x4{0.f, 0.f, 0.f, 0.f};
            else load_g(G + in_off, s);
        }
        load_next(X + in_off, G + in_off);
    }

    auto process_tile = [&](auto first_tag, int64_t tile, bool last) __attribute__((always_inline)) {
        constexpr bool FIRST = decltype(first_tag)::value;
        const int64_t base = tile << 6;
        const int64_t next = last ? tile : tile + t_step;
        int64_t in_off = in_lane + (next << 6);
        int64_t out_off = out_lane + base;
        const int qv = q; // (the per-row store offsets are tile-invariant and may be hoisted)
        opaque(in_off);
        const float *xt = X + in_off, *gt = G + in_off;
        float *ot = OUT + out_off;

        if constexpr (XBUF || GBUF) { // this tile's data becomes current, the next tile's loads go out
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                if constexpr (XBUF) x[s] = xn[s];
                if constexpr (GBUF) z[s] = gn[s];
            }
            if constexpr (REM) {
                xr = xrn;
                zr = grn;
            }
            load_next(xt, gt);
        } else if constexpr (REM) {
            xr = xrn;
            zr = grn;
            load_next_rem(xt, gt);
        }

        f32x4 mg[CARRY ? 4 : 1];      // pre-update column means in the Gram operand layout
        f32x4 ag[CARRY ? NBG : 1][4]; // Gram operands of the blocks finished so far
        if constexpr (CARRY) {
            f32x4 m = x[0];
#pragma unroll
            for (int s = 1; s < NS; ++s) m += x[s];
            if constexpr (REM) m += xr; // zero in the lanes without a remainder row
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                m[e] = sum_over_rows(m[e]) * inv_n;
            }
            // through the (currently idle) staging block: lane (q, c) knows columns 4c..4c+3,
            // the Gram layout wants columns 4(4st + q)..+3
            if (q == 0) *reinterpret_cast<f32x4 *>(&cur[4 * c16]) = m;
#pragma unroll
            for (int st4 = 0; st4 < 4; ++st4) mg[st4] = *reinterpret_cast<const f32x4 *>(&cur[4 * (4 * st4 + q)]);
        }
#pragma unroll
        for (int s = 0; s < NS; ++s) z[s] -= c2h * x[s];
        // phi of the remainder rows: lane (q, c) ends up with that of row 16NB + q
        f32x4 phir = {0.f, 0.f, 0.f, 0.f};
        if constexpr (REM) {
            zr -= c2h * xr;
            for (int r = 0; r < R; ++r) { // wave-uniform trip count
                const float *cr = crem + (4 * r + q) * CREM;
                f32x4 p = cr[NS] * zr;
#pragma unroll
                for (int sg = 0; sg < NB; ++sg) {
                    const f32x4 c4 = *reinterpret_cast<const f32x4 *>(cr + 4 * sg);
#pragma unroll
                    for (int k = 0; k < 4; ++k) p += c4[k] * z[4 * sg + k];
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) p[e] = sum_over_rows(p[e]);
                if (q == r) phir = p;
            }
        }

        // E(b), one of its four store groups: 4 rows x 256 B, lane (rl = q, p = c16)
        auto emit_group = [&](int b, int k) __attribute__((always_inline)) {
            const int urow = 16 * b + 4 * k;     // uniform part of the row index
            const int rloc = 4 * k + qv;         // row within the block
            const int row = urow + qv;
            const int ri = ROWS ? sri[ROWS ? row : 0] : (int)((a0 + (uint32_t)row * dm) & 31u);
            // the row's 64-float window starts on a line boundary: ri floats before the tile, or
            // (REV) 32 - ri floats into it, where it takes in the head of the tile to the right
            const int sh = REV ? ((32 - ri) & 31) : -ri;
            const int o0 = 4 * c16 + sh;         // window offset relative to the tile start
            f32x4 v;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int o = o0 + e; // one address, so nothing is read outside the arrays
                if constexpr (REV) v[e] = cur[(o >= 64) ? (kUpdCur + row * 32 + o - 64) : cur_index(rloc, o)];
                else v[e] = cur[(o < 0) ? (kUpdCur + row * 32 + 32 + o) : cur_index(rloc, o)];
            }
            if ((FULLROWS && !(REM && b == NB)) || row < n) {
                float *dst = ot + (ROWS ? srow[ROWS ? row : 0] : (int64_t)urow * ld) + sh;
                if constexpr (!FIRST) {
                    __builtin_nontemporal_store(v, reinterpret_cast<f32x4 *>(dst));
                } else { // the end of the range the walk starts from: nothing beyond it is ours
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (REV ? (o0 + e < 64) : (o0 + e >= 0)) dst[e] = v[e];
                }
            }
        };
        // after E(b): the block's last (REV: first) 32 columns become the carry of its 16 rows
        auto carry_copy = [&](int b) __attribute__((always_inline)) {
            const int rloc = lane >> 2, cc = (REV ? 0 : 32) + 8 * (lane & 3);
            const f32x4 v0 = *reinterpret_cast<const f32x4 *>(&cur[cur_index(rloc, cc)]);
            const f32x4 v1 = *reinterpret_cast<const f32x4 *>(&cur[cur_index(rloc, cc + 4)]);
            float *dstc = &carry[(16 * b + rloc) * 32 + (cc & 31)];
            *reinterpret_cast<f32x4 *>(dstc) = v0;
            *reinterpret_cast<f32x4 *>(dstc + 4) = v1;
        };
        // G(b), the part that pairs block b with block b0 <= b
        auto gram_pair = [&](int b0, int b) __attribute__((always_inline)) {
            const int pidx = b0 * NBG - (b0 * (b0 - 1)) / 2 + (b - b0);
#pragma unroll
            for (int st4 = 0; st4 < 4; ++st4)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    accg[pidx] = __builtin_amdgcn_mfma_f32_16x16x4f32(ag[b0][st4][e], ag[b][st4][e], accg[pidx], 0, 0, 0);
        };

#pragma unroll
        for (int bi = 0; bi < NB; ++bi) {
            // M(bi), interleaved with E(bi-1) and G(bi-1)
            f32x4 acc[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int sg = 0; sg < NB; ++sg) {
                const f32x4 a4 = As4[(bi * NB + sg) * 64 + lane];
#pragma unroll
                for (int k = 0; k < 4; ++k)
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[k], z[4 * sg + k][t], acc[t], 0, 0, 0);
                if (REM && sg == NB - 1) { // the remainder rows' contraction step
                    const float ar = arem[bi * 64 + lane];
#pragma unroll
                    for (int t = 0; t < 4; ++t) acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(ar, zr[t], acc[t], 0, 0, 0);
                }
                if (!GBUF && bi == NB - 1) { // z rows 4sg..4sg+3 are dead: fetch the next tile's g
#pragma unroll
                    for (int k = 0; k < 4; ++k) load_g(gt, 4 * sg + k);
                }
                if (bi > 0) {
                    // the four store groups of the previous block are spread over the NB step groups
#pragma unroll
                    for (int k = 0; k < 4; ++k)
                        if (!ALIGNED && k * NB / 4 == sg) emit_group(bi - 1, k);
                    if constexpr (CARRY) {
                        if (sg < bi) gram_pair(sg, bi - 1); // pairs (0..bi-1, bi-1): one per step group
                    }
                }
            }
            if (!ALIGNED && bi > 0) carry_copy(bi - 1);
            // epilogue for rows 16bi + 4q + r, then stage the block in LDS
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int s = 4 * bi + r;
                f32x4 o;
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const float phi = fmaf(rho[s], x[s][t], acc[t][r]);
                    o[t] = EMIT ? phi : fmaf(eps, phi, x[s][t]);
                }
                if constexpr (ALIGNED) { // the lane's 16 bytes lie where it loaded x from: whole lines per quarter-wave
                    if (FULLROWS || 16 * bi + 4 * q + r < n)
                        __builtin_nontemporal_store(o, reinterpret_cast<f32x4 *>(OUT + in_lane + base + (ROWS ? xro[ROWS ? s : 0] : (int64_t)(16 * bi + r) * ld)));
                }
                if constexpr (!ALIGNED || CARRY) // staged for the re-aligned stores and/or as Gram operands
                    *reinterpret_cast<f32x4 *>(&cur[cur_index(4 * q + r, 4 * c16)]) = o;
            }
            if constexpr (!XBUF) { // x rows of this block are dead: fetch the next tile's
#pragma unroll
                for (int r = 0; r < 4; ++r) load_x(xt, 4 * bi + r);
            }
            if constexpr (CARRY) {
                // lane (q, rr = c16) takes row rr of this block, columns 4(4st + q)..+3, centred
#pragma unroll
                for (int st4 = 0; st4 < 4; ++st4)
                    ag[bi][st4] = *reinterpret_cast<const f32x4 *>(&cur[cur_index(c16, 4 * (4 * st4 + q))]) - mg[st4];
            }
        }
        // E(NB-1) interleaved with G(NB-1)
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if constexpr (!ALIGNED) emit_group(NB - 1, k);
            if constexpr (CARRY) {
#pragma unroll
                for (int b0 = 0; b0 < NB; ++b0)
                    if (b0 * 4 / NB == k) gram_pair(b0, NB - 1);
            }
        }
        if constexpr (!ALIGNED) carry_copy(NB - 1);
        if constexpr (REM) {
            // the remainder rows: epilogue, staging as rows 0..3 of a further block, one store group
            f32x4 o;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float phi = fmaf(rho_r, xr[t], phir[t]);
                o[t] = EMIT ? phi : fmaf(eps, phi, xr[t]);
            }
            if constexpr (ALIGNED) {
                if (q < R) __builtin_nontemporal_store(o, reinterpret_cast<f32x4 *>(OUT + in_lane + base + rem_x));
            }
            if constexpr (!ALIGNED || CARRY) *reinterpret_cast<f32x4 *>(&cur[cur_index(q, 4 * c16)]) = o;
            if constexpr (CARRY) {
#pragma unroll
                for (int st4 = 0; st4 < 4; ++st4) {
                    const f32x4 v = *reinterpret_cast<const f32x4 *>(&cur[cur_index(c16 & 3, 4 * (4 * st4 + q))]) - mg[st4];
                    ag[NB][st4] = (c16 < R) ? v : f32x4{0.f, 0.f, 0.f, 0.f};
                }
            }
            if constexpr (!ALIGNED) emit_group(NB, 0);
            if constexpr (CARRY) {
#pragma unroll
                for (int b0 = 0; b0 <= NB; ++b0) gram_pair(b0, NB);
            }
            if constexpr (!ALIGNED) carry_copy(NB);
        }
    };

    if constexpr (ALIGNED) { // no left edge to mask
        int64_t tile = t_first;
        for (int64_t k = 0; k < ntiles; ++k, tile += t_step) process_tile(std::false_type{}, tile, k + 1 == ntiles);
    } else if (t0 < t1) {
        process_tile(std::true_type{}, t_first, ntiles == 1);
        int64_t tile = t_first + t_step;
        for (int64_t k = 1; k < ntiles; ++k, tile += t_step) process_tile(std::false_type{}, tile, k + 1 == ntiles);
    }

    // flush: the last r_i columns of the range (REV: its first 32 - r_i) are still in the carry
    if (!ALIGNED && t1 > t0) {
        const int64_t c_end = t1 << 6;
        for (int idx = lane; idx < 16 * NBG * 32; idx += 64) {
            const int row = idx >> 5, cc = idx & 31;
            const int ri = ROWS ? sri[ROWS ? row : 0] : (int)((a0 + (uint32_t)row * dm) & 31u);
            if constexpr (REV) {
                if (row < n && cc < ((32 - ri) & 31)) OUT[(int64_t)row * ld + c_begin + cc] = carry[row * 32 + cc];
            } else {
                if (row < n && cc >= 32 - ri && c_end - 32 + cc >= c_begin)
                    OUT[(ROWS ? srow[ROWS ? row : 0] : (int64_t)row * ld) + c_end - 32 + cc] = carry[row * 32 + cc];
            }
        }
    }

    if constexpr (CARRY) {
        // One partial per workgroup, upper triangle in tri(i, j) order (zeros if all four ranges
        // were empty): the waves' sums meet in their staging areas, which are free by now, and
        // wave p mod 4 adds up and writes block pair p.
        static_assert(NPAIR * 4 * 64 <= kUpdCur + kUpdCarry, "the staging area holds a wave's Gram sums");
#pragma unroll
        for (int p = 0; p < NPAIR; ++p) {
#pragma unroll
            for (int r = 0; r < 4; ++r) cur[(p * 4 + r) * 64 + lane] = accg[p][r];
        }
        __syncthreads();
        const float *all = lds + NB * NB * 64 * 4;
        const int P = n * (n + 1) / 2;
        float *out = gram_out + (int64_t)blockIdx.x * P;
        int p = 0;
#pragma unroll
        for (int b = 0; b < NBG; ++b) {
#pragma unroll
            for (int b2 = b; b2 < NBG; ++b2) {
                if ((p & 3) == wave) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int i = 16 * b + 4 * q + r;
                        const int j = 16 * b2 + c16;
                        const int e = (p * 4 + r) * 64 + lane;
                        const float v = (all[e] + all[(kUpdCur + kUpdCarry) + e]) +
                                        (all[2 * (kUpdCur + kUpdCarry) + e] + all[3 * (kUpdCur + kUpdCarry) + e]);
                        if (i <= j && j < n) out[tri(i, j, n)] = v;
                    }
                }
                ++p;
            }
        }
    }
}

} // namespace svgd
