// Shared device-side helpers and the layout of the handle's device state.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace svgd {

constexpr int kMaxN = 64;                              // particles
constexpr int kMaxPairsFull = kMaxN * (kMaxN + 1) / 2; // upper triangle with diagonal
constexpr int kWave = 64;
// n <= kValuMaxN runs on the vector ALU (one accumulator per pair in registers); larger n on the
// matrix cores, padded to a multiple of 16 rows.  Above 12 the register budget of the vector
// kernels (pair sums carried across steps included) no longer fits without spilling.
constexpr int kValuMaxN = 12;

typedef float f32x4 __attribute__((ext_vector_type(4)));
// rows of X start at i*D floats, so a 4-column group is only 4-byte aligned in general
typedef float f32x4u __attribute__((ext_vector_type(4), aligned(4)));

// Partial-sum formats written by the Gram kernels, both indexed by tri(i, j), i <= j.
enum GramMode : int {
    kModeDiff = 0, // entry (i<j) holds sum_k (x_ik - x_jk)^2; diagonal entries are 0
    kModeGram = 1  // entry (i<=j) holds sum_k y_ik y_jk of the column-centred y = x - mean_i x
};

__host__ __device__ inline int tri(int i, int j, int n) { return i * n - (i * (i - 1)) / 2 + (j - i); }

// Everything the update kernels need from the bandwidth kernel, in device memory.
struct DevState {
    double h;
    double med;
    float two_over_h;
    int n;
};

// Particles given as n separate rows (svgd_step_rows): where row i of X and of G starts, in floats
// relative to row 0 of the same array, and the misalignment of X's row i against a 128-byte line.
// Kernels compiled with ROWS = true take row addresses from this table instead of i * ld.
struct RowTable {
    int64_t x[kMaxN];
    int64_t g[kMaxN];
    int32_t ri[kMaxN]; // (address of X row i / 4) mod 32
    int32_t aligned;   // host side: every row of X and of G starts on a 128-byte boundary
};
// The table travels as a kernel argument (by value: nothing to allocate, copy or keep alive);
// kernels compiled with ROWS = false take this stand-in instead and never read it.
struct NoRows {
    int64_t x[1];
    int64_t g[1];
    int32_t ri[1];
    int32_t aligned;
};
template <bool ROWS> struct RowArg { typedef NoRows type; };
template <> struct RowArg<true> { typedef RowTable type; };

// Offsets (in floats) into the handle's coefficient block.
//   C   [n*n]   C_ij = K_ij / n
//   RHO [n]     rho_i = (2/h) * (sum_j K_ij) / n
//   K   [n*n]   K_ij (kept for svgd_get_last)
constexpr int kOffC = 0;
constexpr int kOffRho = kOffC + kMaxN * kMaxN;
constexpr int kOffK = kOffRho + kMaxN;
constexpr int kCoefFloats = kOffK + kMaxN * kMaxN;

__device__ inline f32x4 load4(const float *__restrict__ row, int64_t col, int64_t D, bool full)
{
    if (full) return *reinterpret_cast<const f32x4u *>(row + col);
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if (col + 0 < D) v.x = row[col + 0];
    if (col + 1 < D) v.y = row[col + 1];
    if (col + 2 < D) v.z = row[col + 2];
    if (col + 3 < D) v.w = row[col + 3];
    return v;
}

// streaming variant for data that is read exactly once (G)
__device__ inline f32x4 load4_stream(const float *__restrict__ row, int64_t col, int64_t D, bool full)
{
    if (full) return __builtin_nontemporal_load(reinterpret_cast<const f32x4u *>(row + col));
    return load4(row, col, D, false);
}

// Sum of v over the four lanes l, l ^ 16, l ^ 32, l ^ 48 (the four 16-lane rows of a wave), in every
// lane, as (v[l] + v[l ^ 16]) + (the same of l ^ 32): the gfx950 row-swap instructions exchange
// whole rows between two registers in the vector ALU, where a shuffle would go through LDS and
// make the wave wait for it twice.
__device__ inline float sum_over_rows(float v)
{
    const unsigned u = __float_as_uint(v);
    const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false); // rows 1 <-> 0 and 3 <-> 2 of the two copies
    const float s = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    const unsigned w = __float_as_uint(s);
    const auto b = __builtin_amdgcn_permlane32_swap(w, w, false, false); // rows 2, 3 <-> 0, 1
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// How the matrix-core passes share the nfull = D / 64 full 64-column tiles among nwg worker
// workgroups of four waves: either every wave owns a contiguous range [t0, t1) (stride 1), or the
// workgroup owns one and its waves take every fourth tile of it, t0, t0 + 4, ... < t1 (adjacent).
// The Gram pass and the update use the same split, so that one can start on the tiles the other
// touched last.
__device__ inline void tile_range(int64_t nfull, int64_t nwg, int64_t wg, int wave, bool adjacent, int64_t &t0,
                                  int64_t &t1)
{
    if (adjacent) {
        const int64_t per = (nfull + nwg - 1) / nwg;
        const int64_t b0 = (wg * per < nfull) ? wg * per : nfull;
        t1 = (b0 + per < nfull) ? b0 + per : nfull;
        t0 = (b0 + wave < t1) ? b0 + wave : t1;
    } else {
        const int64_t nwaves = nwg * 4;
        const int64_t per = (nfull + nwaves - 1) / nwaves;
        const int64_t w = wg * 4 + wave;
        t0 = (w * per < nfull) ? w * per : nfull;
        t1 = (t0 + per < nfull) ? t0 + per : nfull;
    }
}

// rows that all start on a 128-byte boundary
__host__ inline bool rows_aligned(const void *base, int64_t ld)
{
    return (ld & 31) == 0 && (reinterpret_cast<uintptr_t>(base) & 127) == 0;
}

__device__ inline void store4(float *__restrict__ row, int64_t col, int64_t D, bool full, f32x4 v)
{
    if (full) {
        __builtin_nontemporal_store(v, reinterpret_cast<f32x4u *>(row + col));
        return;
    }
    if (col + 0 < D) row[col + 0] = v.x;
    if (col + 1 < D) row[col + 1] = v.y;
    if (col + 2 < D) row[col + 2] = v.z;
    if (col + 3 < D) row[col + 3] = v.w;
}

// Sum over the 64 lanes of a wave, returned in every lane.  Four DPP adds give every lane the sum
// of its row of 16 (quad swap, quad-pair swap, half-row mirror, row mirror); the four row sums are
// then read from lanes 0, 16, 32, 48.  No LDS traffic, unlike shuffle-based reductions.
__device__ inline float wave_sum(float v)
{
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, false));  // quad_perm [1,0,3,2]
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, false));  // quad_perm [2,3,0,1]
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xF, 0xF, false)); // row_half_mirror
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xF, 0xF, false)); // row_mirror
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
    const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
    const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
    return (r0 + r1) + (r2 + r3);
}

} // namespace svgd
