// Host side of the C ABI declared in include/svgd.h: handle, argument validation, launches.
#include "../../include/svgd.h"

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <mutex>
#include <new>
#include <unordered_set>
#include <vector>

#include "bandwidth_kernels.hpp"
#include "common.hpp"
#include "diag_kernels.hpp"
#include "gram_kernels.hpp"
#include "swag_kernels.hpp"
#include "tiny_kernels.hpp"
#include "update_kernels.hpp"

using namespace svgd;

namespace {

constexpr uint32_t kMagic = 0x53564744u; // "SVGD"
constexpr int kMaxParts = 2048;          // upper bound on Gram workgroups (= partial vectors)
constexpr int64_t kMemorySideCacheBytes = (int64_t)256 << 20; // this part's memory-side cache (between L2 and HBM)

} // namespace

struct svgd_ctx {
    uint32_t magic;
    int device;
    int max_n;
    int64_t max_D;
    int num_cu;
    uint32_t flags;
    double h_fixed;
    // Gram partials of the current X left behind by the last svgd_step (SVGD_FLAG_CARRY_GRAM)
    bool carry_valid;
    const float *carry_X;
    int carry_n;
    int64_t carry_D;
    int64_t carry_ld;
    int carry_nparts;
    int64_t carry_off;        // where in `partials` the carried list starts (floats): 0 or the upper half
    hipStream_t carry_stream; // the stream the carried sums were produced on
    int64_t partials_cap;     // floats available in `partials`
    unsigned sweeps;          // in-place updates with carried sums so far: every other one walks X backwards
    int last_n; // 0 = nothing computed yet
    int last_hip_error;
    float *partials;  // [kMaxParts][P]
    double *part2;    // [kSlices][P]
    DevState *state;
    float *coef;      // kCoefFloats
    // optional per-kernel timing (svgd_profile_begin/end): event pairs recorded around launches
    bool profiling;
    unsigned profile_kinds; // bit k set: kernels of kind k are timed
    std::vector<hipEvent_t> ev_pool; // 2 events per record
    std::vector<int> ev_kind;        // SVGD_KERNEL_* of each record
};

namespace {

struct DeviceGuard {
    int prev = -1;
    bool switched = false;
    explicit DeviceGuard(int dev)
    {
        if (hipGetDevice(&prev) == hipSuccess && prev != dev) switched = (hipSetDevice(dev) == hipSuccess);
    }
    ~DeviceGuard()
    {
        if (switched) (void)hipSetDevice(prev);
    }
};

int fail(svgd_ctx *c, hipError_t e)
{
    if (c) c->last_hip_error = (int)e;
    return SVGD_ERR_DEVICE;
}

// Live handles are kept in a registry so that a stale pointer (use after destroy) is rejected
// without being dereferenced.
std::mutex g_live_mutex;
std::unordered_set<svgd_ctx *> &live_handles()
{
    static std::unordered_set<svgd_ctx *> s;
    return s;
}

int check_handle(svgd_ctx *c)
{
    if (!c) return SVGD_ERR_BAD_HANDLE;
    std::lock_guard<std::mutex> lock(g_live_mutex);
    if (!live_handles().count(c) || c->magic != kMagic) return SVGD_ERR_BAD_HANDLE;
    return SVGD_OK;
}

constexpr size_t kMaxProfileRecords = 2048;

// Records a start event on construction and a stop event on destruction when profiling is on.
// The events come from a pool that svgd_profile_begin* has created: nothing is allocated between
// the launches that are being timed.
struct KernelTimer {
    svgd_ctx *c;
    hipStream_t s;
    size_t slot = (size_t)-1;
    KernelTimer(svgd_ctx *ctx, int kind, hipStream_t stream) : c(ctx), s(stream)
    {
        if (!c->profiling || !((c->profile_kinds >> kind) & 1u)) return;
        const size_t idx = c->ev_kind.size();
        if (idx >= kMaxProfileRecords || c->ev_pool.size() < 2 * (idx + 1)) return;
        if (hipEventRecord(c->ev_pool[2 * idx], s) != hipSuccess) { (void)hipGetLastError(); return; }
        c->ev_kind.push_back(kind); // capacity reserved by svgd_profile_begin*
        slot = idx;
    }
    ~KernelTimer()
    {
        if (slot != (size_t)-1) (void)hipEventRecord(c->ev_pool[2 * slot + 1], s);
    }
};

int check_shape(svgd_ctx *c, int n, int64_t D, int64_t ld)
{
    if (n < 1 || D < 1 || ld < D) return SVGD_ERR_INVALID_ARG;
    if (n > c->max_n || D > c->max_D) return SVGD_ERR_TOO_LARGE;
    return SVGD_OK;
}

// n rows of D floats, ld floats apart: the byte ranges from the first to the last element
bool overlaps(const float *a, const float *b, int n, int64_t D, int64_t ld)
{
    const uintptr_t bytes = ((uintptr_t)(n - 1) * (uintptr_t)ld + (uintptr_t)D) * sizeof(float);
    const uintptr_t pa = (uintptr_t)a, pb = (uintptr_t)b;
    return pa < pb + bytes && pb < pa + bytes;
}

// rt != nullptr: the particles are separate rows (svgd_step_rows); the table goes along by value
template <int N>
void launch_gram_valu(const float *X, int64_t D, int64_t ld, float *partials, int grid, hipStream_t s,
                      const RowTable *rt, bool stream_x)
{
    if (rt)
        gram_valu_kernel<N, true><<<grid, 256, 0, s>>>(X, D, ld, partials, *rt);
    else if (stream_x)
        gram_valu_kernel<N, false, true><<<grid, 256, 0, s>>>(X, D, ld, partials, NoRows{});
    else
        gram_valu_kernel<N, false><<<grid, 256, 0, s>>>(X, D, ld, partials, NoRows{});
}

template <int N, bool EMIT, bool CARRY>
void launch_update_valu(float *X, const float *G, float *PHI, float *coef, DevState *st,
                        int64_t D, int64_t ld, float eps, float *gram_out, int grid, hipStream_t s,
                        const RowTable *rt, const FusedArgs &ua)
{
    if constexpr (!EMIT && !CARRY) {
        if (rt) {
            update_valu_kernel<N, false, false, true><<<grid, 256, 0, s>>>(X, G, PHI, coef, st, D, ld, eps, gram_out, *rt, ua);
            return;
        }
    }
    update_valu_kernel<N, EMIT, CARRY, false><<<grid, 256, 0, s>>>(X, G, PHI, coef, st, D, ld, eps, gram_out, NoRows{}, ua);
}

template <int N>
void launch_update_valu_fused(float *X, const float *G, float *coef, DevState *st, int64_t D, int64_t ld, float eps,
                              float *gram_out, int grid, hipStream_t s, const FusedArgs &fa)
{
    update_valu_kernel<N, false, true, false, true><<<grid, 256, 0, s>>>(X, G, nullptr, coef, st, D, ld, eps, gram_out, NoRows{}, fa);
}

#define SVGD_SWITCH_N(n, CALL)                                                                     \
    switch (n) {                                                                                   \
    case 1: CALL(1); break;                                                                        \
    case 2: CALL(2); break;                                                                        \
    case 3: CALL(3); break;                                                                        \
    case 4: CALL(4); break;                                                                        \
    case 5: CALL(5); break;                                                                        \
    case 6: CALL(6); break;                                                                        \
    case 7: CALL(7); break;                                                                        \
    case 8: CALL(8); break;                                                                        \
    case 9: CALL(9); break;                                                                        \
    case 10: CALL(10); break;                                                                      \
    case 11: CALL(11); break;                                                                      \
    default: CALL(12); break;                                                                      \
    }

int clampi(int64_t v, int lo, int hi) { return (int)(v < lo ? lo : (v > hi ? hi : v)); }
int mini(int a, int b) { return a < b ? a : b; }

// How many partial vectors of n(n+1)/2 floats the handle's scratch holds: the upper bound on every
// grid whose workgroups write one partial each.
int max_parts(const svgd_ctx *c, int n)
{
    const int64_t P = (int64_t)n * (n + 1) / 2;
    const int64_t m = c->partials_cap / P;
    return (int)(m < kMaxParts ? m : kMaxParts);
}

// An X that the memory-side cache cannot hold (with a margin: n = 32, D = 2,000,000 just fits and
// behaves like a cached problem).
bool beyond_cache(int n, int64_t ld)
{
    return (int64_t)n * ld * (int64_t)sizeof(float) > kMemorySideCacheBytes + kMemorySideCacheBytes / 4;
}

// Particle counts one to four above a multiple of 16: the matrix-core update treats the extra
// particles as remainder rows (template argument REM of update_mfma_kernel).
bool has_remainder_rows(int n) { return n > 16 && (n & 15) >= 1 && (n & 15) <= 4; }

// Whether the matrix-core update on aligned rows lets the waves of a workgroup share a range.
bool adjacent_tiles(int n, int64_t ld) { return n > 48 || beyond_cache(n, ld); }

// Worker workgroups of the matrix-core update (each walks ranges of 64-column tiles; one more
// workgroup does D mod 64): one per CU - the kernel overlaps its own loads with its multiplies, and
// fewer concurrent row streams keep more HBM pages open.  Exception: 21 to 24 particles, whose
// tiles cost the instructions of 32 rows but move little more than half the bytes, so that the
// fixed costs of a tile show (17 to 20 are 16 rows plus remainder rows, see has_remainder_rows).
// The kernel instances for n not a multiple of 16, n < 32, are built for two waves per SIMD, and
// for those particle counts and an X beyond the memory-side cache two workgroups per CU overlap
// one's arithmetic with the other's loads (with carried sums at D = 5,000,000: n = 24
// 258 -> 241 us; from n = 25 on the gain is below the cost of the longer list of partial sums,
// with 16 or 32 particles the second workgroup costs 2-5 %, and for an X that cache serves it
// costs 9 %).
// The Gram pass splits the tiles the same way.
int update_workers(const svgd_ctx *c, int n, int64_t D, int64_t ld, bool carry)
{
    const int64_t nfull = D / 64;
    const int per_cu = (n >= 17 && n <= 24 && !has_remainder_rows(n) && beyond_cache(n, ld)) ? 2 : 1;
    const int max_workers = mini(c->num_cu * per_cu, (carry ? max_parts(c, n) : kMaxParts) - 1);
    return clampi((nfull + 3) / 4, 1, max_workers);
}

// Passes 1 and 2: Gram partials -> fp64 reduction -> h, K, coefficient tables (all on `s`).
// With use_carry the partials the previous update left in c->partials stand in for pass 1.
// G_next: where the in-place update that follows this call will read its scores (null: none, or
// an update that writes phi elsewhere); carry_next: that update will carry pair sums.  Both only
// steer the order in which pass 1 visits X.
int run_kernel_matrix(svgd_ctx *c, const float *X, int n, int64_t D, int64_t ld, hipStream_t s, bool use_carry,
                      const RowTable *rt = nullptr, const float *G_next = nullptr, bool carry_next = false)
{
    const int P = n * (n + 1) / 2;
    const int cap_parts = max_parts(c, n);
    int nparts, mode;
    const float *partials = c->partials; // where the list of partials for pass 2 starts
    // streaming loads in pass 1: X well beyond what the memory-side cache could keep for the update
    const bool big_x = (int64_t)n * ld * (int64_t)sizeof(float) > 2 * kMemorySideCacheBytes;
    const bool x_aligned = rt ? rt->aligned != 0 : rows_aligned(X, ld);
    if (use_carry) {
        nparts = c->carry_nparts;
        partials += c->carry_off;
        mode = (n <= 8) ? kModeDiff : kModeGram; // the update kernels mirror the Gram kernels' formats
    } else if (n <= kValuMaxN) {
        const int64_t ngroups = (D + 3) / 4;
        nparts = clampi((ngroups + 255) / 256, 1, mini(c->num_cu * 3, cap_parts)); // all resident at once; each ends with a reduction
        mode = (n <= 8) ? kModeDiff : kModeGram;
        const bool stream_x = big_x;
        KernelTimer t(c, SVGD_KERNEL_GRAM, s);
#define CALL(N) launch_gram_valu<N>(X, D, ld, c->partials, nparts, s, rt, stream_x)
        SVGD_SWITCH_N(n, CALL)
#undef CALL
    } else {
        KernelTimer t(c, SVGD_KERNEL_GRAM, s);
        mode = kModeGram;
        const int NB = (n + 15) / 16;
        const int64_t nfull = D / 64;
        nparts = clampi((D + 255) / 256, 1, mini(c->num_cu * 2, cap_parts));
        // the ranges of the update that follows (tile_range) and how many of each range's first
        // tiles three quarters of the memory-side cache can hold
        const bool aligned_next = G_next && x_aligned && (rt || rows_aligned(G_next, ld));
        const bool shared_ranges = aligned_next && adjacent_tiles(n, ld);
        int64_t nranges = (int64_t)update_workers(c, n, D, ld, carry_next) * (shared_ranges ? 1 : 4);
        int64_t per = (nfull + nranges - 1) / nranges > 0 ? (nfull + nranges - 1) / nranges : 1;
        int64_t hot = (3 * kMemorySideCacheBytes / 4) / ((int64_t)n * 256) / nranges;
        if (shared_ranges) hot &= ~(int64_t)3; // four waves share the start of a range
        if (hot > per) hot = per;
        if (per * nranges >= ((int64_t)1 << 31) - 1) { // the kernel maps 32-bit indices: one range, nothing kept
            nranges = 1;
            per = nfull > 0 ? nfull : 1;
            hot = 0;
        }
        const bool stream_x = big_x && x_aligned; // slabs of unaligned rows share lines
        const uint32_t stride = 4u * (uint32_t)nparts, cold = (uint32_t)(per - hot);
        GramOrder go{(uint32_t)nranges, (uint32_t)per, (uint32_t)hot, 0, 0, 0, 0};
        if (cold) { go.q_cold = stride / cold; go.r_cold = stride % cold; }
        if (hot) { go.q_hot = stride / (uint32_t)hot; go.r_hot = stride % (uint32_t)hot; }
        // (the order is only worth its bookkeeping for an X well beyond the memory-side cache)
#define GRAM(NBV)                                                                                            \
    do {                                                                                                     \
        if (rt && stream_x) gram_mfma_kernel<NBV, true, 2><<<nparts, 64 * kGramWaves, 0, s>>>(X, n, D, ld, c->partials, *rt, go); \
        else if (rt && big_x) gram_mfma_kernel<NBV, true, 1><<<nparts, 64 * kGramWaves, 0, s>>>(X, n, D, ld, c->partials, *rt, go); \
        else if (rt) gram_mfma_kernel<NBV, true, 0><<<nparts, 64 * kGramWaves, 0, s>>>(X, n, D, ld, c->partials, *rt, go); \
        else if (stream_x) gram_mfma_kernel<NBV, false, 2><<<nparts, 64 * kGramWaves, 0, s>>>(X, n, D, ld, c->partials, NoRows{}, go); \
        else if (big_x) gram_mfma_kernel<NBV, false, 1><<<nparts, 64 * kGramWaves, 0, s>>>(X, n, D, ld, c->partials, NoRows{}, go); \
        else gram_mfma_kernel<NBV, false, 0><<<nparts, 64 * kGramWaves, 0, s>>>(X, n, D, ld, c->partials, NoRows{}, go); \
    } while (0)
        if (NB == 1) GRAM(1);
        else if (NB == 2) GRAM(2);
        else if (NB == 3) GRAM(3);
        else GRAM(4);
#undef GRAM
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(c, e);

    // few partials of few pairs: the bandwidth kernel sums them itself
    const bool direct = P <= kBwThreads && (int64_t)nparts * P <= kDirectMaxFloats;
    if (!direct) {
        KernelTimer t(c, SVGD_KERNEL_REDUCE, s);
        reduce_partials_kernel<<<dim3((P + 255) / 256, kSlices), 256, 0, s>>>(partials, nparts, P, c->part2);
    }
    e = hipGetLastError();
    if (e != hipSuccess) return fail(c, e);
    {
        KernelTimer t(c, SVGD_KERNEL_BANDWIDTH, s);
        bandwidth_kernel<<<1, kBwThreads, 0, s>>>(c->part2, direct ? partials : nullptr, nparts, n, mode, c->h_fixed,
                                                  c->state, c->coef);
    }
    e = hipGetLastError();
    if (e != hipSuccess) return fail(c, e);
    c->last_n = n;
    return SVGD_OK;
}

// Pass 3.  EMIT = false: X updated in place; EMIT = true: phi written to PHI.  CARRY (in-place,
// the update also leaves the Gram partials of the new X in c->partials.
template <bool EMIT, bool CARRY>
int run_update(svgd_ctx *c, float *X, const float *G, float *PHI, int n, int64_t D, int64_t ld, float eps,
               hipStream_t s, const RowTable *rt = nullptr)
{
    KernelTimer t(c, SVGD_KERNEL_UPDATE, s);
    // With carried sums one update follows the other with nothing but tiny kernels in between:
    // every other one walks X from the far end, so that it starts on what the previous one
    // touched last (the part of X that the memory-side cache still holds).
    FusedArgs ua{};
    if (!EMIT && CARRY) ua.reverse = (int)(c->sweeps++ & 1u);
    // the four waves of a workgroup on adjacent tiles: always at n > 48; below only for an X beyond
    // the memory-side cache (n = 32, D = 2,000,000, which just fits it, ran 3 % slower that way)
    ua.adjacent = adjacent_tiles(n, ld);
    if (n <= kValuMaxN) {
        const int64_t ngroups = (D + 3) / 4;
        // fewer, longer-lived workgroups when each one ends with a reduction of its pair sums
        // (with the pair sums of 9 to 12 particles in registers only one workgroup fits a CU)
        const int per_cu = CARRY ? (n <= 8 ? 2 : 1) : 8;
        const int grid = clampi((ngroups + 255) / 256, 1, mini(c->num_cu * per_cu, CARRY ? max_parts(c, n) : kMaxParts));
        if (CARRY) {
            c->carry_nparts = grid;
            c->carry_off = 0;
        }
#define CALL(N) launch_update_valu<N, EMIT, CARRY>(X, G, PHI, c->coef, c->state, D, ld, eps, c->partials, grid, s, rt, ua)
        SVGD_SWITCH_N(n, CALL)
#undef CALL
    } else {
        // workers walk contiguous ranges of full 64-column tiles; one more workgroup does D mod 64
        const int grid = update_workers(c, n, D, ld, CARRY) + 1;
        const int NB = (n + 15) / 16;
        if (CARRY) { // one partial per workgroup, the tail's included
            c->carry_nparts = grid;
            c->carry_off = 0;
        }
        // rows that all start on a 128-byte boundary (X's and G's) need no re-aligned stores and
        // can be read with streaming loads
        const bool aligned = !EMIT && (rt ? rt->aligned != 0 : rows_aligned(X, ld) && rows_aligned(G, ld));
#define UPD(NBV, FULL)                                                                                       \
    do {                                                                                                     \
        if (!EMIT && !CARRY && rt && aligned)                                                                \
            update_mfma_kernel<NBV, false, FULL, false, true, true><<<grid, 256, 0, s>>>(X, G, PHI, c->coef, c->state, n, D, ld, eps, c->partials, *rt, ua); \
        else if (!EMIT && !CARRY && rt)                                                                      \
            update_mfma_kernel<NBV, false, FULL, false, false, true><<<grid, 256, 0, s>>>(X, G, PHI, c->coef, c->state, n, D, ld, eps, c->partials, *rt, ua); \
        else if (!EMIT && aligned)                                                                           \
            update_mfma_kernel<NBV, false, FULL, CARRY, true, false><<<grid, 256, 0, s>>>(X, G, PHI, c->coef, c->state, n, D, ld, eps, c->partials, NoRows{}, ua); \
        else if (CARRY && ua.reverse)                                                                        \
            update_mfma_kernel<NBV, false, FULL, CARRY, false, false, false, CARRY><<<grid, 256, 0, s>>>(X, G, PHI, c->coef, c->state, n, D, ld, eps, c->partials, NoRows{}, ua); \
        else                                                                                                 \
            update_mfma_kernel<NBV, EMIT, FULL, CARRY, false, false><<<grid, 256, 0, s>>>(X, G, PHI, c->coef, c->state, n, D, ld, eps, c->partials, NoRows{}, ua); \
    } while (0)
        // one to four particles beyond a multiple of 16 ride along as remainder rows of the kernel
        // for that multiple
#define UPD_REM(NBV)                                                                                         \
    do {                                                                                                     \
        if (!EMIT && !CARRY && rt && aligned)                                                                \
            update_mfma_kernel<NBV, false, true, false, true, true, false, false, true><<<grid, 256, 0, s>>>(X, G, PHI, c->coef, c->state, n, D, ld, eps, c->partials, *rt, ua); \
        else if (!EMIT && !CARRY && rt)                                                                      \
            update_mfma_kernel<NBV, false, true, false, false, true, false, false, true><<<grid, 256, 0, s>>>(X, G, PHI, c->coef, c->state, n, D, ld, eps, c->partials, *rt, ua); \
        else if (!EMIT && aligned)                                                                           \
            update_mfma_kernel<NBV, false, true, CARRY, true, false, false, false, true><<<grid, 256, 0, s>>>(X, G, PHI, c->coef, c->state, n, D, ld, eps, c->partials, NoRows{}, ua); \
        else if (CARRY && ua.reverse)                                                                        \
            update_mfma_kernel<NBV, false, true, CARRY, false, false, false, CARRY, true><<<grid, 256, 0, s>>>(X, G, PHI, c->coef, c->state, n, D, ld, eps, c->partials, NoRows{}, ua); \
        else                                                                                                 \
            update_mfma_kernel<NBV, EMIT, true, CARRY, false, false, false, false, true><<<grid, 256, 0, s>>>(X, G, PHI, c->coef, c->state, n, D, ld, eps, c->partials, NoRows{}, ua); \
    } while (0)
        const bool rem = has_remainder_rows(n);
        if (rem && n < 32) UPD_REM(1);
        else if (rem && n < 48) UPD_REM(2);
        else if (rem) UPD_REM(3);
        else if (n == 16) UPD(1, true);
        else if (NB == 1) UPD(1, false);
        else if (n == 32) UPD(2, true);
        else if (n == 48) UPD(3, true);
        else if (n == 64) UPD(4, true);
        else if (NB == 2) UPD(2, false);
        else if (NB == 3) UPD(3, false);
        else UPD(4, false);
#undef UPD_REM
#undef UPD
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(c, e);
    return SVGD_OK;
}

// The fused step: one launch that starts with pass 2 in every workgroup (from the partials the
// previous update left at carry_off), updates X and leaves the partials of the new X in the other
// half of the scratch.  For short lists only: every workgroup reads the whole list.
// Every workgroup sums the whole list with its 256 threads - by groups of threads when there are few
// pairs (see kernel_matrix_prologue) - so what bounds the prologue is the number of partials one
// thread adds up, one dependent batch of 16 loads after the other.
constexpr int kFusedMaxChain = 160;

bool can_fuse(const svgd_ctx *c, int n)
{
    const int64_t P = (int64_t)n * (n + 1) / 2, half = (c->partials_cap / 2) & ~(int64_t)63;
    // On the matrix-core path (n > 12) the prologue runs with one wave per SIMD and measured slower
    // than the two launches it replaces (n = 16, D = 8,577: 15.1 against 12.4 us per step): only on request.
    const int max_n = (c->flags & SVGD_FLAG_FUSE_MFMA) ? 32 : kValuMaxN;
    if (n > max_n || (int64_t)c->carry_nparts * P > half) return false;
    int64_t chain;
    if (2 * P <= 256) {
        const int64_t KL = 256 / P < 32 ? 256 / P : 32;
        chain = (c->carry_nparts + KL - 1) / KL;
    } else {
        chain = (int64_t)c->carry_nparts * ((P + 255) / 256);
    }
    return chain <= kFusedMaxChain;
}

int run_update_fused(svgd_ctx *c, float *X, const float *G, int n, int64_t D, int64_t ld, float eps, hipStream_t s)
{
    KernelTimer t(c, SVGD_KERNEL_UPDATE, s);
    const int64_t P = (int64_t)n * (n + 1) / 2, half = (c->partials_cap / 2) & ~(int64_t)63;
    const FusedArgs fa{c->partials + c->carry_off, c->carry_nparts, c->h_fixed, (int)(c->sweeps++ & 1u), 0};
    const int64_t out_off = c->carry_off == 0 ? half : 0;
    float *gram_out = c->partials + out_off;
    const int cap = (int)(half / P < kMaxParts ? half / P : kMaxParts); // partials that fit into a half
    int grid;
    if (n <= kValuMaxN) {
        const int64_t ngroups = (D + 3) / 4;
        // all workgroups resident at once (9 to 12 particles: one per CU), or the prologue is paid twice
        grid = clampi((ngroups + 255) / 256, 1, mini(c->num_cu * (n <= 8 ? 2 : 1), cap));
#define CALL(N) launch_update_valu_fused<N>(X, G, c->coef, c->state, D, ld, eps, gram_out, grid, s, fa)
        SVGD_SWITCH_N(n, CALL)
#undef CALL
    } else {
        const int64_t nfull = D / 64;
        grid = clampi((nfull + 3) / 4, 1, mini(c->num_cu, cap - 1)) + 1;
        const bool aligned = rows_aligned(X, ld) && rows_aligned(G, ld);
#define UPD(NBV, FULL)                                                                                       \
    do {                                                                                                     \
        if (aligned)                                                                                         \
            update_mfma_kernel<NBV, false, FULL, true, true, false, true><<<grid, 256, 0, s>>>(X, G, nullptr, c->coef, c->state, n, D, ld, eps, gram_out, NoRows{}, fa); \
        else                                                                                                 \
            update_mfma_kernel<NBV, false, FULL, true, false, false, true><<<grid, 256, 0, s>>>(X, G, nullptr, c->coef, c->state, n, D, ld, eps, gram_out, NoRows{}, fa); \
    } while (0)
        if (has_remainder_rows(n)) { // 17..20
            if (aligned)
                update_mfma_kernel<1, false, true, true, true, false, true, false, true><<<grid, 256, 0, s>>>(X, G, nullptr, c->coef, c->state, n, D, ld, eps, gram_out, NoRows{}, fa);
            else
                update_mfma_kernel<1, false, true, true, false, false, true, false, true><<<grid, 256, 0, s>>>(X, G, nullptr, c->coef, c->state, n, D, ld, eps, gram_out, NoRows{}, fa);
        }
        else if (n == 16) UPD(1, true);
        else if (n < 16) UPD(1, false);
        else if (n == 32) UPD(2, true);
        else UPD(2, false);
#undef UPD
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(c, e);
    c->carry_nparts = grid;
    c->carry_off = out_off;
    c->last_n = n;
    return SVGD_OK;
}

// The single-launch path: sizes at which one workgroup does the whole step faster than three
// dependent launches.  It neither reads nor leaves carried pair sums.
bool is_tiny(int n, int64_t D) { return n <= kTinyMaxN && (int64_t)n * D <= kTinyMaxElems; }

template <int WHAT>
int run_tiny(svgd_ctx *c, float *X, const float *G, float *PHI, int n, int64_t D, int64_t ld, float eps, hipStream_t s)
{
    {
        KernelTimer t(c, WHAT == kTinyBandwidth ? SVGD_KERNEL_BANDWIDTH : SVGD_KERNEL_UPDATE, s);
#define TINY(N) step_tiny_kernel<N, WHAT><<<1, kTinyThreads, 0, s>>>(X, G, PHI, D, ld, eps, c->h_fixed, c->state, c->coef)
        switch (n) {
        case 1: TINY(1); break;
        case 2: TINY(2); break;
        case 3: TINY(3); break;
        case 4: TINY(4); break;
        case 5: TINY(5); break;
        case 6: TINY(6); break;
        case 7: TINY(7); break;
        default: TINY(8); break;
        }
#undef TINY
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(c, e);
    c->last_n = n;
    return SVGD_OK;
}

// ---------------------------------------------------------------------------------------------
// The entry point that allocates nothing: its scratch is a file-scope device array, one copy per
// GPU, resolved to a device address once per device.
// ---------------------------------------------------------------------------------------------
constexpr int kStaticMaxParts = 528;                         // partial vectors of n(n+1)/2 <= 2080 floats: 2 * 256 + 1 fit
constexpr size_t kStaticPartialsBytes = (size_t)kStaticMaxParts * kMaxPairsFull * sizeof(float);
constexpr size_t kStaticPart2Bytes = (size_t)kSlices * kMaxPairsFull * sizeof(double);
constexpr size_t kStaticCoefBytes = (size_t)kCoefFloats * sizeof(float);
constexpr size_t kStaticStateBytes = 256;
constexpr size_t kStaticBytes = kStaticPartialsBytes + kStaticPart2Bytes + kStaticCoefBytes + kStaticStateBytes;
static_assert(kStaticPartialsBytes % 256 == 0 && kStaticPart2Bytes % 256 == 0 && kStaticCoefBytes % 256 == 0,
              "every part of the scratch starts on a 256-byte boundary");
static_assert(sizeof(DevState) <= kStaticStateBytes, "state block");

// In host code this name is only a stand-in for the symbol: the memory is reached through the
// address that hipGetSymbolAddress returns for the current device (static_ctx below).
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

constexpr int kMaxDevices = 64;
struct StaticCtx {
    bool ready = false;
    svgd_ctx ctx;
};
std::mutex g_static_mutex;
StaticCtx g_static[kMaxDevices];

// The per-device context of svgd_step_static, set up on the first call on that device (which must
// be the current one).  Returns nullptr and sets *rc on failure.
svgd_ctx *static_ctx(int dev, int *rc)
{
    std::lock_guard<std::mutex> lock(g_static_mutex);
    StaticCtx &sc = g_static[dev];
    if (sc.ready) return &sc.ctx;
    unsigned char *ptr = nullptr;
    hipError_t e = hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || ptr == nullptr) {
        (void)hipGetLastError();
        *rc = SVGD_ERR_DEVICE;
        return nullptr;
    }
    int cus = 0;
    e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess || cus < 1) {
        (void)hipGetLastError();
        *rc = SVGD_ERR_DEVICE;
        return nullptr;
    }
    svgd_ctx &c = sc.ctx;
    c.magic = kMagic;
    c.device = dev;
    c.max_n = SVGD_MAX_PARTICLES;
    c.max_D = SVGD_STATIC_MAX_D;
    c.num_cu = cus > 256 ? 256 : cus; // keeps the Gram grid (2 workgroups per CU, one for the tail) within kStaticMaxParts
    c.flags = 0;
    c.h_fixed = 0.0;
    c.carry_valid = false;
    c.carry_X = nullptr;
    c.carry_n = 0;
    c.carry_D = c.carry_ld = 0;
    c.carry_nparts = 0;
    c.carry_off = 0;
    c.carry_stream = nullptr;
    c.sweeps = 0;
    c.last_n = 0;
    c.last_hip_error = 0;
    c.partials = reinterpret_cast<float *>(ptr);
    c.partials_cap = (int64_t)kStaticMaxParts * kMaxPairsFull;
    c.part2 = reinterpret_cast<double *>(ptr + kStaticPartialsBytes);
    c.coef = reinterpret_cast<float *>(ptr + kStaticPartialsBytes + kStaticPart2Bytes);
    c.state = reinterpret_cast<DevState *>(ptr + kStaticPartialsBytes + kStaticPart2Bytes + kStaticCoefBytes);
    c.profiling = false;
    c.profile_kinds = 0;
    sc.ready = true;
    return &c;
}

} // namespace

extern "C" {

int svgd_create(svgd_handle_t *out, int max_n, int64_t max_D, int device_id, uint32_t flags)
{
    if (!out) return SVGD_ERR_INVALID_ARG;
    *out = nullptr;
    if (max_n < 1 || max_D < 1 || (flags & ~(uint32_t)(SVGD_FLAG_CARRY_GRAM | SVGD_FLAG_FUSE_MFMA)) != 0 || device_id < -1)
        return SVGD_ERR_INVALID_ARG;
    if (max_n > SVGD_MAX_PARTICLES || max_D > SVGD_MAX_D) return SVGD_ERR_TOO_LARGE;

    svgd_ctx *c = new (std::nothrow) svgd_ctx();
    if (!c) return SVGD_ERR_ALLOC;
    c->magic = 0;
    c->max_n = max_n;
    c->max_D = max_D;
    c->flags = flags;
    c->h_fixed = 0.0;
    c->carry_valid = false;
    c->carry_X = nullptr;
    c->carry_n = 0;
    c->carry_D = 0;
    c->carry_ld = 0;
    c->carry_nparts = 0;
    c->carry_off = 0;
    c->carry_stream = nullptr;
    c->sweeps = 0;
    c->partials_cap = 0;
    c->last_n = 0;
    c->last_hip_error = 0;
    c->partials = nullptr;
    c->part2 = nullptr;
    c->state = nullptr;
    c->coef = nullptr;
    c->profiling = false;
    c->profile_kinds = ~0u;

    hipError_t e;
    int dev = device_id;
    if (dev < 0) {
        e = hipGetDevice(&dev);
        if (e != hipSuccess) { delete c; return SVGD_ERR_DEVICE; }
    }
    int count = 0;
    e = hipGetDeviceCount(&count);
    if (e != hipSuccess || dev >= count) { delete c; return e != hipSuccess ? SVGD_ERR_DEVICE : SVGD_ERR_INVALID_ARG; }
    c->device = dev;
    DeviceGuard guard(dev);
    int cus = 0;
    e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess || cus < 1) { delete c; return SVGD_ERR_DEVICE; }
    c->num_cu = cus > 512 ? 512 : cus; // keeps every persistent grid within kMaxParts workgroups

    const size_t P = (size_t)max_n * (max_n + 1) / 2;
    bool ok = hipMalloc(&c->partials, (size_t)kMaxParts * P * sizeof(float)) == hipSuccess &&
              hipMalloc(&c->part2, (size_t)kSlices * P * sizeof(double)) == hipSuccess &&
              hipMalloc(&c->state, sizeof(DevState)) == hipSuccess &&
              hipMalloc(&c->coef, (size_t)kCoefFloats * sizeof(float)) == hipSuccess;
    if (!ok) {
        (void)hipGetLastError();
        (void)hipFree(c->partials);
        (void)hipFree(c->part2);
        (void)hipFree(c->state);
        (void)hipFree(c->coef);
        delete c;
        return SVGD_ERR_ALLOC;
    }
    c->partials_cap = (int64_t)kMaxParts * (int64_t)P;
    c->magic = kMagic;
    {
        std::lock_guard<std::mutex> lock(g_live_mutex);
        live_handles().insert(c);
    }
    *out = c;
    return SVGD_OK;
}

int svgd_set_bandwidth(svgd_handle_t c, double h_fixed)
{
    int rc = check_handle(c);
    if (rc) return rc;
    if (std::isnan(h_fixed) || std::isinf(h_fixed)) return SVGD_ERR_INVALID_ARG;
    c->h_fixed = h_fixed > 0.0 ? h_fixed : 0.0;
    return SVGD_OK;
}

int svgd_forget_carry(svgd_handle_t c)
{
    int rc = check_handle(c);
    if (rc) return rc;
    c->carry_valid = false;
    return SVGD_OK;
}

int svgd_bandwidth_ld(svgd_handle_t c, const float *X, int n, int64_t D, int64_t ld, double *h_out_host,
                      void *stream)
{
    int rc = check_handle(c);
    if (rc) return rc;
    if (!X) return SVGD_ERR_INVALID_ARG;
    rc = check_shape(c, n, D, ld);
    if (rc) return rc;
    DeviceGuard guard(c->device);
    hipStream_t s = (hipStream_t)stream;
    if (is_tiny(n, D)) {
        rc = run_tiny<kTinyBandwidth>(c, const_cast<float *>(X), nullptr, nullptr, n, D, ld, 0.f, s);
    } else {
        c->carry_valid = false; // the partials buffer is about to be overwritten
        rc = run_kernel_matrix(c, X, n, D, ld, s, false);
    }
    if (rc) return rc;
    if (h_out_host) {
        hipError_t e = hipMemcpyAsync(h_out_host, &c->state->h, sizeof(double), hipMemcpyDeviceToHost, s);
        if (e == hipSuccess) e = hipStreamSynchronize(s);
        if (e != hipSuccess) return fail(c, e);
    }
    return SVGD_OK;
}

int svgd_bandwidth(svgd_handle_t c, const float *X, int n, int64_t D, double *h_out_host, void *stream)
{
    return svgd_bandwidth_ld(c, X, n, D, D, h_out_host, stream);
}

int svgd_step_ld(svgd_handle_t c, float *X, const float *G, int n, int64_t D, int64_t ld, float eps,
                 void *stream)
{
    int rc = check_handle(c);
    if (rc) return rc;
    if (!X || !G || !std::isfinite(eps)) return SVGD_ERR_INVALID_ARG;
    rc = check_shape(c, n, D, ld);
    if (rc) return rc;
    if (overlaps(X, G, n, D, ld)) return SVGD_ERR_INVALID_ARG;
    DeviceGuard guard(c->device);
    hipStream_t s = (hipStream_t)stream;
    const bool carry_mode = (c->flags & SVGD_FLAG_CARRY_GRAM) != 0;
    // the carried sums (and the tables derived from them) were written on carry_stream: a call
    // on another stream is not ordered after that work and recomputes from X
    const bool use_carry = carry_mode && c->carry_valid && c->carry_X == X && c->carry_n == n &&
                           c->carry_D == D && c->carry_ld == ld && c->carry_stream == s;
    c->carry_valid = false;
    if (is_tiny(n, D)) return run_tiny<kTinyStep>(c, X, G, nullptr, n, D, ld, eps, s);
    if (use_carry && can_fuse(c, n)) {
        rc = run_update_fused(c, X, G, n, D, ld, eps, s); // the whole step in one launch
    } else {
        rc = run_kernel_matrix(c, X, n, D, ld, s, use_carry, nullptr, G, carry_mode);
        if (rc) return rc;
        if (!use_carry) c->sweeps = 0; // a Gram pass ends at the near end of X: the update starts there
        if (!carry_mode) return run_update<false, false>(c, X, G, nullptr, n, D, ld, eps, s);
        rc = run_update<false, true>(c, X, G, nullptr, n, D, ld, eps, s);
    }
    if (rc) return rc;
    c->carry_valid = true;
    c->carry_X = X;
    c->carry_n = n;
    c->carry_D = D;
    c->carry_ld = ld;
    c->carry_stream = s;
    return SVGD_OK;
}

int svgd_step(svgd_handle_t c, float *X, const float *G, int n, int64_t D, float eps, void *stream)
{
    return svgd_step_ld(c, X, G, n, D, D, eps, stream);
}

int svgd_step_rows(svgd_handle_t c, float *const *X_rows, const float *const *G_rows, int n, int64_t D, float eps,
                   void *stream)
{
    int rc = check_handle(c);
    if (rc) return rc;
    if (!X_rows || !G_rows || !std::isfinite(eps)) return SVGD_ERR_INVALID_ARG;
    rc = check_shape(c, n, D, D);
    if (rc) return rc;
    // every row: non-null, 4-byte aligned; no two of the 2n rows may overlap
    struct Span { uintptr_t lo, hi; };
    Span spans[2 * SVGD_MAX_PARTICLES];
    const uintptr_t bytes = (uintptr_t)D * sizeof(float);
    for (int i = 0; i < n; ++i) {
        const uintptr_t px = (uintptr_t)X_rows[i], pg = (uintptr_t)G_rows[i];
        if (!px || !pg || (px & 3) || (pg & 3)) return SVGD_ERR_INVALID_ARG;
        spans[2 * i] = {px, px + bytes};
        spans[2 * i + 1] = {pg, pg + bytes};
    }
    std::sort(spans, spans + 2 * n, [](const Span &a, const Span &b) { return a.lo < b.lo; });
    for (int i = 1; i < 2 * n; ++i)
        if (spans[i].lo < spans[i - 1].hi) return SVGD_ERR_INVALID_ARG;
    // row starts relative to row 0 (float pointers are 4-byte aligned, so the differences are whole floats)
    RowTable rt;
    rt.aligned = 1;
    for (int i = 0; i < n; ++i)
        if (((uintptr_t)X_rows[i] | (uintptr_t)G_rows[i]) & 127u) rt.aligned = 0;
    for (int i = 0; i < kMaxN; ++i) {
        const int k = i < n ? i : 0;
        rt.x[i] = (int64_t)(((intptr_t)X_rows[k] - (intptr_t)X_rows[0]) / (intptr_t)sizeof(float));
        rt.g[i] = (int64_t)(((intptr_t)G_rows[k] - (intptr_t)G_rows[0]) / (intptr_t)sizeof(float));
        rt.ri[i] = (int32_t)(((uintptr_t)X_rows[k] >> 2) & 31u);
    }
    DeviceGuard guard(c->device);
    hipStream_t s = (hipStream_t)stream;
    c->carry_valid = false; // the partials buffer is about to be overwritten; nothing is carried for separate rows
    float *X = X_rows[0];
    const float *G = G_rows[0];
    rc = run_kernel_matrix(c, X, n, D, D, s, false, &rt);
    if (rc) return rc;
    return run_update<false, false>(c, X, G, nullptr, n, D, D, eps, s, &rt);
}

int svgd_phi_ld(svgd_handle_t c, const float *X, const float *G, int n, int64_t D, int64_t ld, float *PHI,
                void *stream)
{
    int rc = check_handle(c);
    if (rc) return rc;
    if (!X || !G || !PHI) return SVGD_ERR_INVALID_ARG;
    rc = check_shape(c, n, D, ld);
    if (rc) return rc;
    if (overlaps(X, PHI, n, D, ld) || overlaps(G, PHI, n, D, ld)) return SVGD_ERR_INVALID_ARG;
    DeviceGuard guard(c->device);
    hipStream_t s = (hipStream_t)stream;
    if (is_tiny(n, D)) return run_tiny<kTinyPhi>(c, const_cast<float *>(X), G, PHI, n, D, ld, 0.f, s);
    c->carry_valid = false; // the partials buffer is about to be overwritten
    rc = run_kernel_matrix(c, X, n, D, ld, s, false);
    if (rc) return rc;
    return run_update<true, false>(c, const_cast<float *>(X), G, PHI, n, D, ld, 0.f, s);
}

int svgd_phi(svgd_handle_t c, const float *X, const float *G, int n, int64_t D, float *PHI, void *stream)
{
    return svgd_phi_ld(c, X, G, n, D, D, PHI, stream);
}

int svgd_step_static(float *X, const float *G, int n, int64_t D, int64_t ld, float eps, void *stream)
{
    if (!X || !G || !std::isfinite(eps) || n < 1 || D < 1 || ld < D) return SVGD_ERR_INVALID_ARG;
    if (n > SVGD_MAX_PARTICLES || D > SVGD_STATIC_MAX_D) return SVGD_ERR_TOO_LARGE;
    if (overlaps(X, G, n, D, ld)) return SVGD_ERR_INVALID_ARG;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return SVGD_ERR_DEVICE;
    }
    if (dev < 0 || dev >= kMaxDevices) return SVGD_ERR_DEVICE;
    int rc = SVGD_OK;
    svgd_ctx *c = static_ctx(dev, &rc);
    if (!c) return rc;
    // Every part of the scratch that a kernel reads has been written by an earlier kernel of the
    // same call (partials by all workgroups of the pairwise-d2 pass, their sums, the state and
    // the coefficient tables by the passes after it): nothing has to start at zero.
    hipStream_t s = (hipStream_t)stream;
    if (is_tiny(n, D)) return run_tiny<kTinyStep>(c, X, G, nullptr, n, D, ld, eps, s);
    rc = run_kernel_matrix(c, X, n, D, ld, s, false, nullptr, G, false);
    if (rc) return rc;
    return run_update<false, false>(c, X, G, nullptr, n, D, ld, eps, s);
}

int svgd_get_last(svgd_handle_t c, double *h_out, float *K_host, void *stream)
{
    int rc = check_handle(c);
    if (rc) return rc;
    if (c->last_n < 1) return SVGD_ERR_INVALID_ARG;
    DeviceGuard guard(c->device);
    hipStream_t s = (hipStream_t)stream;
    hipError_t e = hipSuccess;
    if (h_out) e = hipMemcpyAsync(h_out, &c->state->h, sizeof(double), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess && K_host)
        e = hipMemcpyAsync(K_host, c->coef + kOffK, (size_t)c->last_n * c->last_n * sizeof(float),
                           hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return fail(c, e);
    return SVGD_OK;
}

int svgd_diag_copy(void *dst, const void *src, int64_t nbytes, void *stream)
{
    if (!dst || !src || nbytes < 16 || (nbytes & 15) || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15))
        return SVGD_ERR_INVALID_ARG;
    diag_copy_kernel<<<2048, 256, 0, (hipStream_t)stream>>>((const f32x4 *)src, (f32x4 *)dst, nbytes >> 4);
    return hipGetLastError() == hipSuccess ? SVGD_OK : SVGD_ERR_DEVICE;
}

int svgd_diag_axpy_rows(float *X, const float *G, int n, int64_t D, int64_t ld, float s, int pattern,
                        int workgroups, void *stream)
{
    const int base = pattern & 15, reverse = (pattern >> 4) & 1;
    if (!X || !G || n < 1 || D < 1 || ld < D || workgroups < 1 || workgroups > 65536 || pattern < 0 || pattern > 31 || base > 11)
        return SVGD_ERR_INVALID_ARG;
    if (overlaps(X, G, n, D, ld)) return SVGD_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
#define AXPY(PAT, U, NT) diag_axpy_rows_kernel<PAT, U, NT><<<workgroups, 256, 0, st>>>(X, G, n, D, ld, s, reverse)
    switch (base) {
    case 0: AXPY(0, 8, 0); break;
    case 1: AXPY(1, 8, 0); break;
    case 2: AXPY(0, 16, 0); break;
    case 3: AXPY(1, 16, 0); break;
    case 4: AXPY(0, 8, 1); break;
    case 5: AXPY(1, 8, 1); break;
    case 6: AXPY(0, 16, 1); break;
    case 7: AXPY(1, 16, 1); break;
    case 8: AXPY(0, 8, 2); break;
    case 9: AXPY(1, 8, 2); break;
    case 10: AXPY(0, 16, 2); break;
    default: AXPY(1, 16, 2); break;
    }
#undef AXPY
    return hipGetLastError() == hipSuccess ? SVGD_OK : SVGD_ERR_DEVICE;
}

int svgd_diag_read_rows(const float *X, int n, int64_t D, int64_t ld, float *sink, int pattern, int workgroups,
                        void *stream)
{
    if (!X || !sink || n < 1 || D < 1 || ld < D || workgroups < 1 || workgroups > 65536 || pattern < 0 || pattern > 3)
        return SVGD_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    switch (pattern) {
    case 0: diag_read_rows_kernel<0, 0><<<workgroups, 256, 0, st>>>(X, n, D, ld, sink); break;
    case 1: diag_read_rows_kernel<1, 0><<<workgroups, 256, 0, st>>>(X, n, D, ld, sink); break;
    case 2: diag_read_rows_kernel<0, 1><<<workgroups, 256, 0, st>>>(X, n, D, ld, sink); break;
    default: diag_read_rows_kernel<1, 1><<<workgroups, 256, 0, st>>>(X, n, D, ld, sink); break;
    }
    return hipGetLastError() == hipSuccess ? SVGD_OK : SVGD_ERR_DEVICE;
}

int swag_update_moments(float *mean, float *sqmean, const float *X, int n, int64_t D, int64_t count,
                        void *stream)
{
    if (!mean || !sqmean || !X || n < 1 || D < 1 || count < 0) return SVGD_ERR_INVALID_ARG;
    if (overlaps(mean, X, n, D, D) || overlaps(sqmean, X, n, D, D) || overlaps(mean, sqmean, n, D, D))
        return SVGD_ERR_INVALID_ARG;
    const int64_t total = (int64_t)n * D;
    const int64_t ngroups = (total + 3) / 4;
    int cus = 0, dev = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
        return SVGD_ERR_DEVICE;
    const int grid = clampi((ngroups + 255) / 256, 1, cus * 8);
    const float inv = (float)(1.0 / ((double)count + 1.0));
    swag_moments_kernel<<<grid, 256, 0, (hipStream_t)stream>>>(mean, sqmean, X, total, inv, count == 0);
    return hipGetLastError() == hipSuccess ? SVGD_OK : SVGD_ERR_DEVICE;
}

int svgd_profile_begin_kinds(svgd_handle_t c, unsigned kinds)
{
    int rc = check_handle(c);
    if (rc) return rc;
    if ((kinds & ((1u << SVGD_KERNEL_KINDS) - 1u)) == 0) return SVGD_ERR_INVALID_ARG;
    {   // all events and the record list exist before the first timed launch
        DeviceGuard guard(c->device);
        try {
            c->ev_kind.reserve(kMaxProfileRecords);
            c->ev_pool.reserve(2 * kMaxProfileRecords);
        } catch (...) {
            return SVGD_ERR_ALLOC;
        }
        while (c->ev_pool.size() < 2 * kMaxProfileRecords) {
            hipEvent_t e;
            hipError_t rc_e = hipEventCreate(&e);
            if (rc_e != hipSuccess) return fail(c, rc_e);
            c->ev_pool.push_back(e);
        }
    }
    c->ev_kind.clear();
    c->profile_kinds = kinds;
    c->profiling = true;
    return SVGD_OK;
}

int svgd_profile_begin(svgd_handle_t c) { return svgd_profile_begin_kinds(c, ~0u); }

int svgd_profile_end_records(svgd_handle_t c, double *ms_sum, int *count, int *rec_kind, float *rec_ms,
                             int rec_cap, int *rec_count)
{
    int rc = check_handle(c);
    if (rc) return rc;
    if (!ms_sum || !count || rec_cap < 0 || (rec_cap > 0 && (!rec_kind || !rec_ms))) return SVGD_ERR_INVALID_ARG;
    c->profiling = false;
    for (int k = 0; k < SVGD_KERNEL_KINDS; ++k) { ms_sum[k] = 0.0; count[k] = 0; }
    if (rec_count) *rec_count = 0;
    DeviceGuard guard(c->device);
    for (size_t r = 0; r < c->ev_kind.size(); ++r) {
        hipError_t e = hipEventSynchronize(c->ev_pool[2 * r + 1]);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, c->ev_pool[2 * r], c->ev_pool[2 * r + 1]);
        if (e != hipSuccess) { c->ev_kind.clear(); return fail(c, e); }
        ms_sum[c->ev_kind[r]] += (double)ms;
        count[c->ev_kind[r]] += 1;
        if ((int)r < rec_cap) {
            rec_kind[r] = c->ev_kind[r];
            rec_ms[r] = ms;
            if (rec_count) *rec_count = (int)r + 1;
        }
    }
    c->ev_kind.clear();
    return SVGD_OK;
}

int svgd_profile_end(svgd_handle_t c, double *ms_sum, int *count)
{
    return svgd_profile_end_records(c, ms_sum, count, nullptr, nullptr, 0, nullptr);
}

int svgd_destroy(svgd_handle_t c)
{
    int rc = check_handle(c);
    if (rc) return rc;
    {
        std::lock_guard<std::mutex> lock(g_live_mutex);
        live_handles().erase(c);
    }
    c->magic = 0;
    hipError_t e = hipSuccess, t;
    {
        DeviceGuard guard(c->device);
        if ((t = hipFree(c->partials)) != hipSuccess) e = t;
        if ((t = hipFree(c->part2)) != hipSuccess) e = t;
        if ((t = hipFree(c->state)) != hipSuccess) e = t;
        if ((t = hipFree(c->coef)) != hipSuccess) e = t;
        for (hipEvent_t ev : c->ev_pool) (void)hipEventDestroy(ev);
    }
    delete c;
    return e == hipSuccess ? SVGD_OK : SVGD_ERR_DEVICE;
}

int svgd_last_device_error(svgd_handle_t c)
{
    if (check_handle(c)) return 0;
    return c->last_hip_error;
}

const char *svgd_status_string(int status)
{
    switch (status) {
    case SVGD_OK: return "SVGD_OK";
    case SVGD_ERR_INVALID_ARG: return "SVGD_ERR_INVALID_ARG";
    case SVGD_ERR_BAD_HANDLE: return "SVGD_ERR_BAD_HANDLE";
    case SVGD_ERR_TOO_LARGE: return "SVGD_ERR_TOO_LARGE";
    case SVGD_ERR_ALLOC: return "SVGD_ERR_ALLOC";
    case SVGD_ERR_DEVICE: return "SVGD_ERR_DEVICE";
    default: return "SVGD_ERR_UNKNOWN";
    }
}

} // extern "C"
