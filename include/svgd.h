/*
 * svgd.h - C ABI of the MI355X (gfx950) SVGD all-particle update library.
 *
 * One SVGD step over n particles (paper App. B.2, "SVGD in Push": the leader's per-pair kernel
 * and kernel-gradient accumulation followed by the followers' in-place parameter update), in the
 * score/ascent convention and with the median-heuristic bandwidth:
 *
 *     d2_ij  = |x_i - x_j|^2
 *     h      = median(all n*n entries of d2) / ln(n+1)        (h <= 0 -> h = 1)
 *     K_ij   = exp(-d2_ij / h)                                 (the paper's exp(-|.|^2/(2 l^2)), h = 2 l^2)
 *     phi_i  = (1/n) sum_j [ K_ij g_j + (2/h) K_ij (x_i - x_j) ]
 *     x_i   <- x_i + eps * phi_i                               (every phi_i from the pre-step X)
 *
 * Particle i is the flattened parameter vector of one network (App. B.2: every particle's
 * parameters are gathered into one flat vector); g_i is its score grad log p(x_i) (a caller
 * holding loss gradients passes g = -grad; parameters without a gradient contribute zeros, as
 * in the paper's routine).
 *
 * Conventions for every entry point
 *   - X, G, PHI are DEVICE pointers to n x D fp32, row-major, leading dimension D (row i starts
 *     at element i*D) or, in the *_ld calls, ld >= D.  Only 4-byte alignment is required.  D and
 *     ld are 64-bit.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is
 *     enqueued on it; calls return before the work completes unless stated otherwise.
 *   - The caller owns X, G, PHI.  The handle owns its scratch (partial sums, K, h), allocated
 *     once in svgd_create and freed in svgd_destroy; svgd_step/svgd_phi/svgd_bandwidth never
 *     allocate.  The calls on one handle must be stream-ordered: one host thread at a time, and
 *     a call on another stream than the previous one only after the caller has ordered that
 *     stream behind the earlier work (different handles are independent).
 *   - Return value: SVGD_OK (0) or a negative svgd_status.  No entry point aborts or throws.
 *     Non-finite DATA is not checked and propagates as IEEE NaN/Inf.
 */
#ifndef SVGD_H
#define SVGD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct svgd_ctx *svgd_handle_t;

enum svgd_status {
    SVGD_OK = 0,
    SVGD_ERR_INVALID_ARG = -1, /* null pointer, n < 1, D < 1, ld < D, non-finite eps, X aliases G/PHI */
    SVGD_ERR_BAD_HANDLE = -2,  /* null handle or handle already destroyed */
    SVGD_ERR_TOO_LARGE = -3,   /* n > max_n, D > max_D, or max_n / max_D beyond SVGD_MAX_PARTICLES / SVGD_MAX_D */
    SVGD_ERR_ALLOC = -4,       /* device or host allocation failed */
    SVGD_ERR_DEVICE = -5       /* a HIP call failed; see svgd_last_device_error */
};

#define SVGD_MAX_PARTICLES 64
/* Longest particle a handle accepts: 2^36 parameters (256 GiB per particle, more than the part holds;
 * the kernels count 64-column tiles in 32 bits). */
#define SVGD_MAX_D ((int64_t)1 << 36)

/*
 * svgd_create flag.  The kernel matrix of step t+1 depends only on X after step t (paper App. B.2,
 * closing remarks: a particle is updated only after the whole kernel matrix of the previous
 * iterate exists).  With this flag svgd_step, while it still holds every updated column on chip,
 * also accumulates the pairwise sums of the NEW X, and the next svgd_step on the same (X, n, D)
 * skips its own pass over X (and, when the list of carried sums is short - small and medium
 * problems - runs as a single kernel launch).  The caller promises that between two svgd_step calls X is modified
 * by nobody else; after touching X (or to be safe) call svgd_forget_carry.  svgd_bandwidth and
 * svgd_phi always recompute from X and drop the carried sums, and so does a svgd_step on another
 * stream than the step that produced them.
 * Successive steps on carried sums walk the columns of X in alternating directions (the new X is
 * the same either way), so that each starts on the part of X that is still in the memory-side
 * cache; the direction is chosen when the call is made.  A caller who captures steps into a HIP
 * graph keeps that benefit by capturing an even number of consecutive steps per graph.
 */
#define SVGD_FLAG_CARRY_GRAM 1u
/*
 * With carried sums, a step whose list of carried partial sums is short runs as ONE kernel launch
 * (the update kernel derives h and K itself, in every workgroup) - by default only on the
 * vector-ALU path, n <= 12, where that measures faster than two launches.  This flag extends it to
 * 13 <= n <= 32, where it measures slower (one launch of 15 us against two launches in 12 us at
 * n = 16, D = 8,577): for measurements, and for callers to whom the launch count matters more.
 */
#define SVGD_FLAG_FUSE_MFMA 2u

/*
 * Create a handle for problems up to max_n particles (1..SVGD_MAX_PARTICLES) of up to max_D (<= SVGD_MAX_D)
 * parameters each on HIP device `device_id` (-1 = the current device); the sizes play the part of
 * the paper's `num_particles` and of the flattened parameter count of its networks (App. B.2, the
 * arguments of the top-level SVGD inference call; its `lengthscale` is svgd_set_bandwidth, its
 * `lr` the eps of svgd_step).  `flags`: 0 or an OR of the SVGD_FLAG_* values above.  Allocates the handle's
 * device scratch: 8192 * max_n * (max_n + 1) / 2 bytes of partial sums (17 MB at max_n = 64) and
 * about 0.2 MB of tables.  On success *out receives the handle.
 */
int svgd_create(svgd_handle_t *out, int max_n, int64_t max_D, int device_id, uint32_t flags);

/*
 * Fix the bandwidth: h > 0 selects the paper's fixed-lengthscale kernel (App. B.2,
 * `lengthscale` l with h = 2 l^2) and skips the median; h <= 0 restores the median heuristic
 * (the default).  Takes effect for subsequent calls.
 */
int svgd_set_bandwidth(svgd_handle_t h, double h_fixed);

/* Drop the pairwise sums carried from the last svgd_step (see SVGD_FLAG_CARRY_GRAM). */
int svgd_forget_carry(svgd_handle_t h);

/*
 * Compute d2, h, K and the row sums of K for X (device, n x D) and keep them in the handle
 * (App. B.2: the radius^2 / exp step of the per-pair kernel, done once for all pairs).
 * If h_out_host is non-NULL the stream is synchronised and *h_out_host (HOST memory) receives h;
 * with NULL nothing is copied and the call does not synchronise.
 */
int svgd_bandwidth(svgd_handle_t h, const float *X, int n, int64_t D, double *h_out_host,
                   void *stream);

/*
 * One whole SVGD step, in place: X <- X + eps * phi(X, G).  X (device, n x D) is read, then
 * overwritten; G (device, n x D) is read only (App. B.2: the leader's per-pair kernel value and
 * kernel-gradient accumulation and the followers' parameter update, all particles at once).
 * Does not synchronise or allocate.
 */
int svgd_step(svgd_handle_t h, float *X, const float *G, int n, int64_t D, float eps, void *stream);

/*
 * Diagnostic variant of svgd_step: the same kernels, but phi itself - the averaged update vector
 * that App. B.2's leader sends to each follower - is written to PHI (device, n x D) and X is left
 * untouched.
 */
int svgd_phi(svgd_handle_t h, const float *X, const float *G, int n, int64_t D, float *PHI,
             void *stream);

/*
 * The same three calls for particles stored with a leading dimension: row i of X, G and PHI
 * starts at element i*ld of its array (ld >= D, the same ld for all arrays of one call; the
 * ld - D floats between rows are neither read nor written).  svgd_bandwidth, svgd_step and
 * svgd_phi are these with ld = D.  A caller who can choose the layout should make ld a multiple
 * of 32 floats and allocate on a 128-byte boundary: every row then starts on a cache-line
 * boundary, no line is shared by two rows or fetched twice, and the large-n update runs 3-4 %
 * faster than on densely packed rows (paper App. B.2 gathers each particle into a flat vector of
 * its own; how those vectors are spaced in memory is this library's choice to offer).
 * Carried pair sums (SVGD_FLAG_CARRY_GRAM) are keyed on (X, n, D, ld).
 */
int svgd_bandwidth_ld(svgd_handle_t h, const float *X, int n, int64_t D, int64_t ld,
                      double *h_out_host, void *stream);
int svgd_step_ld(svgd_handle_t h, float *X, const float *G, int n, int64_t D, int64_t ld, float eps,
                 void *stream);
int svgd_phi_ld(svgd_handle_t h, const float *X, const float *G, int n, int64_t D, int64_t ld,
                float *PHI, void *stream);

/*
 * svgd_step for particles that are n separately allocated vectors (App. B.2: the leader gathers
 * every particle's parameters and gradients, each particle's own flat vector, before it forms
 * the pairwise terms; here they are used where they lie, no copy into one matrix).  X_rows and
 * G_rows are HOST arrays of n DEVICE pointers: X_rows[i] is particle i's D parameters, G_rows[i]
 * its D scores (fp32, 4-byte aligned, any spacing or order; the 2n vectors must not overlap).
 * The arrays are read during the call and need not outlive it.  Plain step: bandwidth from the
 * median (or svgd_set_bandwidth), pair sums recomputed from X; carried sums are neither used nor
 * left behind.  Same results as svgd_step on the packed matrix.  Fastest when all 2n vectors
 * start on 128-byte boundaries (what separately allocated buffers do): then results are stored
 * directly and G is streamed past the caches, as for a matrix with padded rows; otherwise every
 * row has its own alignment, stores are re-aligned per row and nothing streams.  INVALID_ARG: null or misaligned row pointer, overlapping rows; otherwise as svgd_step.
 * Does not synchronise or allocate.
 */
int svgd_step_rows(svgd_handle_t h, float *const *X_rows, const float *const *G_rows, int n, int64_t D,
                   float eps, void *stream);

/*
 * Copy the bandwidth and kernel matrix (App. B.2: the per-pair kernel values, which the paper's
 * routine reads back one by one) of the most recent svgd_bandwidth/svgd_step/svgd_phi call
 * to HOST memory: *h_out (nullable) receives h; K_host (nullable, row-major) receives K and must
 * have room for n*n floats with the n of that call - the library copies exactly that many and
 * cannot check the buffer.  Synchronises `stream` first.  INVALID_ARG if no step has run yet.
 */
int svgd_get_last(svgd_handle_t h, double *h_out, float *K_host, void *stream);

/*
 * Per-kernel timing for benchmarks.  Between svgd_profile_begin and svgd_profile_end every kernel
 * launched through this handle is bracketed by a pair of HIP events on the stream it is launched
 * on.  svgd_profile_end waits for those events and fills ms_sum[k] / count[k] (HOST arrays of
 * SVGD_KERNEL_KINDS entries) with the total elapsed milliseconds and the number of launches of
 * kernel kind k, then switches recording off.  At most 2048 launches are recorded per session;
 * the events are created by svgd_profile_begin*, none while recording.
 * Not every kind runs in every step: a short list of partial sums is reduced inside the
 * BANDWIDTH kernel (no REDUCE launch), carried pair sums replace the GRAM pass, a short list of
 * carried sums at n <= 32 is consumed by the UPDATE kernel itself (the whole step is then that one
 * launch), and problems with n <= 8 and n * D <= 16384 run as one kernel, which is counted as
 * UPDATE (as BANDWIDTH when svgd_bandwidth launches it).
 */
enum svgd_kernel_kind {
    SVGD_KERNEL_GRAM = 0,      /* pairwise-d2 partial sums (pass over X) */
    SVGD_KERNEL_REDUCE = 1,    /* fp64 reduction of the partials */
    SVGD_KERNEL_BANDWIDTH = 2, /* median, h, K, coefficient tables */
    SVGD_KERNEL_UPDATE = 3,    /* fused update (pass over X and G, X written) */
    SVGD_KERNEL_KINDS = 4
};
int svgd_profile_begin(svgd_handle_t h);
/* The same, timing only the kinds whose bit (1u << kind) is set in `kinds`: every timed kernel
 * costs two event records on the stream, a few microseconds between kernels. */
int svgd_profile_begin_kinds(svgd_handle_t h, unsigned kinds);
int svgd_profile_end(svgd_handle_t h, double *ms_sum, int *count);
/* The same, and the single launches as well: record r < min(rec_cap, launches recorded), in launch
 * order, puts its kernel kind into rec_kind[r] and its elapsed milliseconds into rec_ms[r] (HOST
 * arrays of rec_cap entries; may be NULL with rec_cap = 0); *rec_count (nullable) receives the
 * number of records written. */
int svgd_profile_end_records(svgd_handle_t h, double *ms_sum, int *count, int *rec_kind, float *rec_ms,
                             int rec_cap, int *rec_count);

/*
 * Diagnostic: a plain device-to-device copy kernel of nbytes (a multiple of 16; dst and src
 * DEVICE pointers, 16-byte aligned, not overlapping), enqueued on `stream`.  It reads and writes
 * exactly nbytes, which makes it the yardstick for scaling hardware byte counters when the
 * other kernels are profiled.
 */
int svgd_diag_copy(void *dst, const void *src, int64_t nbytes, void *stream);

/*
 * Diagnostic: the memory traffic of the fused update and nothing else - x_i <- x_i + s * g_i in
 * place for n rows of D floats, ld floats apart (X, G DEVICE pointers as in svgd_step_ld; 12 bytes
 * moved per element over the same 2n row streams, no kernel matrix, no contraction).  Timing it on
 * the buffers a benchmark uses gives the rate that this part's memory system sustains for the
 * update's read-read-write mix, the practical ceiling beside the nominal HBM peak.  `pattern`
 * 0 and 2: a wave instruction covers 4 rows x 256 bytes (the matrix-core update's shape), 1 and 3:
 * 1 KiB of one row (the vector-ALU update's shape), with 8 (patterns 0, 1) or 16 (2, 3) loads per
 * array in flight per lane; patterns 4..7 are 0..3 with the loads carrying the streaming
 * (no-allocate) hint as well as the stores, 8..11 are 0..3 with that hint on the loads of G only
 * (the update's own policy: X stays cacheable); adding 16 to a pattern walks the columns from the
 * far end, so that calls which alternate p and p + 16 start each pass on what the previous one
 * left in the memory-side cache, as successive steps of a CARRY_GRAM handle do.  Other values:
 * SVGD_ERR_INVALID_ARG.  `workgroups` (1..65536) of 256 threads stride over the column tiles.
 * Enqueued on `stream` of the current device; does not synchronise or allocate.
 */
int svgd_diag_axpy_rows(float *X, const float *G, int n, int64_t D, int64_t ld, float s, int pattern,
                        int workgroups, void *stream);

/*
 * Diagnostic: the memory traffic of the pairwise-distance pass and nothing else - every element of
 * the n rows of X (DEVICE, D floats each, ld floats apart, 4-byte aligned) is read once, 4 bytes
 * per element, and added up; workgroup w leaves its sum in sink[w] (DEVICE array of `workgroups`
 * floats, the caller's).  Timing it on the buffers a benchmark uses gives the rate that this part's
 * memory system sustains for a pure read of these row streams: the practical ceiling of the pass
 * that forms the pair sums.  `pattern` 0: a wave instruction covers 4 rows x 256 bytes (the
 * matrix-core pass's shape), 1: 1 KiB of one row (the vector-ALU pass's shape); 2, 3: the same
 * with the streaming (no-allocate) hint on the loads.  Other values: SVGD_ERR_INVALID_ARG.
 * `workgroups` (1..65536) of 256 threads stride over the column tiles.  Enqueued on `stream` of the
 * current device; does not synchronise or allocate.
 */
int svgd_diag_read_rows(const float *X, int n, int64_t D, int64_t ld, float *sink, int pattern, int workgroups,
                        void *stream);

/*
 * Multi-SWAG running moments (paper Sec. 2: SWAG keeps the first and second moments of a
 * network's parameter trajectory, multi-SWAG for every particle of the ensemble).  Absorbs one
 * more iterate X (DEVICE, n x D fp32, row-major, contiguous) into the running means after `count`
 * earlier updates (count = 0 overwrites them):
 *     mean <- (count*mean + x)/(count+1),   sqmean <- (count*sqmean + x*x)/(count+1),
 * in place in mean and sqmean (DEVICE, same shape as X, caller-owned, must not overlap X or each
 * other).  The diagonal SWAG covariance is sqmean - mean^2.  Needs no handle; enqueued on `stream`
 * of the current device; does not synchronise or allocate.  INVALID_ARG: null pointer, n < 1,
 * D < 1, count < 0, overlapping arrays.
 */
int swag_update_moments(float *mean, float *sqmean, const float *X, int n, int64_t D, int64_t count,
                        void *stream);

/*
 * svgd_step_ld for callers that cannot allocate: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  No handle: the scratch (partial sums, their reduction,
 * h, K and the coefficient tables, 4.6 MB) is a static device array inside the library, one copy
 * per GPU, held until the process ends.  Plain step on the current device: median-heuristic
 * bandwidth, pair sums recomputed from X every call (nothing is carried), X updated in place;
 * same kernels and results as svgd_step_ld on a handle created with flags = 0.  Calls no
 * hipMalloc/hipFree or any other allocating routine and does not synchronise; the first call on
 * a device looks up the array's device address (make that call outside graph capture).
 * Limits: n <= SVGD_MAX_PARTICLES, D <= SVGD_STATIC_MAX_D, else SVGD_ERR_TOO_LARGE.  Every call
 * on one GPU uses the same scratch, which keeps the previous call's contents (each call
 * overwrites what it reads; nothing needs clearing): calls that overlap in time on one GPU -
 * different streams without ordering between them, several host threads - race.  Other errors as
 * svgd_step_ld.
 */
#define SVGD_STATIC_MAX_D ((int64_t)1 << 32)
int svgd_step_static(float *X, const float *G, int n, int64_t D, int64_t ld, float eps, void *stream);

/* Free the handle's scratch and invalidate the handle.  The caller synchronises beforehand. */
int svgd_destroy(svgd_handle_t h);

/* hipError_t value of the most recent failed HIP call on this handle (0 if none). */
int svgd_last_device_error(svgd_handle_t h);

/* Static, human-readable name of a status code. */
const char *svgd_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* SVGD_H */
