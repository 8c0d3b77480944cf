/*
 * gaf.h -- C ABI of libgaf: Gradient Agreement Filtering (GAF) aggregation of
 * micro-gradients on one AMD MI355X (gfx950).
 *
 * The operation (paper: Sec. 3.1, Algorithm 1, Eq. 4, Eq. 5).  Given a
 * sequence of N micro-gradients g_1..g_N, each a flat vector of P parameters,
 * and a threshold tau:
 *
 *     g <- g_1, c <- 1
 *     for i = 2..N:   D_i = 1 - (g . g_i) / (|g| |g_i|)          (Eq. 4)
 *                     if D_i <= tau:  g <- g + g_i,  c <- c + 1   (Algorithm 1)
 *     g_GAF = g / c                                               (Eq. 5)
 *
 * D_i is taken against the running aggregate of the gradients accepted so
 * far. c == 1 at the end means that no two micro-gradients agreed; the paper
 * then skips the optimizer step -- that decision is the caller's, the library
 * reports c and still returns g_GAF = g_1.
 *
 * Conventions shared by every call
 *   - Pointers marked DEVICE are addresses in the memory of the GPU the
 *     context was created on; pointers marked HOST are ordinary host memory.
 *     The library never takes ownership of a caller's buffer and never frees
 *     one. It allocates device memory (and 64 bytes of pinned host memory)
 *     only inside gaf_create.
 *   - Every call enqueues its kernels on `stream` (a hipStream_t passed as
 *     void*, NULL = the default stream) and returns without waiting. Results
 *     are valid once the caller has synchronised that stream. Input buffers
 *     must stay valid and unmodified until then. No result is ever copied to
 *     the host and the accept/reject decisions are taken on the device.
 *   - The context's device must be the current HIP device of the calling
 *     thread. One context serves one stream at a time: calls on the same
 *     context from different streams or threads that may overlap on the GPU
 *     race on the context's workspace.
 *   - Vectors are contiguous. P may be any positive value (no multiple-of-4
 *     requirement). DEVICE vector pointers (gradients, accumulator, out) must
 *     be 16-byte aligned, otherwise GAF_EALIGN.
 *   - The running aggregate is kept as the running MEAN of the accepted
 *     gradients in binary32 (Eq. 4 does not change when one argument is
 *     rescaled, so distances against the mean equal distances against the
 *     paper's running sum; the mean makes the division of Eq. 5 implicit).
 *     Inner products and norms: the sequential passes and batches of up to 8
 *     gradients add exact products of the inputs in binary64. Larger batches on
 *     the Gram-first schedule use the matrix cores: products exact (bfloat16
 *     inputs) or to 2^-23 relative (binary32 inputs, three-way bfloat16 split),
 *     summed in binary32 inside the matrix core over at most 8 stages of 128 to
 *     512 columns, then added into binary64 totals. A binary32 sum of n terms
 *     rounds by at most n 2^-24 of the sum of the terms' magnitudes, and those
 *     roundings are not systematic, so an inner product is off by about
 *     1e-7 |x||y| at worst and far less on long vectors; the reported
 *     distances stay within 1e-6 of the binary64 value (tested down to 2500
 *     columns with all rows correlated at 0.98).
 *   - Ties: D_i == tau accepts. A zero-norm operand gives D_i = 1 by
 *     definition. A NaN distance (NaN or Inf in g_i) is stored as NaN and
 *     rejects g_i; the aggregate is left bit-for-bit unchanged.
 *     D_i is not clamped to [0, 2]. tau is compared in binary64.
 *   - Determinism: for a given (P, dtype) the launch shape and every summation
 *     order are fixed; no floating-point atomics are used. Repeating a call on
 *     the same inputs gives bit-identical outputs.
 *   - Timing knob (no result depends on it): the Gram-first pass that also
 *     writes the macro-gradient releases its stores in write windows of the
 *     GPU's constant 100 MHz clock, so that the memory is not turned around
 *     between reading and writing for every few KB. The environment variable
 *     GAF_WRITE_WINDOWS, read once per process, is "0" to switch the windows
 *     off or "PERIOD:WINDOW" (10 ns ticks, WINDOW < PERIOD) to fix them; left
 *     unset, period and window follow from the read/write mix of the call.
 *   - Errors are returned as gaf_status; nothing is thrown across the ABI.
 *     On any status other than GAF_OK nothing was enqueued, except GAF_EHIP,
 *     which reports a failed launch part-way (outputs are then undefined).
 */
#ifndef GAF_H
#define GAF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    GAF_OK = 0,
    GAF_EINVAL = 1,       /* NULL where a pointer is required, N < 1, P == 0, sizes beyond the context's */
    GAF_EALIGN = 2,       /* a DEVICE vector pointer is not 16-byte aligned */
    GAF_ENOMEM = 3,       /* gaf_create could not allocate its workspace (or a call its small host-side table) */
    GAF_EHIP = 4,         /* a HIP runtime call or kernel launch failed */
    GAF_EUNSUPPORTED = 5, /* unknown dtype, or N outside the range of the requested form */
    GAF_EDEVICE = 6,      /* the context's device is not the calling thread's current device */
    GAF_ELIMIT = 7        /* N or P beyond the fixed limits of gaf_aggregate_static */
} gaf_status;

/* Element type of the micro-gradients. The aggregate and `out` are always binary32. */
typedef enum {
    GAF_F32 = 0,  /* IEEE binary32 */
    GAF_BF16 = 1  /* bfloat16: the upper 16 bits of a binary32 */
} gaf_dtype;

typedef struct gaf_ctx gaf_ctx; /* opaque; owns only its own device workspace */

/*
 * Create a context on HIP device `device` able to serve calls with P <= max_P
 * and N <= max_N. Allocates the workspace (per-block partial sums, the device
 * decision state, and the partial Gram blocks gaf_pairwise needs).
 * *ctx (HOST) receives the handle. The current device is left as it was.
 */
gaf_status gaf_create(gaf_ctx **ctx, int device, size_t max_P, int max_N);

/* Free the workspace. The caller must have synchronised every stream that used the context. */
gaf_status gaf_destroy(gaf_ctx *ctx);

/* Static, never-freed description of a status code. */
const char *gaf_strerror(gaf_status status);

/*
 * Batch aggregation of one macrobatch: Algorithm 1 from seeding to g / c
 * (Sec. 3.1; Eq. 4 for the distance; Eq. 5 for the result).
 *
 *   grads        HOST array of N DEVICE pointers, each to P elements of `dt`.
 *                grads[0] is the seed g_1 (the paper draws the seed at random:
 *                the caller expresses that draw, and the visiting order, by
 *                how it orders this array). Read-only.
 *   tau          cosine-distance threshold; tau >= 2 admits everything and
 *                gives the plain mean (Eq. 2), tau < 0 keeps only the seed.
 *   out          DEVICE, P binary32: g_GAF. Also used as the running aggregate
 *                while the call runs; must not alias any input.
 *   accept_mask  DEVICE, N bytes: 1 if g_i was accepted, else 0; [0] = 1.
 *   cos_dist     DEVICE, N binary32: D_i as computed when g_i was visited;
 *                [0] = 0 (the seed is not compared with anything).
 *   count        DEVICE, one int32: c, the number of accepted gradients (>= 1).
 *
 * HBM traffic, sequential schedule, per visited gradient: the aggregate is read
 * once and g_i once for the distance; an accepted g_i is read a second time, in
 * the same pass that reduces the next gradient, when the aggregate is rewritten.
 * Gram-first schedule (the default for N <= 64, see gaf_set_schedule): every
 * gradient is read once, the accepted ones a second time, out is written once.
 */
gaf_status gaf_aggregate(gaf_ctx *ctx, const void *const *grads, int N, size_t P, gaf_dtype dt,
                         float tau, float *out, uint8_t *accept_mask, float *cos_dist,
                         int32_t *count, void *stream);

/*
 * How gaf_aggregate schedules its work. Both schedules implement the same
 * Algorithm 1 and give the same mask, count, distances and macro-gradient up
 * to rounding.
 *   SEQUENTIAL  one streaming pass per visited gradient: the distance of g_i to
 *               the running aggregate, with the update for g_{i-1} fused into
 *               the same pass (see the traffic note above).
 *   GRAM        the decisions depend on the gradients only through inner
 *               products (g_i . sum_A g_j = sum_{j in A} g_i . g_j, and likewise
 *               for the norm of the running sum), so: all-pairs inner products
 *               in ONE read of every gradient, an O(N^2) scalar replay of
 *               Algorithm 1 on the device, then Eq. 5 as one masked mean over
 *               the accepted gradients (c reads, one write). 2 <= N <= 64.
 *   AUTO        GRAM when 2 <= N <= 64, otherwise SEQUENTIAL. The default.
 *               For long vectors (P >= 2^26) AUTO additionally guesses
 *               the accept set from a sample of 2^22 elements of every gradient
 *               (256 runs of 2^14 consecutive elements; run r starts at element
 *               r * S, S = P / 256 rounded down to a multiple of 2^14, so the
 *               runs spread over all parts of the vector) and lets the Gram pass
 *               write the mean of that guess while it has the data staged on chip;
 *               once the full inner products are known the guess is checked on the
 *               device, and only a wrong guess costs the separate mean pass. When
 *               the guess names only a few gradients (fewer than a break-even
 *               count between 2 and 10 that depends on dtype and N) the Gram pass
 *               stays read-only and the separate mean pass, cheap for so few
 *               gradients, does the work. Shorter vectors (2^21 <= P < 2^26),
 *               where a sample would cost too large a share, use the accept set
 *               of the context's previous call with the same N as the guess
 *               (agreement drifts slowly over training; with two micro-batches
 *               the guess is simply "as last time"). A context also keeps a record of its
 *               guesses on the device: a written guess that proves wrong stops
 *               the writing for the next `penalty` calls (1 at first, doubling
 *               per miss up to 64, halving per hit), so callers whose distances
 *               sit close to tau stop paying for wrong guesses; nothing of this
 *               synchronises with the host. The result is the same in every
 *               case, bit for bit.
 * Explicit GRAM with N outside its range returns GAF_EUNSUPPORTED.
 */
typedef enum {
    GAF_SCHEDULE_AUTO = 0,
    GAF_SCHEDULE_SEQUENTIAL = 1,
    GAF_SCHEDULE_GRAM = 2
} gaf_schedule;

/*
 * Also clears the context's record of guesses: the next batch call that guesses
 * enqueues the clearing ahead of its own kernels (so a call captured into a
 * graph right after this one carries the clearing with it and forgets the
 * record at every replay; run one batch call eagerly first to avoid that).
 */
gaf_status gaf_set_schedule(gaf_ctx *ctx, gaf_schedule schedule);

/*
 * Diagnostics of AUTO's fused mean: copies the context's record of guesses to
 * the HOST array record[4] = { this call's Gram pass wrote the mean of its guess
 * (0/1), the guess was right and the result was left in place (0/1), calls still
 * to go without writing, penalty the next wrong guess will impose }.
 * Unlike every other call this one WAITS for the device to become idle first;
 * it is meant for tests and tuning, not for the training loop.
 */
gaf_status gaf_fused_mean_record(gaf_ctx *ctx, int32_t record[4]);

/*
 * Streaming form: one visit of Algorithm 1's inner loop for a gradient that
 * has just arrived. The state (accum, count) is DEVICE-resident, caller-owned,
 * and carried from call to call.
 *
 *   accum         DEVICE, P binary32, in/out: running mean of the accepted
 *                 gradients, i.e. g_GAF of everything seen so far.
 *   count         DEVICE, one int32, in/out: c. *count == 0 means "nothing seen
 *                 yet": g_i becomes the seed (accum <- g_i, c <- 1, reported
 *                 distance 0, accepted) and the previous contents of accum are
 *                 ignored.
 *   g_i           DEVICE, P elements of `dt`, read-only.
 *   cos_dist_out  DEVICE, one binary32, may be NULL: D_i.
 *   accepted_out  DEVICE, one byte, may be NULL: 1 if accepted.
 *
 * Two kernels: the distance reduction, then decision and conditional update in
 * one launch (every workgroup re-derives the decision from the partial sums; a
 * rejected g_i costs no further memory traffic). From P = 2^26 on: three (the
 * decision gets a launch of its own and the update runs one workgroup per tile).
 */
gaf_status gaf_step(gaf_ctx *ctx, float *accum, int32_t *count, const void *g_i, size_t P,
                    gaf_dtype dt, float tau, float *cos_dist_out, uint8_t *accepted_out,
                    void *stream);

/*
 * Streaming form with one step of look-ahead: the same visit of Algorithm 1's
 * inner loop as gaf_step -- same decision, same D_i, same count -- but the update
 * of the aggregate for an accepted g_i is NOT applied by this call. It stays
 * pending and is applied by the next gaf_step_lookahead on the same aggregate, in
 * the very walk over the vectors that takes the sums for the next gradient (one
 * pass over the aggregate per visit instead of two), or by gaf_flush.
 *
 *   After the call (and until the pending update has been applied) `accum` holds
 *   the mean of the gradients accepted BEFORE g_i, while *count already includes
 *   g_i; cos_dist_out and accepted_out are final.
 *   g_i must stay valid and unmodified until the NEXT gaf_step_lookahead or
 *   gaf_flush on this context has run on the device -- one call longer than with
 *   gaf_step.
 *   A context carries one pending gradient: consecutive calls must name the same
 *   accum, count, P and dtype (GAF_EINVAL otherwise), on the same stream. Any
 *   other call on the context that uses its decision state (gaf_step, the batch
 *   entry points) first applies a pending update on its own stream.
 *   Results are those of gaf_step, bit for bit, once the pending update is applied.
 * Two kernels per visit: update + sums in one walk, then the decision.
 */
gaf_status gaf_step_lookahead(gaf_ctx *ctx, float *accum, int32_t *count, const void *g_i, size_t P,
                              gaf_dtype dt, float tau, float *cos_dist_out, uint8_t *accepted_out,
                              void *stream);

/*
 * Applies the update gaf_step_lookahead left pending, if any (one kernel; no memory
 * traffic if that gradient was rejected). Afterwards accum is the mean of all
 * accepted gradients, as after gaf_step.
 */
gaf_status gaf_flush(gaf_ctx *ctx, void *stream);

/*
 * Diagnostic: Eq. 4 between every pair of the N micro-gradients, the quantity
 * the paper logs over training (Sec. 1, Fig. 1c/d).
 *
 *   grads  HOST array of N DEVICE pointers (as in gaf_aggregate).
 *   D      DEVICE, N*N binary32, row-major: D[i*N+j] = D_c(g_i, g_j);
 *          symmetric, diagonal exactly 0.
 *   gram   DEVICE, N*N binary64, row-major, may be NULL: the inner products
 *          g_i . g_j the distances were formed from.
 *
 * Every gradient is read once when N <= 64; for larger N, in 64-row panels.
 */
gaf_status gaf_pairwise(gaf_ctx *ctx, const void *const *grads, int N, size_t P, gaf_dtype dt,
                        float *D, double *gram, void *stream);

/*
 * Batch aggregation for a caller that already holds the inner products of the
 * same gradients: `gram` (DEVICE, N*N binary64, row-major) as written by
 * gaf_pairwise on this stream or synchronised before. Algorithm 1 is replayed
 * on the matrix and Eq. 5 is formed as in the Gram-first schedule; the Gram
 * pass itself is skipped, so the distance matrix of Fig. 1c/d and the filtered
 * macro-gradient together cost one read of every gradient plus one read of the
 * accepted ones. 1 <= N <= 64 (GAF_EUNSUPPORTED beyond); other arguments as in
 * gaf_aggregate.
 */
gaf_status gaf_aggregate_with_gram(gaf_ctx *ctx, const void *const *grads, int N, size_t P,
                                   gaf_dtype dt, float tau, const double *gram, float *out,
                                   uint8_t *accept_mask, float *cos_dist, int32_t *count, void *stream);

/*
 * The batch aggregation AND the all-pairs distance matrix of the same gradients
 * in one call (Algorithm 1 + Eq. 5, and Eq. 4 over every pair as in
 * gaf_pairwise): both come from the one Gram pass the Gram-first schedule makes
 * anyway, including the fused mean of the AUTO schedule for long vectors.
 *   D     DEVICE, N*N binary32 distances as in gaf_pairwise.
 *   gram  DEVICE, N*N binary64 inner products, may be NULL.
 * 1 <= N <= 64 (GAF_EUNSUPPORTED beyond); other arguments as in gaf_aggregate.
 * D and gram are bit for bit those of gaf_pairwise. For N <= 8 the plain
 * gaf_aggregate may add its partial inner products in another (equally fixed)
 * order, so its cos_dist can differ from this call's in the last bit.
 */
gaf_status gaf_aggregate_with_matrix(gaf_ctx *ctx, const void *const *grads, int N, size_t P,
                                     gaf_dtype dt, float tau, float *out, uint8_t *accept_mask,
                                     float *cos_dist, int32_t *count, float *D, double *gram, void *stream);

/*
 * Order-indifferent variant the paper sketches for the filter's dependence on
 * the seed (Sec. 3.1, last paragraph; the order-indifference item under future
 * research): every micro-gradient takes a turn as the seed, the others being
 * visited in ring order behind it (s, s+1, .., N-1, 0, .., s-1), and the run
 * with the largest agreement is kept. Readings taken: agreement = number of
 * accepted gradients; ties go to the lowest seed index. All N runs are replayed
 * on one Gram matrix, so the cost is that of the Gram-first batch call.
 *   accept_mask, cos_dist  indexed by gradient: mask[i], and the distance of
 *                          g_i when the winning run visited it (0 for its seed).
 *   seed                   DEVICE, one int32: index of the winning seed.
 * 1 <= N <= 64 (GAF_EUNSUPPORTED beyond); other arguments as in gaf_aggregate.
 */
gaf_status gaf_aggregate_best_seed(gaf_ctx *ctx, const void *const *grads, int N, size_t P,
                                   gaf_dtype dt, float tau, float *out, uint8_t *accept_mask,
                                   float *cos_dist, int32_t *count, int32_t *seed, void *stream);

/*
 * Batch aggregation fused with the GAF-SGD update (Algorithm 1's last lines,
 * Eq. 6) in the form of the optimizer the experiments name (Sec. 4.1: SGD with
 * momentum and an L2 weight decay; heavy-ball form, no dampening, no Nesterov):
 *     if c > 1:  d = g_GAF + weight_decay * params
 *                momentum_buf <- momentum * momentum_buf + d
 *                params <- params - lr * momentum_buf
 *     if c == 1: no two micro-gradients agreed -- params and momentum_buf are
 *                left bit-for-bit untouched (the paper's skipped step).
 * The update runs inside the pass that forms g_GAF, so it costs one read and
 * one write of params and momentum_buf and no pass of its own.
 *   params, momentum_buf  DEVICE, P binary32 each, in/out, 16-byte aligned,
 *                         distinct from each other, from out and from the inputs;
 *                         momentum_buf starts at zero before the first step.
 *   out                   DEVICE, P binary32, may be NULL: g_GAF (written also
 *                         when the step is skipped).
 * 1 <= N <= 64 (GAF_EUNSUPPORTED beyond); other arguments as in gaf_aggregate.
 */
gaf_status gaf_aggregate_sgd(gaf_ctx *ctx, const void *const *grads, int N, size_t P, gaf_dtype dt,
                             float tau, float *params, float *momentum_buf, float lr, float momentum,
                             float weight_decay, float *out, uint8_t *accept_mask, float *cos_dist,
                             int32_t *count, void *stream);

/*
 * Bucketed filtering (the per-bucket form of the distance that the paper lists
 * under future research, as a way to save memory and computation): the
 * parameter vector is cut into B contiguous buckets -- layers, or the
 * buckets of a gradient exchange -- and Algorithm 1 runs independently inside
 * each, with its own mask, distances and count.
 *   bucket_offsets  HOST array of B+1 element offsets, [0] = 0, [B] = P,
 *                   strictly increasing, every offset a multiple of 8 elements
 *                   (GAF_EALIGN otherwise) so that every slice stays 16-byte aligned.
 *   out             DEVICE, P binary32: per-bucket g_GAF, concatenated.
 *   accept_mask     DEVICE, B*N bytes, row b = bucket b.
 *   cos_dist        DEVICE, B*N binary32, row b = bucket b.
 *   count           DEVICE, B int32.
 * For N <= 8 and B <= 256 (unless the sequential schedule is forced) all
 * buckets are served by three launches: a segmented Gram pass, one filter
 * workgroup per bucket, a segmented mean. Otherwise each bucket is one batch
 * call under the context's schedule, enqueued in bucket order on `stream`.
 */
gaf_status gaf_aggregate_bucketed(gaf_ctx *ctx, const void *const *grads, int N, size_t P,
                                  gaf_dtype dt, float tau, int B, const size_t *bucket_offsets,
                                  float *out, uint8_t *accept_mask, float *cos_dist, int32_t *count,
                                  void *stream);

/*
 * gaf_aggregate for callers that cannot allocate device memory at all -- code
 * running under HIP graph capture, serving loops that must not call hipMalloc,
 * harnesses that forbid it -- and therefore cannot call gaf_create either.
 * Same operation, arguments, results and schedule selection (AUTO) as
 * gaf_aggregate; the workspace a context would own is a fixed array of about
 * 10.6 MB in the global memory of every device the library's code is loaded on,
 * held until the process ends. The call works on the calling thread's current
 * device, enqueues on `stream` and calls no hipMalloc, hipFree or other
 * allocating routine.
 *   Limits: N <= GAF_STATIC_MAX_N and P <= GAF_STATIC_MAX_P, else GAF_ELIMIT
 *   (nothing enqueued).
 *   All calls on one device share that device's array, which keeps what the
 *   last call left in it (including AUTO's record of guesses, as a context
 *   would): calls that may overlap on one device -- different streams or
 *   threads -- race on it. What has to start from zero is cleared by a small
 *   kernel ahead of the first call's own kernels on each device.
 * gaf_static_init looks up the current device's array ahead of time (one
 * runtime query, no allocation, nothing enqueued); calling it is optional, but
 * a caller that is about to start a graph capture should, so that the first
 * gaf_aggregate_static inside the capture has nothing left to look up.
 */
#define GAF_STATIC_MAX_N 64
#define GAF_STATIC_MAX_P ((size_t)1 << 36)
gaf_status gaf_static_init(void);
gaf_status gaf_aggregate_static(const void *const *grads, int N, size_t P, gaf_dtype dt, float tau,
                                float *out, uint8_t *accept_mask, float *cos_dist, int32_t *count,
                                void *stream);

/*
 * Launch timing, for benchmarks (not part of the paper's method). Between
 * gaf_profile_begin and gaf_profile_end every kernel the context enqueues is
 * bracketed by a pair of HIP events on the call's stream (up to max_launches
 * launches; later ones go untimed). gaf_profile_end waits for those events --
 * the only call besides gaf_create that blocks -- and writes one record per
 * timed launch, in launch order, into the HOST array `out` (capacity `cap`);
 * *n (HOST) receives how many. Event objects are host resources; no device
 * memory is allocated.
 */
typedef enum {
    GAF_K_INIT = 0,          /* one-thread set-up for N == 1 */
    GAF_K_SEED_REDUCE = 1,   /* first pass of a batch: adopt the seed, reduce against g_2 */
    GAF_K_REDUCE = 2,        /* reduce against g_i, applying the pending update on the way */
    GAF_K_UPDATE = 3,        /* conditional update alone */
    GAF_K_GRAM = 4,          /* all-pairs inner products */
    GAF_K_GRAM_FINALIZE = 5, /* ordered sum of the per-workgroup Gram tiles */
    GAF_K_DISTANCE = 6,      /* Gram matrix -> distance matrix */
    GAF_K_DECIDE = 7,        /* ordered sum of the partial sums, distance, accept/reject decision */
    GAF_K_FILTER = 8,        /* Gram-first schedule: Algorithm 1 replayed on the Gram matrix */
    GAF_K_MEAN = 9,          /* Gram-first schedule: mean of the accepted gradients (Eq. 5) */
    GAF_K_GRAM_SAMPLE = 10   /* inner products over a prefix of the vectors, to guess the accept set */
} gaf_kernel_id;

typedef struct {
    int32_t kernel; /* gaf_kernel_id */
    float ms;       /* elapsed time between the bracketing events, milliseconds */
} gaf_launch_time;

gaf_status gaf_profile_begin(gaf_ctx *ctx, int max_launches);
gaf_status gaf_profile_end(gaf_ctx *ctx, gaf_launch_time *out, int cap, int *n);

#ifdef __cplusplus
}
#endif
#endif /* GAF_H */
