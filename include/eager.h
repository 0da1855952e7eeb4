/*
 * eager.h - C ABI of the eager-SGD hot path on one MI355X (gfx950).
 *
 * What the library computes (paper: "Taming Unbalanced Training Workloads in Deep
 * Learning with Partial Collective Operations", PPoPP'20):
 *
 *   P processes train data-parallel.  Each round every process owns a fresh gradient
 *   G_p and a send buffer R_p that is either empty (G_null) or holds the gradient the
 *   process finished too late for the previous round (Section 5, walk-through of
 *   Fig. 7).  A partial allreduce (Section 4) does not wait for everybody: processes
 *   that are on time ("active", Section 7.1) contribute R_p + G_p and end with an empty
 *   send buffer; late ("passive") processes contribute only R_p, and the gradient they
 *   finish late becomes the new R_p.  The sum of the contributions is scaled by 1/P
 *   (Algorithm 2, line 6) and handed to the update rule U (Algorithm 2, lines 7-8),
 *   here heavy-ball momentum SGD:  v <- mu*v + u ;  w <- w - lr*v.
 *
 *   All P processes are simulated on one GPU: their gradient and send buffers are
 *   P device arrays, and one kernel pass per round does reduce + carry + update.
 *
 * Conventions
 *   - Every function returns an eager_status; no exception crosses the boundary.
 *   - "device" pointers are HIP device memory owned by the caller; the library never
 *     allocates, frees or clears them.  "host" pointers are ordinary host memory.
 *   - Kernels are enqueued on the caller's stream (a hipStream_t passed as void*,
 *     NULL = the default stream).  No call synchronises the device, allocates or clears
 *     device memory, so a sequence of calls can be captured in a HIP graph; the first use
 *     of a kernel sets a function attribute, so run one round eagerly before capturing.
 *   - Arena layout: each of G_p, R_p, w, v, recv is one flat array per process in
 *     which bucket b occupies elements [bucket_offset[b], bucket_offset[b] +
 *     bucket_numel[b]).  Bucket starts are multiples of 16 bytes of the gradient type
 *     (4 fp32 / 8 bf16 elements).  Elements between consecutive buckets of one call's
 *     range are padding that the library may read and overwrite; they carry no data.
 *   - A context is not thread-safe; distinct contexts are independent.
 */
#ifndef EAGER_H
#define EAGER_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct eager_ctx eager_ctx;   /* opaque: bucket table, send-buffer validity, last error */

typedef enum { EAGER_SOLO = 0, EAGER_MAJORITY = 1, EAGER_QUORUM = 2 } eager_mode;
typedef enum { EAGER_F32 = 0, EAGER_BF16 = 1 } eager_dtype;          /* type of G only */
typedef enum { EAGER_ORDER_FIXED = 0, EAGER_ORDER_FAST = 1 } eager_order;

typedef enum {
    EAGER_OK = 0,
    EAGER_EINVAL = 1,    /* bad argument: NULL, P outside 1..64, misaligned pointer, empty range */
    EAGER_ESHAPE = 2,    /* bucket table malformed (overlap, misaligned start, negative size)    */
    EAGER_ESTATE = 3,    /* plan does not fit the context or the entry point, or a bucket is
                            given the same round twice                                           */
    EAGER_EDEVICE = 4,   /* a HIP call or a kernel launch failed                                 */
    EAGER_ENOMEM = 5,    /* host allocation failed                                               */
    EAGER_ELIMIT = 6     /* beyond the fixed capacity of the entry point that allocates nothing  */
} eager_status;

#define EAGER_MAX_P 64
#define EAGER_FLAG_STRICT_QUORUM 1u

/* Participation of one round: bit p of `mask` is the response bit s_t^p of Section 6.1
 * (whether the process's update entered this round's result).  nap = number of active processes (Section 7.1). */
typedef struct {
    int32_t  mode;        /* eager_mode */
    int32_t  P;
    uint64_t step;        /* round index t */
    uint64_t mask;
    int32_t  initiator;   /* rank that triggered the round */
    int32_t  nap;         /* popcount(mask) >= 1 (Lemma 1, quorum size) */
    uint32_t flags;       /* EAGER_FLAG_* the plan was made under (0 for a plan built by hand
                             without such a promise) */
    uint32_t reserved;    /* 0 */
} eager_plan;

/* Update rule U of Algorithm 2, lines 7-8: momentum SGD.  params/momentum are device
 * arena base pointers (fp32, 16-byte aligned), updated in place. */
typedef struct {
    float *params;
    float *momentum;
    float  lr;
    float  mu;
} eager_opt;

/*
 * Create a context for P processes and n_buckets layer-wise buckets (Section 3: one
 * reduction per layer, possibly fused).  bucket_offset / bucket_numel: host arrays of
 * n_buckets element counts, copied.  Buckets must be ascending and disjoint, starts
 * aligned as described above.  All send buffers start empty.
 *   order FIXED: contributions are added in ascending rank order starting from +0.0f,
 *                1/P is one fp32 multiplication, the update rule is two fused
 *                multiply-adds - results are reproducible bit for bit.
 *   order FAST : the library may reassociate the sum and contract multiply-adds.
 * Errors: EINVAL (NULL, P, n_buckets < 1, unknown dtype/order), ESHAPE, ENOMEM.
 */
int eager_create(eager_ctx **out, int P, int n_buckets, const int64_t *bucket_offset,
                 const int64_t *bucket_numel, int grad_dtype, int order);
int eager_destroy(eager_ctx *ctx);                 /* NULL is allowed */

/* Text of the last error of this context (owned by the context, valid until its next
 * call); eager_status_string names a status code (static storage). */
const char *eager_last_error(const eager_ctx *ctx);
const char *eager_status_string(int status);

/* Digest of the sources and headers this library was compiled from, as the build script
 * computes it ("unknown" for a build that bypassed the script); static storage.  The test
 * suite compares it with the digest of the sources in the tree, so that a stale library is
 * never the one that gets tested or timed. */
const char *eager_source_hash(void);

/*
 * Decide who is active in round `step` from the times (ms, host array of P doubles,
 * measured from a common origin per round) at which the processes reach the collective.
 * Host only, pure, deterministic.
 *   EAGER_SOLO     (Section 4.1) the first process to arrive is the initiator.
 *   EAGER_MAJORITY (Section 4.2) the initiator is a rank all processes derive from a
 *                  shared seed: SplitMix64 output function of seed + (step+1)*gamma,
 *                  reduced mod P.
 * Active = the initiator and every process that arrived no later than the initiator
 * plus window_ms (Section 7.1; the window models the activation reaching processes that
 * arrive at a similar time, Section 4.2; use 0 for the paper's definition).  Ties count
 * as on time; a tie for first place goes to the lowest rank.
 * flags: EAGER_FLAG_STRICT_QUORUM (majority only) also waits for ceil(P/2) arrivals, the
 *        literal reading of "at least half of the processes" (Section 4.2, first paragraph);
 *        the flag is recorded in out->flags, and eager_partial_allreduce_majority refuses a
 *        plan that carries it with fewer than ceil(P/2) active processes.
 * Errors: EINVAL (NULL, P outside 1..64, unknown mode, NaN time, negative window).
 */
int eager_plan_participation(int mode, int P, const double *arrival_ms, uint64_t seed,
                             uint64_t step, double window_ms, uint32_t flags,
                             eager_plan *out);

/*
 * The spectrum between solo, majority and a full allreduce that the paper's conclusions
 * (Section 9) propose: the round triggers when `quorum` (1..P) processes have reached the
 * collective.  The initiator is the quorum-th arrival (ties: lowest rank first); active =
 * every process that arrived no later than the initiator plus window_ms.  quorum = 1 gives
 * the solo participation set, quorum = P a full allreduce.  out->mode is EAGER_QUORUM.
 * Host only, pure.  Errors: EINVAL (NULL, P outside 1..64, quorum outside 1..P, NaN time,
 * negative window).
 */
int eager_plan_quorum(int P, const double *arrival_ms, int quorum, uint64_t step,
                      double window_ms, eager_plan *out);

/*
 * Processes that keep their own clock (Section 5, last paragraph): the k-th call of a process
 * belongs to the k-th execution of the collective, and the processes whose call has reached the
 * execution that is open wait at it.  eager_plan_open_round decides, from who is waiting, whether
 * execution `round` is triggered now:
 *   EAGER_SOLO      (Section 4.1) as soon as anybody waits; the initiator is the lowest waiting
 *                   rank (several wait only if they arrived at the same instant)
 *   EAGER_MAJORITY  (Section 4.2) when the designated initiator of this round - the rank all
 *                   processes draw from the shared seed, eager_designated_initiator - waits
 *   EAGER_QUORUM    (Section 9) when `quorum` (1..P) processes wait; the initiator is `newest`
 * waiting: bit p = process p waits (not empty); newest: the rank among them that arrived last.
 * *triggered becomes 1 or 0; when 1, *out is the plan of the execution: the waiting processes
 * are the active ones (they arrived no later than the initiator, Section 7.1), step = round.
 * Host only, pure.  Errors: EINVAL (NULL, P outside 1..64, unknown mode, empty or out-of-range
 * waiting set, newest not waiting, quorum outside 1..P in quorum mode).
 */
int eager_designated_initiator(uint64_t seed, uint64_t round, int P, int *rank);
int eager_plan_open_round(int mode, int P, uint64_t waiting, int newest, int quorum,
                          uint64_t seed, uint64_t round, int *triggered, eager_plan *out);

/*
 * One round of the partial allreduce over buckets [b0, b1) (Section 5; Algorithm 2
 * line 6), optionally fused with the update rule (lines 7-8).
 *   plan    host; produced by eager_plan_participation or built by the caller
 *   grads   host array of P device pointers: G_p arena bases (fp32 or bf16 as created),
 *           16-byte aligned, read only
 *   resid   host array of P device pointers: R_p arena bases (fp32), 16-byte aligned.
 *           Read where the process' send buffer is non-empty, written for passive
 *           processes; content is meaningful only where the validity bit is set
 *   recv    device, fp32 arena base or NULL: receive buffer, gets u = sum/P (Section
 *           4.1.1: holds the value of the latest execution)
 *   opt     host or NULL.  Non-NULL: w and v are updated in the same pass.  NULL:
 *           only recv is produced (then recv must not be NULL)
 * On success the validity of every bucket in the range becomes ~mask (the late processes).
 * The three entry points run the same kernels and differ in what they accept:
 * _solo requires plan->mode == EAGER_SOLO, _majority EAGER_MAJORITY, _quorum EAGER_QUORUM;
 * _majority also requires nap >= ceil(P/2) of a plan whose flags hold EAGER_FLAG_STRICT_QUORUM.
 * Errors: EINVAL (NULL, alignment, b0 >= b1, range), ESTATE (mode or P mismatch,
 * initiator not in mask, nap != popcount(mask), mask beyond P bits, unknown flag bits, a strict
 * majority plan without its quorum, bucket already stepped with this plan->step), EDEVICE.
 * Launch shapes are checked for every run of the call before the first kernel is enqueued, so
 * EDEVICE can only come from the HIP runtime; after EDEVICE the buckets of the call are in an
 * undefined state (some runs may have been enqueued): set their validity again with
 * eager_set_valid before going on.  Non-finite gradients are not an error; they
 * propagate through the arithmetic.
 */
int eager_partial_allreduce_solo(eager_ctx *ctx, const eager_plan *plan, int b0, int b1,
                                 const void *const *grads, float *const *resid,
                                 float *recv, const eager_opt *opt, void *stream);
int eager_partial_allreduce_majority(eager_ctx *ctx, const eager_plan *plan, int b0, int b1,
                                     const void *const *grads, float *const *resid,
                                     float *recv, const eager_opt *opt, void *stream);
int eager_partial_allreduce_quorum(eager_ctx *ctx, const eager_plan *plan, int b0, int b1,
                                   const void *const *grads, float *const *resid,
                                   float *recv, const eager_opt *opt, void *stream);

/*
 * One round over the whole model in which the gradient a late process finishes becomes its send
 * buffer WITHOUT being copied (Section 5: the late gradient is "stored in the send buffer" - here
 * the buffer it was produced in simply takes that role).  For fp32 gradients only, where both
 * buffers have the same layout.  The round reads the on-time gradients, the pending send buffers,
 * w and v, and writes w and v: 4 * (active + pending) + 16 bytes per element instead of
 * 4 * P + 4 * pending + 4 * late + 16.  Results (w, v, recv, and what every pending send buffer
 * holds) are those of eager_partial_allreduce_* bit for bit.
 *   grads, resid   host arrays of P device pointers as above, but the call MODIFIES them: for
 *                  every late process p the two entries are exchanged - resid[p] then points to
 *                  the buffer that holds the late gradient (pending, validity bit set) and
 *                  grads[p] to the former send buffer, whose content has been delivered and which
 *                  is free for the process's next gradient.  Entries of on-time processes stay.
 *                  The caller must use the tables as they come back for every later call.
 *                  (Under stream capture the pointers are fixed in the graph as they were when
 *                  the call was captured, like the plan; a replay repeats that one round on
 *                  those buffers and does not exchange anything again.)
 * Any plan mode is accepted; the range is always every bucket of the context (the exchange of a
 * process's arena pointers concerns all of its buckets).
 * Errors: as eager_partial_allreduce_*; ESTATE also for a context with bf16 gradients.  On an
 * error the tables are unchanged.
 */
int eager_partial_allreduce_exchange(eager_ctx *ctx, const eager_plan *plan, const void **grads,
                                     float **resid, float *recv, const eager_opt *opt,
                                     void *stream);

/*
 * Processes that lag by more than one round (Section 5, last paragraph).  The entry points
 * above assume that every process that is not on time still finishes its gradient before
 * the next round (it is stored into the send buffer as part of the round).  With
 * eager_partial_allreduce_lagging, processes in `absent` (a mask disjoint from plan->mask)
 * finish no gradient in this round's window: they contribute what their send buffer holds
 * and store nothing (grads[p] is not read and may be NULL); afterwards their send buffer is
 * empty.  Any plan mode is accepted.  When such a process finishes a gradient later, between
 * two rounds, eager_stash puts it into the send buffer of buckets [b0, b1): R_p <- G if the
 * buffer is empty, R_p <- R_p + G if it still holds an undelivered gradient (one fp32 add
 * per element, buffer first), and marks the buffer non-empty.  A late process of a round is
 * exactly an absent one followed by eager_stash of its gradient.
 * Errors: as eager_partial_allreduce_*; ESTATE if absent intersects plan->mask or has bits
 * beyond P; eager_stash: EINVAL (NULL, alignment, process or range outside), EDEVICE.
 */
int eager_partial_allreduce_lagging(eager_ctx *ctx, const eager_plan *plan, uint64_t absent,
                                    int b0, int b1, const void *const *grads,
                                    float *const *resid, float *recv, const eager_opt *opt,
                                    void *stream);
int eager_stash(eager_ctx *ctx, int process, int b0, int b1, const void *grad, float *resid,
                void *stream);

/*
 * The round in which nobody hands over a gradient (what is left in the send buffers when
 * training ends; Section 6.1: every update is applied once, now or later): every pending send
 * buffer of buckets [b0, b1) is delivered - u = (sum of the pending R_p, ascending rank, from
 * +0.0f) / P goes to recv and, with opt, through the update rule like any other round's result
 * (u = 0 where nothing was pending: the momentum still acts) - and all send buffers of the range
 * are empty afterwards.  It has no initiator and no round index (a plan cannot express it:
 * Lemma 1 wants at least one active process), so it may follow any round.
 * Errors: EINVAL (NULL resid, alignment, range, recv and opt both NULL), EDEVICE.
 */
int eager_flush(eager_ctx *ctx, int b0, int b1, float *const *resid, float *recv,
                const eager_opt *opt, void *stream);

/* The update rule alone (Algorithm 2, lines 7-8) on buckets [b0, b1): reads u from
 * `update` (device fp32 arena, e.g. a receive buffer), updates opt->params/momentum.
 * Errors: EINVAL, EDEVICE. */
int eager_sgd_step(eager_ctx *ctx, int b0, int b1, const float *update,
                   const eager_opt *opt, void *stream);

/*
 * A weight view per process (processes that lag by more than one round apply only the
 * results they see, so their weights differ; Section 5, last paragraph).
 * eager_sgd_step_views applies the update rule with one read of `update` to each of the
 * n_views (1..64) parameter/momentum pairs (host arrays of device pointers, fp32 arenas,
 * 16-byte aligned, pairwise distinct) - the processes that see this result.
 * eager_average_views is the periodic model synchronisation: every listed array is
 * replaced by the average of all of them (sum in the order given starting from +0.0f, times
 * 1/n_views in fp32: the arithmetic of a round in which everybody is on time); call it once
 * for the parameter views and once for the momentum views.
 * Errors: EINVAL (NULL, alignment, n_views, range, the same buffer listed twice), EDEVICE.
 */
int eager_sgd_step_views(eager_ctx *ctx, int b0, int b1, const float *update, int n_views,
                         float *const *params, float *const *momentum, float lr, float mu,
                         void *stream);
int eager_average_views(eager_ctx *ctx, int b0, int b1, int n_views, float *const *views,
                        void *stream);

/*
 * Variants of the update rule U (the paper leaves U generic, Algorithm 2 line 7).  They apply
 * to every later fused round and eager_sgd_step of this context:
 *     g  = u + weight_decay * w        (skipped when weight_decay == 0)
 *     v' = mu * v + g
 *     w' = w - lr * (nesterov ? g + mu * v' : v')
 * each line one fused multiply-add in fixed-order mode.  The default (0, 0) is heavy-ball
 * momentum SGD.  Errors: EINVAL (negative or non-finite weight_decay, nesterov not 0/1).
 */
int eager_set_update_rule(eager_ctx *ctx, float weight_decay, int nesterov);

/*
 * Optional per-bucket by-products of a round, computed in the same pass over HBM (what
 * layer-wise update rules and gradient-norm monitoring need; U is generic in the paper):
 *   sumsq_update  sum of u_i^2 over the bucket's elements with finite u_i, u = the averaged
 *                 result of the round (Algorithm 2 line 6); squares and sums in fp64
 *   sumsq_params  the same over the parameters w_i BEFORE the update (0 without opt)
 *   nonfinite     number of elements whose u_i is NaN or infinite
 * The sums are formed in a fixed order (no atomics): reproducible bit for bit from run to run
 * for a given launch shape; against another implementation compare with a tolerance.
 */
typedef struct {
    double   sumsq_update;
    double   sumsq_params;
    uint64_t nonfinite;
    float    rate;          /* written by eager_sgd_step_lars; 0 after a round */
    uint32_t reserved;
} eager_bucket_stats;

/*
 * eager_stats_attach: from now on every eager_partial_allreduce_* call of this context also
 * writes stats[b] for each bucket b it covers (overwritten by every call).
 *   stats      device array of n_buckets entries, 16-byte aligned, caller-owned; NULL detaches
 *   workspace  device memory, 16-byte aligned, caller-owned, at least
 *              eager_stats_workspace_bytes() bytes; the library keeps the bucket table, one
 *              32-byte record per wavefront of the round kernel and 129 per bucket there.  It
 *              must stay allocated while attached, and is shared by all calls of this context: with
 *              statistics attached, the calls of a context must be ordered (one stream, or
 *              events), and no other context may use the same workspace concurrently
 *   stream     the bucket table is written into the workspace by a small kernel on this stream
 *              (rounds that use the statistics must be ordered after it, e.g. on the same
 *              stream)
 * Needs the default number of streams in flight per wavefront (launch key "chunk" of
 * eager_tuning.h at 0 or 16); otherwise the next round fails with ESTATE.  One extra small
 * kernel runs per launch.
 * Errors: EINVAL (NULL ctx, workspace too small or misaligned), ENOMEM, EDEVICE.
 */
int eager_stats_workspace_bytes(const eager_ctx *ctx, int64_t *bytes);
int eager_stats_attach(eager_ctx *ctx, eager_bucket_stats *stats, void *workspace,
                       int64_t workspace_bytes, void *stream);

/*
 * eager_sgd_step with a rate per layer (layer = bucket): layer-wise adaptive rate scaling (You,
 * Gitman, Ginsburg 2017), one more instance of the generic update rule U of Algorithm 2
 * line 7, for the large batches that the paper's Section 7.3 says need tuned rates.  With
 * u = update (the averaged result of a round run with recv and without opt), per bucket b over
 * its finite elements, norms from fp64 sums of squares:
 *     rate_b = trust * |w_b| / (|u_b| + weight_decay * |w_b| + eps)   if |w_b| > 0 and |u_b| > 0
 *            = 1                                                      otherwise
 * (fp64, rounded to fp32 once), then per element, with weight_decay and nesterov as set by
 * eager_set_update_rule:
 *     g = rate_b * (u + weight_decay * w);  v' = mu * v + g;
 *     w' = w - lr * (nesterov ? g + mu * v' : v')
 * Two passes over the buckets (norms, then update: 8 + 20 bytes per element); padding between
 * buckets takes the rate of the bucket before it.
 * Needs eager_stats_attach: the workspace holds the partial sums, and stats[b] of every bucket
 * in [b0, b1) is overwritten with sumsq_update, sumsq_params (before the step), nonfinite and
 * rate.  The sums are formed in a fixed order (reproducible run to run); another summation
 * order can move a rate by one unit in the last place, so against another implementation
 * compare w and v with a tolerance even in fixed-order mode.
 * Errors: EINVAL (NULL or misaligned pointers, trust <= 0, eps < 0, non-finite), ESHAPE,
 * ESTATE (no statistics attached), EDEVICE.  Enqueues on `stream`, never synchronises.
 */
int eager_sgd_step_lars(eager_ctx *ctx, int b0, int b1, const float *update, const eager_opt *opt,
                        float trust, float eps, void *stream);

/*
 * eager_sgd_step_lars for callers that cannot allocate device memory at all - code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc - and so cannot bring the
 * workspace that eager_stats_attach wants.  Same kernels and the same results bit for bit; the
 * workspace (bucket table, per-wavefront records, partials) is a fixed device array inside the
 * library instead, EAGER_STATIC_SCRATCH_BYTES per GPU, held until the process ends.  The call
 * allocates, frees and copies nothing: the bucket table is written by a small kernel from the
 * kernel arguments.  No eager_stats_attach is needed (an attached workspace is left alone).
 *   stats   device array of n_buckets entries, 16-byte aligned, caller-owned: receives
 *           sumsq_update, sumsq_params (before the step), nonfinite and rate of every bucket in
 *           [b0, b1)
 * Limits: a context of at most EAGER_STATIC_MAX_BUCKETS buckets whose arena spans at most
 * EAGER_STATIC_MAX_ELEMENTS elements (first bucket start to last bucket end); beyond that the
 * call returns EAGER_ELIMIT and launches nothing.
 * All calls on one GPU share the array and it keeps the last call's contents (every record that
 * is read has been written by the same call before, so nothing needs clearing): calls that
 * overlap in time on one GPU - two streams, two contexts, two threads - race; order them.
 * Errors: as eager_sgd_step_lars without ESTATE; EINVAL also for a NULL or misaligned stats;
 * ELIMIT; EDEVICE.
 */
#define EAGER_STATIC_MAX_BUCKETS 512
#define EAGER_STATIC_MAX_ELEMENTS (1ll << 27)
#define EAGER_STATIC_SCRATCH_BYTES 18884864ll
int eager_sgd_step_lars_static(eager_ctx *ctx, int b0, int b1, const float *update,
                               const eager_opt *opt, float trust, float eps,
                               eager_bucket_stats *stats, void *stream);

/* Send-buffer validity of one bucket (bit p: R_p holds an undelivered gradient);
 * together with w, v, R and the round index this is all the state a resume needs. */
int eager_get_valid(const eager_ctx *ctx, int bucket, uint64_t *valid_mask);
int eager_set_valid(eager_ctx *ctx, int bucket, uint64_t valid_mask);

#ifdef __cplusplus
}
#endif
#endif /* EAGER_H */
