/*
 * gcada.h -- C-ABI of the G-CADA hot path for AMD MI355X (gfx950).
 *
 * G-CADA (grouping-based communication-adaptive distributed Adam) runs a parameter-server
 * loop over G groups of M_G workers; every worker of a group holds the same data shard
 * (paper Sec. IV).  This library simulates all groups of that loop on ONE GPU.  One call of
 * gcada_step is one iteration k of Algorithm 1 for all groups at once:
 *
 *   a1  each group g evaluates the minibatch gradient (gradient of the SUM of the per-sample
 *       losses over its minibatch xi_g^k, Sec. II-A) twice on the same samples: at the current
 *       iterate theta^k and at theta_stale_g = theta^{k - tau_g}, the iterate of its last upload;
 *   a2  stat_g = || grad(theta^k; xi_g^k) - grad(theta_stale_g; xi_g^k) ||^2 -- the quantity
 *       that the left side of the selection rule Eq. (9) estimates (Sec. III) -- is compared
 *       with rhs = (c/D) * sum_{d=1..D} || theta^{k+1-d} - theta^{k-d} ||^2 (right side of
 *       Eq. (9) with c_d = c/D).  Group g is selected when stat_g > rhs, or tau_g >= D
 *       (Algorithm 1), or rhs == 0;
 *   a3  the lazily aggregated gradient (Sec. IV; Eq. (3)) is updated with the innovations of the
 *       selected groups: agg += grad_g - last_g, last_g <- grad_g, tau_g <- 1; the other groups
 *       keep their stored gradient and tau_g <- tau_g + 1 (Algorithm 1);
 *   a4  server update, Eq. (8a)-(8c): h <- b1 h + (1-b1) agg;  v <- b2 vhat + (1-b2) agg^2;
 *       vhat <- max(vhat, v);  theta^{k+1} = theta^k - alpha h / sqrt(eps + vhat);  and
 *       || theta^{k+1} - theta^k ||^2 enters the history of Eq. (9).
 *
 * Every step above runs in hand-written HIP kernels; there is no CPU fallback.  All entry
 * points return a status code (0 = GCADA_OK) and never throw or abort; on error, output
 * arguments are left untouched and gcada_last_error gives a message.
 *
 * Pointers are marked [host] or [device].  "Borrowed" memory stays owned by the caller and
 * must stay valid while the context uses it.  Unless said otherwise a call is asynchronous on
 * the given HIP stream and does not synchronise with the host.  A context is not thread-safe;
 * all calls on one context must use one stream (or be ordered by the caller).
 *
 * Parameter vector layout theta[p]:
 *   logistic regression: theta[d], no intercept; labels y in {-1,+1};
 *                        loss = log(1 + exp(-y x.theta)) + (l2/2)||theta||^2 per sample.
 *   MLP: for each layer l = 1..L:  W_l (n_l x n_{l-1}, row-major) then b_l (n_l);
 *        a_l = ReLU(W_l a_{l-1} + b_l), logits = W_L a_{L-1} + b_L, softmax cross-entropy,
 *        ReLU'(0) = 0.
 */
#ifndef GCADA_H
#define GCADA_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gcada_ctx gcada_ctx;   /* opaque, owned by the library */

enum {
    GCADA_OK = 0,
    GCADA_EINVAL = 1,   /* bad argument (message says which)            */
    GCADA_ENOMEM = 2,   /* device or host allocation failed             */
    GCADA_EDEVICE = 3,  /* a HIP call failed                            */
    GCADA_ESTATE = 4    /* call order: shards / theta not set yet, ...  */
};

/* GCADA_LINREG: linear model with the quadratic error loss 0.5 (x.theta - y)^2, the model of
 * the paper's experiment (Sec. VI); real-valued fp32 targets.  It shares every kernel of
 * GCADA_LOGREG; only the residual of a row differs. */
enum { GCADA_LOGREG = 0, GCADA_MLP = 1, GCADA_LINREG = 2 };
enum { GCADA_F32 = 0, GCADA_BF16 = 1 };

#define GCADA_MAX_WIDTHS 8

/* Model and batch geometry (Algorithm 1's problem statement). */
typedef struct gcada_dims {
    int32_t model;      /* GCADA_LOGREG | GCADA_MLP | GCADA_LINREG                           */
    int32_t dtype;      /* storage type of X and of the weights the gradients are evaluated
                           at: GCADA_F32, or GCADA_BF16 (MLP only: bf16 X, bf16 copy of theta,
                           fp32 accumulation, fp32 master theta and moments)                 */
    int32_t n_widths;   /* LOGREG, LINREG: 1; MLP: number of layer widths incl. input, 2..8  */
    int32_t widths[GCADA_MAX_WIDTHS]; /* LOGREG, LINREG: {d}; MLP: {n_0, ..., n_L}           */
    int32_t batch;      /* mu: minibatch size per group (fixed, Sec. II-A)                   */
    float   l2;         /* lambda >= 0; must be 0 for GCADA_BF16                             */
} gcada_dims;

/*
 * Create a context for G groups of M_G workers (Sec. IV), history depth / maximum age D >= 1
 * and rule constant c >= 0 (Eq. (9)), stepsize alpha > 0, momentum weights beta1, beta2 in
 * [0,1) and eps > 0 (Eq. (8a)-(8c)).  M_G only enters gcada_cost_model; the numerics do not
 * depend on it (one gradient per selected group is uploaded, Sec. IV).
 * Allocates all state on the current HIP device.  Synchronous.
 * Errors: GCADA_EINVAL (dims / ranges), GCADA_ENOMEM, GCADA_EDEVICE.
 */
int gcada_create(const gcada_dims* dims /*[host]*/, int32_t G, int32_t M_G, int32_t D, double c,
                 double alpha, double beta1, double beta2, double eps,
                 gcada_ctx** out /*[host]*/);

/* Frees the context and all device state.  NULL is allowed.  Synchronous. */
void gcada_destroy(gcada_ctx* ctx);

/*
 * Give group g its data shard D_g (Sec. IV: all workers of a group hold the same shard, so one
 * copy per group).  X: rows x widths[0], row-major with leading dimension ld (elements), fp32 or
 * bf16 per dims.dtype.  y: rows entries; fp32 in {-1,+1} for LOGREG, int32 class id in
 * [0, n_L) for MLP.  Both [device], BORROWED until destroy or the next set_shard for g.
 * Errors: GCADA_EINVAL (g, rows < 1, ld < widths[0], NULL).
 */
int gcada_set_shard(gcada_ctx* ctx, int32_t g, const void* X /*[device]*/,
                    const void* y /*[device]*/, int64_t rows, int64_t ld);

/*
 * Start a run (Algorithm 1's initialisation): theta^0 <- theta0 (copied), h = vhat = agg = 0,
 * stored gradients 0, every stale iterate = theta^0, every age tau_g = D (so step 0 selects all
 * groups), empty history, k = 0.  theta0: p floats, [host] or [device].  Synchronous.
 */
int gcada_set_theta(gcada_ctx* ctx, const float* theta0);

/*
 * One iteration k for all groups (steps a1-a4 above).
 *   idx:      [device] G*mu int32 row ids, idx[g*mu + i] in [0, rows_g): group g's minibatch
 *             xi_g^k; or NULL for the cyclic window rows (k*mu + i) mod rows_g.  Borrowed until
 *             the step has run.  Ids are not range-checked on the device.
 *   mask_out: [device] or pinned-host, G bytes: 1 if group g was selected; may be NULL.
 *   loss_out: [device] or pinned-host, 1 float: mean over all G*mu samples of the per-sample
 *             loss at theta^k (including (l2/2)||theta^k||^2); may be NULL.
 *   stream:   a hipStream_t (NULL = default stream).
 * Asynchronous; outputs are written in stream order.  Calls no allocator.
 * Errors: GCADA_ESTATE (a shard or theta missing; or a launch of an earlier step failed part-way),
 * GCADA_EDEVICE (launch failure; or a wait between workgroups inside a kernel of an EARLIER step
 * gave up -- some kernels let their workgroups hand results to each other and bound that wait, so a
 * device held by another stream cannot hang them.  The kernels report it to a pinned host word
 * which this call reads first, without touching the device: it sees the failures of the steps
 * that have finished on the device by then, at the latest after the caller has synchronised).
 * After either of the two the state is not valid and every further step fails until
 * gcada_set_theta or gcada_set_state has replaced it.
 */
int gcada_step(gcada_ctx* ctx, const int32_t* idx, uint8_t* mask_out, float* loss_out,
               void* stream);

/*
 * Views of the device state, valid until the next gcada_step / set_* / destroy.  Asynchronous:
 * the buffers hold the result of the last step once the stream that step was given has reached
 * it.  (After a step of the whole-row logistic path with GCADA_OPT_FUSED_FINISH the newest entry
 * of dtheta_sq is still spread over the kernel's blocks; this call then enqueues one small
 * kernel on THAT stream, which must still exist, to add it up.  gcada_get_state does the same
 * and waits.)
 */
typedef struct gcada_state_view {
    int64_t p;               /* number of parameters                                          */
    int32_t G, D, M_G;
    int64_t k;               /* iterations done (host mirror of the device counter)           */
    int64_t slot_stride;     /* floats between consecutive slots of theta_ring                */
    int64_t grad_stride;     /* floats between consecutive groups in grad and last (>= p)     */
    int32_t cur_slot;        /* theta^k is slot k mod (D+1); theta^{k-t} is slot (k-t) mod (D+1) */
    float*   theta_ring;     /* [device] (D+1) slots of p floats: the last D+1 iterates       */
    float*   h;              /* [device] p                                                    */
    float*   vhat;           /* [device] p                                                    */
    float*   agg;            /* [device] p: lazily aggregated gradient                        */
    float*   gbuf;           /* [device] two halves of G rows of grad_stride floats.  Row
                                (which[g]*G + g) holds the gradient group g uploaded last; a step
                                writes group g's fresh gradient to the other half's row g and an
                                upload flips which[g].  So after a step the fresh gradient of g is
                                row which[g] if mask[g], else the other half's row (that row is
                                unspecified under GCADA_OPT_LAZY_GRADIENT_STORE)                */
    int32_t* which;          /* [device] G, each 0 or 1                                        */
    int32_t* tau;            /* [device] G ages                                               */
    double*  dtheta_sq;      /* [device] D: ||theta^{j+1}-theta^j||^2 stored at index j mod D */
    double*  stat;           /* [device] G: stat_g of the last step                           */
    double*  rhs;            /* [device] 1: threshold of the last step                        */
    uint8_t* mask;           /* [device] G: selection of the last step                        */
    double*  loss;           /* [device] 1: loss of the last step                             */
} gcada_state_view;

int gcada_state(gcada_ctx* ctx, gcada_state_view* out /*[host]*/);

/* Whole state in caller-owned HOST buffers, for checkpoints and step-by-step comparison. */
typedef struct gcada_state_host {
    float*   theta;        /* p                                   */
    float*   h;            /* p                                   */
    float*   vhat;         /* p                                   */
    float*   agg;          /* p                                   */
    float*   theta_stale;  /* G x p: theta^{k - tau_g} per group  */
    float*   last;         /* G x p                               */
    int32_t* tau;          /* G, each in [1, D]                   */
    double*  dtheta_sq;    /* D, index j mod D as above           */
    int64_t  k;
} gcada_state_host;

/* Copy the state out (fills the buffers and k).  Synchronises the device.  GCADA_EDEVICE when a
 * wait inside a kernel of one of the steps so far gave up (see gcada_step). */
int gcada_get_state(gcada_ctx* ctx, gcada_state_host* out /*[host]*/);

/*
 * Overwrite the state.  Groups with equal tau must carry equal theta_stale rows (they are one
 * iterate of the history); the row of the lowest such g is used.  Errors: GCADA_EINVAL when a
 * tau is outside [1, D] or k < 0.  Synchronises the device.
 */
int gcada_set_state(gcada_ctx* ctx, const gcada_state_host* in /*[host]*/);

/*
 * Host-only cost model of Sec. II-B / Sec. V for one iteration of G groups of M_G workers with
 * minibatch size mu, from the selection mask and seeded per-worker compute times T
 * (G x M_G doubles, [host], e.g. iid Exp(eta)):
 *   time  = max over selected groups of the min over the group's workers (the server waits
 *           for the fastest worker of each selected group; 0 if nothing is selected),
 *   comm  = |selected| * (M_G + 1)   (downloads + uploads, Eq. (5), (19)),
 *   comp  = |selected| * M_G * mu    (Eq. (6), (22)).
 * Any of the three outputs may be NULL (T may be NULL when time is).  Touches no device.
 * Errors: GCADA_EINVAL (G, M_G, mu < 1, NULL mask, time without T).
 */
int gcada_cost_model(int32_t G, int32_t M_G, int32_t mu, const uint8_t* mask /*[host] G*/,
                     const double* T /*[host] G*M_G*/, double* time, int64_t* comm,
                     int64_t* comp);

/*
 * Tuning switches (defaults in brackets).  GCADA_OPT_SINGLE_PASS_LOGREG [1]: compute the logistic
 * gradients with the kernel that reads the minibatch from HBM once (whole-row register tiles)
 * when the shape allows it (d <= 256 with mu <= 128 and few groups: the whole iteration in one
 * launch; otherwise d <= 4096, a multiple of 4, any mu: whole-row register tiles of 16 times
 * 16 / (d / 256 rounded up to a power of two) rows, the last tile of a group possibly partly
 * empty; or 4096 < d <= 65,536, a multiple of 4, with mu >= 5: 4-row tiles shared by a team of
 * ceil(d / 4096) workgroups; 16-byte aligned shards); 0 forces the general two-pass kernels.
 * All compute the same step a1.
 * GCADA_OPT_FUSED_FINISH [1]: after the whole-row tile kernel, add the tile partials, select
 * (Eq. (9)), sum the innovations and update (Eq. (8a)-(8c)) in ONE launch whose blocks meet once
 * inside the kernel (at most 64 blocks, one per compute unit; the wait is bounded: if the blocks
 * cannot all run at once -- another stream holding the device -- the step is reported as failed,
 * GCADA_EDEVICE from a later gcada_step, gcada_state or gcada_get_state, instead of hanging);
 * 0 uses the separate reduce and server kernels.  Same arithmetic per element either way.
 * GCADA_OPT_LAZY_GRADIENT_STORE [1 for an MLP whose G fresh gradients are 64 MiB or more, else 0;
 * ignored for the linear models]: with the gradient-difference rule every group evaluates both
 * gradients in every step, but only an uploading group's fresh gradient is ever read again (the
 * innovation of Eq. (8a)'s aggregate).  With 1, the weight-gradient kernels write the fresh
 * gradient only for the groups that are selected whatever the statistic says (age D reached, or
 * an empty history), and after the selection one more launch writes it for the other selected
 * groups, recomputed from the signals and activations still in place (same products in the same
 * order: the same bits).  Iterates, aggregate, stored gradients, statistic and mask are
 * identical either way; the `gbuf` row of a group that did NOT upload is then unspecified.
 * GCADA_OPT_GRAM_STATISTIC [1; takes effect for a bf16 MLP under the lazy gradient store when
 * mu (n_0 + n_1) <= n_0 n_1 and the first forward GEMM reads the shard rows in place]: both
 * iterates see the same minibatch X, so the first layer's share of stat_g is
 * || (dZ_1 - dZ~_1)^T X ||^2 = <X X^T, (dZ_1 - dZ~_1)(dZ_1 - dZ~_1)^T>: two mu x mu Gram matrices
 * instead of two n_1 x n_0 weight gradients, and the first layer's gradient is formed only for
 * the groups that upload.  Same statistic up to rounding (the signal difference is rounded to
 * bf16 once more); 0 computes it from the two weight gradients.
 * GCADA_OPT_DEFERRED_FINISH [0]: whole-row logistic path (d <= 4096) when all tiles of a step fit the
 * device at once (G * ceil(mu / tile rows) workgroups, at most one per compute unit, at least d / 64):
 * ONE launch per step.  The rows a step reads depend on its row ids only, not on the iterate, so the
 * finish of step k (reduce, selection, innovation sum, update) runs at the head of the launch of
 * step k+1, while all workgroups wait for their rows; the new iterate reaches the tiles through
 * tagged words inside the launch.  Consequence for the caller: mask_out and loss_out of the call
 * for step k are written by the NEXT gcada_step (or by gcada_state / gcada_get_state /
 * gcada_set_option (any option but GCADA_OPT_EXPIRE_NEXT_WAIT) / gcada_set_rule /
 * gcada_time_gradient_stage, which run a finish that is still to come; gcada_set_theta / gcada_set_state discard it) and stay borrowed until then; gcada_state's
 * k counts the steps issued.  Same arithmetic: the state is bit-identical to the two-launch path.
 * GCADA_OPT_EXPIRE_NEXT_WAIT [0]: a diagnostic for tests of the error path.  With 1, the kernels of
 * the NEXT gcada_step that wait for other workgroups' words look for words nobody publishes and
 * give up after a few polls: every kernel runs to its end, the step's results are invalid, and the
 * failure is reported as described under gcada_step.  Cleared by that step.
 * Errors: GCADA_EINVAL (unknown option).
 */
enum { GCADA_OPT_SINGLE_PASS_LOGREG = 1, GCADA_OPT_FUSED_FINISH = 2, GCADA_OPT_LAZY_GRADIENT_STORE = 3,
       GCADA_OPT_GRAM_STATISTIC = 4, GCADA_OPT_EXPIRE_NEXT_WAIT = 5,
       GCADA_OPT_DEFERRED_FINISH = 6 };
int gcada_set_option(gcada_ctx* ctx, int32_t option, int32_t value);

/*
 * One iteration with per-worker minibatches (Sec. IV, Algorithm 1 taken literally): every worker
 * m of group g draws its own minibatch xi_m^k, and the gradient the server receives from a
 * selected group is that of the group's FASTEST worker, xi_g^k := xi_m^k with m = argmin_m T_m^k
 * (ties: the lowest m).  Everything else is gcada_step on the minibatches so chosen.
 *   idx_workers: [device] G*M_G*mu int32 row ids, idx_workers[(g*M_G + m)*mu + i].
 *   delays:      [device] G*M_G doubles, the compute times T_m^k of this iteration (Sec. II-B).
 *   worker_out:  [device] G int32: the worker whose minibatch was used; may be NULL.
 * Asynchronous, no allocator.  Errors as gcada_step, and GCADA_EINVAL for NULL idx_workers/delays.
 */
int gcada_step_workers(gcada_ctx* ctx, const int32_t* idx_workers, const double* delays,
                       int32_t* worker_out, uint8_t* mask_out, float* loss_out, void* stream);

/*
 * Selection rule.  GCADA_RULE_GRADIENT_DIFFERENCE [default]: group g is selected when the squared
 * norm of the difference of its two same-minibatch gradients (at theta^k and at its stale
 * iterate) exceeds the threshold -- the quantity the paper's condition estimates (Sec. III, IV).
 * GCADA_RULE_SERVER: the condition as the paper states it for the parameter server (Sec. IV):
 * selected when L_g^2 ||theta^k - theta^{k - tau_g}||^2 > (c/D) sum_{d<=D} ||theta^{k+1-d} -
 * theta^{k-d}||^2, or when the age tau_g has reached D, or when the threshold is 0.  The decision
 * then precedes the gradient stage and only the selected groups evaluate a gradient, once, at
 * theta^k (Algorithm 1); the returned loss is the mean over the evaluated samples (0 when no
 * group is selected), and gcada_state's stat holds the left sides.
 * L [host, G doubles, copied]: the smoothness constants L_g, an input of Algorithm 1; may be
 * NULL when they were given before.  May be called between steps.
 * Errors: GCADA_EINVAL (unknown rule, negative or non-finite L_g, GCADA_RULE_SERVER without L, or
 * GCADA_RULE_SERVER on a context with D > 64).
 */
enum { GCADA_RULE_GRADIENT_DIFFERENCE = 0, GCADA_RULE_SERVER = 1 };
int gcada_set_rule(gcada_ctx* ctx, int32_t rule, const double* L);

/*
 * Smoothness constants of the groups' local functions (Sec. IV: the average loss over the
 * group's shard) for the linear models: L_g = kappa * lambda_max(X_g^T X_g) / rows_g + lambda,
 * kappa = 1/4 (logistic) or 1 (quadratic error), the eigenvalue by `iters` steps of power
 * iteration on the shard (two passes over the shard per step; synchronises `stream`).
 * L_out [host, G doubles].  Errors: GCADA_EINVAL (MLP, NULL, iters < 1), GCADA_ESTATE (a shard
 * is missing), GCADA_EDEVICE.
 */
int gcada_estimate_smoothness(gcada_ctx* ctx, int32_t iters, double* L_out, void* stream);

/*
 * gcada_estimate_smoothness for callers that cannot allocate device memory -- code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels and arithmetic, but
 *   - the scratch of the power iteration (two d-vectors, one value per shard row, up to 256 x d
 *     partial sums) lives in a static device array of the library, 2 Mi doubles = 16 MiB, which
 *     every GPU the library runs on holds until the process ends; a shard that needs more is
 *     refused with GCADA_EINVAL (lr-type shapes up to about d = 4096 with 65,536 rows fit);
 *   - L_out is [device] (or pinned host), G doubles, written in stream order; nothing is copied to
 *     or from pageable host memory, and the call does not synchronise;
 *   - it calls no hipMalloc / hipFree nor any allocating library routine.
 * All calls on one GPU share that GPU's array (whatever the context): two calls that overlap in
 * time on one GPU race, so order them on one stream or with events.  The array keeps the last
 * call's contents; nothing in it has to start at zero (every word read was written by this call).
 * Errors: as gcada_estimate_smoothness, plus GCADA_EINVAL when a shard exceeds the array.
 */
int gcada_estimate_smoothness_static(gcada_ctx* ctx, int32_t iters, double* L_out /*[device]*/, void* stream);

/*
 * Diagnostics for benchmarks: run only the dominant kernel(s) of step a1 -- the kernels that
 * read the minibatch; gcada_timed_stage names them -- `reps` times back to back on `stream`
 * between two HIP events; repetition r uses the minibatch idx + r*idx_stride (G*mu ids each, as in
 * gcada_step; give distinct minibatches, or the rows are served from cache after the first
 * repetition; idx may be NULL for the cyclic window).  These kernels write only
 * scratch and the fresh-gradient rows, so the run's state (theta, moments, aggregate, stored
 * gradients, ages, history, k) is unchanged.  Synchronises the stream; returns the mean
 * duration per repetition in milliseconds.  Creates and destroys two events (not for use
 * under graph capture).  Errors: GCADA_EINVAL (reps < 1), GCADA_ESTATE, GCADA_EDEVICE.
 */
int gcada_time_gradient_stage(gcada_ctx* ctx, const int32_t* idx, int64_t idx_stride, int32_t reps,
                              void* stream, double* ms_per_rep /*[host]*/);

/*
 * Name of what gcada_time_gradient_stage times for this context and its current shards, e.g.
 * "lr_tile_kernel" (the single kernel that reads the minibatch), "lr_forward+lr_backward",
 * "mlp gradient stage".  Returns a pointer valid until the next call on this context.
 */
const char* gcada_timed_stage(gcada_ctx* ctx);

/*
 * Diagnostic for benchmarks, next to the roofline of the HBM-bound kernels of step a1: the rate, in
 * GB/s (1e9 bytes per second), at which this device reads `bytes` of contiguous device memory
 * [device, 16-byte aligned, at least 64 MiB; use far more than the 256 MB of last-level cache] with
 * a plain streaming kernel -- the best of a fixed set of launch shapes (1 to 16 workgroups per
 * compute unit, 256 to 1024 threads, 8 or 16 loads of 16 bytes in flight per thread, ordinary or
 * non-temporal loads), `reps` launches each between two HIP events.  gbps_plain_loads (may be
 * NULL): the best of the shapes with ordinary loads alone.  Needs no context.  Synchronises the
 * stream; allocates one word and two events.  Errors: GCADA_EINVAL, GCADA_EDEVICE (message under
 * the NULL context).
 */
int gcada_hbm_read_calibration(const void* buf /*[device]*/, int64_t bytes, int32_t reps, void* stream,
                               double* gbps /*[host]*/, double* gbps_plain_loads /*[host]*/);

/*
 * Benchmark diagnostic beside the measurement of step a1 (Sec. II-A: one read of every group's
 * minibatch rows) for wide linear models: GB/s of a kernel that reads the rows idx selects from the
 * context's shards in the access pattern of the wide-row gradient kernel (rows cut into pieces of
 * 4096 columns that go to the members of a team of workgroups, four rows per tile, three tiles in
 * flight, one workgroup barrier per tile) and does nothing else -- what that access pattern allows
 * on this machine.  idx [device]: reps + 1 minibatches of G * batch row ids each, idx_stride ids
 * apart (launch r reads minibatch r; minibatch 0 is read once more as a warm-up).  Requires a
 * linear fp32 model with 8192 <= width <= 65,536, a multiple of 4096; batch a multiple of 4; every
 * shard set, rows 16-byte aligned.  Synchronises the stream; allocates one word and two events.
 * Errors: GCADA_EINVAL, GCADA_ESTATE, GCADA_EDEVICE.
 */
int gcada_gather_read_calibration(gcada_ctx* ctx, const int32_t* idx /*[device]*/, int64_t idx_stride, int32_t reps,
                                  void* stream, double* gbps /*[host]*/);

/* Message of the last error on this context ("" if none); NULL ctx: last gcada_create error. */
const char* gcada_last_error(const gcada_ctx* ctx);

/* Library version string. */
const char* gcada_version(void);

#ifdef __cplusplus
}
#endif
#endif /* GCADA_H */
