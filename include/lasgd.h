/*
 * lasgd.h -- C ABI of the LASGD update library for MI355X (gfx950).
 *
 * LASGD (Locally Asynchronous SGD): every worker keeps taking local SGD steps
 * while an All-Reduce of the models it and its peers "sent" is in flight, and
 * when the mean z_t arrives replaces its model by z_t plus the progress it
 * made meanwhile (Algorithm 1, Sec. 4).  This library holds K workers
 * ("replicas", the paper's P nodes) on ONE GPU and implements the per-iteration
 * arithmetic of that algorithm; the All-Reduce becomes a reduction over the K
 * sent models in device memory, run on a second stream.
 *
 * Conventions
 *   - One opaque context owns all K replicas.  Every operation is an
 *     asynchronous enqueue on a stream borrowed from the caller; nothing
 *     blocks the host except lasgd_read_state, lasgd_sync and lasgd_destroy.
 *   - All pointers named "device" are HIP device pointers; all others are
 *     host pointers.  Config and pointer arrays are copied during the call.
 *   - Errors are return codes; nothing throws or aborts.  Every argument and
 *     call-order check precedes the first stream operation, so a call refused
 *     with INVALID, STATE or UNSUPPORTED enqueues nothing and leaves the context
 *     unchanged.  A HIP failure in the middle of a call (LASGD_ERR_HIP) can leave
 *     a stream dependency or a kernel enqueued; the context's call-order state
 *     then reflects what was enqueued.  The text of the last failure is
 *     available from lasgd_last_error.
 *   - Calls on one context must come from one host thread at a time, with the
 *     device the context was created on current.
 *
 * Memory owned by the caller:  parameters x[k][t] and gradients g[k][t]
 *   (one device buffer per replica k and tensor t, numel[t] elements, 16-byte
 *   aligned, fp32 or bf16 according to `storage`), and both streams.
 * Memory owned by the library:  momentum v[k], sent models s[k], the mean z,
 *   the fp32 master copy of the parameters when storage is bf16, and the
 *   descriptor tables.
 *
 * Paper <-> calls.  Prologue (steps 1-5): lasgd_local_step(eta_0),
 *   lasgd_snapshot, lasgd_average.  Loop iteration without global update
 *   (steps 6-8): lasgd_local_step(eta).  With global update (steps 6-9):
 *   lasgd_step_merge(eta, 1) then lasgd_average -- or, unfused,
 *   lasgd_local_step, lasgd_merge(1), lasgd_average -- or, everything in one
 *   pass, lasgd_step_merge_average(eta).  The clocks t, t^i and tau_i are the
 *   caller's; the library only enforces a legal order.
 */
#ifndef LASGD_H
#define LASGD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lasgd_ctx lasgd_ctx;

typedef enum {
    LASGD_OK = 0,
    LASGD_ERR_INVALID = 1,     /* bad argument: NULL, K < 1, numel < 1, misaligned or
                                  NULL device pointer, non-finite lr, bad index        */
    LASGD_ERR_STATE = 2,       /* legal arguments, illegal order (see each call)      */
    LASGD_ERR_ALLOC = 3,       /* device or host allocation failed                    */
    LASGD_ERR_HIP = 4,         /* any other HIP runtime failure                       */
    LASGD_ERR_UNSUPPORTED = 5  /* size beyond what the kernels index (see create)     */
} lasgd_status;

typedef enum { LASGD_F32 = 0, LASGD_BF16 = 1 } lasgd_dtype;

/* Which array lasgd_read_state copies out. */
typedef enum {
    LASGD_STATE_X = 0,   /* local model x^i as fp32 (the master copy when storage is bf16) */
    LASGD_STATE_V = 1,   /* momentum buffer                                               */
    LASGD_STATE_S = 2,   /* model last sent to the All-Reduce, x^i_t                      */
    LASGD_STATE_Z = 3    /* All-Reduce result z_t (replica index ignored)                 */
} lasgd_state;

typedef struct {
    int32_t K;                    /* replicas resident on this GPU (the paper's P, Sec. 3); 1..64 */
    int32_t n_tensors;            /* entries in the parameter list; >= 1                          */
    const int64_t *numel;         /* host [n_tensors], each >= 1                                  */
    lasgd_dtype storage;          /* dtype of the caller's parameters and gradients               */
    float momentum;               /* mu >= 0 (Sec. 5.2: Nesterov momentum); 0 = plain SGD of Alg. 1 */
    int32_t nesterov;             /* 1: look-ahead form, 0: heavy ball                            */
    const float *weight_decay;    /* host [n_tensors] L2 coefficients, or NULL => wd_scalar everywhere */
    float wd_scalar;
    void *main_stream;            /* hipStream_t for local steps, snapshot, merge (NULL = default stream) */
    void *side_stream;            /* hipStream_t the mean is computed on; may equal main_stream   */
} lasgd_config;

/* Launch-shape knobs; results never depend on them.  Zero in any field keeps
 * the built-in default for that field. */
typedef struct {
    int32_t vec;           /* 128-bit vectors per lane per tile: 1, 2 or 4 (tile = 256*vec elements) */
    int32_t kper_step;     /* replicas one wave handles back to back in local_step (1..K)            */
    int32_t kper_merge;    /* same for merge / step_merge; K keeps each z tile in registers          */
    int32_t max_blocks;    /* cap on workgroups per launch (grid-stride beyond it); <0 = no cap      */
    int32_t avg_split;     /* waves of a workgroup that share one tile's K replicas in average (1,2,4) */
    int32_t avg_max_blocks;/* cap on workgroups of the average kernel; <0 = no cap                   */
    int32_t nontemporal;   /* 1: streaming hint on loads, 2: on stores, 3: both, 4: none             */
    int32_t chunk_step;    /* work-item order of local_step / snapshot: tiles are taken in chunks of this
                              many; inside a chunk replica after replica.  1 = the replicas of a tile are
                              adjacent; <0 = whole replica after whole replica                       */
    int32_t chunk_merge;   /* same for merge / step_merge (a chunk's z tiles are reused K times within
                              a short window; multiples of 32 keep a tile on one XCD's L2)           */
    int32_t waves_per_block; /* independent waves per workgroup in the multi-tensor kernels: 1, 2 or 4  */
    int32_t race_probe;    /* debugging aid, 1 = on, <0 = off (default): lasgd_average first fills z with NaN
                              on the side stream, so a global update that did not wait for the mean shows
                              as NaN in the parameters.  Results are unchanged when the ordering holds.  */
    int32_t group_r;       /* replicas one wave takes at a time in the one-workgroup-per-tile kernels
                              (lasgd_step_merge_average, lasgd_sgd_ar_step): 1, 2 or 4; the workgroup has
                              ceil(K / group_r) waves, at most 16.  <0 = default (chosen from K)            */
} lasgd_tuning;

/*
 * Create a context for K replicas of a parameter list and allocate the
 * library-owned state (v = 0, s, z, master copy), on the current device.
 * Errors: INVALID (NULL, K outside 1..64, n_tensors < 1, numel < 1, negative or
 * non-finite momentum / weight decay, unknown storage), UNSUPPORTED (a padded
 * replica larger than 2^31 - 2^20 elements), ALLOC, HIP.  *out is NULL on failure.
 */
lasgd_status lasgd_create(const lasgd_config *cfg, lasgd_ctx **out);

/*
 * Attach replica k's buffers: params[t] and grads[t] are device pointers to
 * numel[t] elements of the storage dtype, 16-byte aligned; the host arrays
 * [n_tensors] are copied, the device buffers stay the caller's and must
 * outlive their use.  May be called again to re-point a replica (e.g. at a
 * rotating gradient buffer); waits for work already enqueued.  16-byte
 * alignment is all that is required; for full speed let every tensor start on
 * a 1 KiB boundary (512 bytes for bf16), the size of one wave's access: the
 * library's own arrays are laid out that way, and tiles that start 256 or 512
 * bytes off such a boundary stream 3-5 % slower on MI355X.
 * Errors: INVALID (NULL, k out of range, NULL or misaligned entry), HIP.
 */
lasgd_status lasgd_bind(lasgd_ctx *ctx, int32_t k, void *const *params, void *const *grads);

/*
 * bf16 storage only: master <- exact widening of the bound parameters,
 * v <- 0 (Algorithm 1 step 1).  Required once before the first step.
 * Errors: STATE (storage is fp32; a replica is unbound), HIP.
 */
lasgd_status lasgd_init_master(lasgd_ctx *ctx);

/*
 * Local update of all K replicas (Algorithm 1 steps 3 and 7, with the optimizer
 * of Sec. 5.2):  g' = g + wd*x;  v = mu*v + g';  d = g' + mu*v (Nesterov) or v;
 * x = x - lr*d.  Reads g, x, v; writes x, v (bf16 storage: acts on the master
 * and also rewrites the bf16 parameters).  Main stream.
 * Errors: INVALID (non-finite lr), STATE (a replica is unbound; bf16 master not
 * initialised), HIP.
 */
lasgd_status lasgd_local_step(lasgd_ctx *ctx, float lr);

/*
 * The send of Algorithm 1 (steps 4 and 9c): the model handed to the All-Reduce is
 * kept, s[k] <- x[k].  Main stream.
 * Errors: STATE (an average is in flight and not yet merged: the side stream
 * may still be reading s), HIP.
 */
lasgd_status lasgd_snapshot(lasgd_ctx *ctx);

/*
 * The All-Reduce itself (Sec. 3, Eq. 8): z = (1/K) sum_k s[k], accumulated in
 * fp64 and rounded once.  Runs on the side stream after everything enqueued so
 * far on the main stream; the main stream does not wait for it.
 * Errors: STATE (no snapshot since the last merge that did not re-snapshot;
 * a previous average is still unmerged), HIP.
 */
lasgd_status lasgd_average(lasgd_ctx *ctx);

/*
 * The test of Algorithm 1 step 9 (has the All-Reduce ended?): *done = 1 if the
 * last average has finished on the device, else 0.  Never blocks.
 * Errors: INVALID (NULL), STATE (no average launched; or the last average was
 * issued while its stream was being captured into a graph -- a recorded mean
 * runs whenever the graph is replayed and cannot be polled through this call), HIP.
 */
lasgd_status lasgd_average_done(lasgd_ctx *ctx, int32_t *done);

/*
 * Global update (Algorithm 1 step 9a-b): x[k] <- z + (x[k] - s[k]); with
 * resnapshot != 0 also s[k] <- x[k] (step 9c).  The main stream first waits for
 * the pending average.
 * Errors: STATE (no average launched since the last merge), HIP.
 */
lasgd_status lasgd_merge(lasgd_ctx *ctx, int32_t resnapshot);

/*
 * Steps 7 and 9a-c of one loop iteration in a single pass over memory:
 * exactly lasgd_local_step(lr) followed by lasgd_merge(resnapshot), with the
 * same roundings.
 * Errors: as lasgd_local_step and lasgd_merge.
 */
lasgd_status lasgd_step_merge(lasgd_ctx *ctx, float lr, int32_t resnapshot);

/*
 * One loop iteration with global update AND the next All-Reduce in a single pass
 * (Algorithm 1 steps 7 and 9a-c, then Sec. 3 Eq. 8 on the models just re-sent):
 * exactly lasgd_step_merge(lr, 1) followed by lasgd_average, same roundings, but
 * the K replicas of each tile meet in on-chip memory, so the sent models are not
 * read back for the mean.  Everything runs on the main stream (after the pending
 * average), nothing on the side stream; afterwards the new mean counts as
 * launched, exactly as after lasgd_average.  Meant for cadences with nothing to
 * overlap the All-Reduce with (a global update every step, tau_max = 1 in Sec. 5.2).
 * Errors: as lasgd_step_merge, plus STATE when the pending average is partial or
 * partly merged, or elastic coefficients other than 1 are set.
 */
lasgd_status lasgd_step_merge_average(lasgd_ctx *ctx, float lr);

/* ---- extended calls: replicas at their own pace, partial All-Reduce, elastic
 *      coefficients, the SGD All-Reduce comparator ----------------------------
 *
 * In Algorithm 1 every node runs its own loop: it takes between 1 and tau_max
 * local steps per All-Reduce, with a step size indexed by its own clock, and
 * each node takes its global update whenever it notices the result, independently
 * of the others (Sec. 4).  With K nodes batched
 * on one GPU this becomes a bit mask per call (bit k = replica k takes part)
 * and a step size per replica.  The same masks express the partial All-Reduce
 * the paper proposes as future work (Sec. 6): the mean is taken over the
 * participants only and divided by their number; a replica that sits a round
 * out neither sends nor merges in it.  Order rules, per replica: it must have
 * sent (snapshot, or merge with resnapshot) before it is averaged; it may not
 * be snapshotted while a mean it takes part in is unmerged; a new mean cannot
 * start before every participant of the previous one has merged (one z buffer).
 * Each plain call above equals its _ex form with all K bits set and equal step sizes.
 */

/* Local update of the replicas in `mask` (may be empty); lr: host [K], entry k
 * read only if bit k is set.  Errors: as lasgd_local_step, plus INVALID for a
 * NULL array, a bit beyond K or a non-finite entry. */
lasgd_status lasgd_local_step_ex(lasgd_ctx *ctx, const float *lr, uint64_t mask);

/* s[k] <- x[k] for the replicas in `mask` (non-empty).
 * Errors: as lasgd_snapshot (STATE only if the pending mean involves one of them). */
lasgd_status lasgd_snapshot_ex(lasgd_ctx *ctx, uint64_t mask);

/* z <- mean over the replicas in `mask` (non-empty) of s[k]; with beta != 1
 * (lasgd_set_elastic) blended into the previous centre.  Side stream.
 * Errors: as lasgd_average, per participant. */
lasgd_status lasgd_average_ex(lasgd_ctx *ctx, uint64_t mask);

/* Global update of the replicas in `mask` (non-empty subset of the pending
 * mean's participants that have not merged yet). */
lasgd_status lasgd_merge_ex(lasgd_ctx *ctx, uint64_t mask, int32_t resnapshot);

/* One pass in which the replicas in step_mask take a local update (lr: host [K])
 * and those in merge_mask (non-empty) then take the global update; a replica may
 * be in either, both or neither. */
lasgd_status lasgd_step_merge_ex(lasgd_ctx *ctx, const float *lr, uint64_t step_mask,
                                 uint64_t merge_mask, int32_t resnapshot);

/*
 * Elastic coefficients of Sec. 3 (Eq. 5-6; alpha = eta*rho, beta = P*gamma) for
 * all later calls: the mean becomes z <- (1-beta) z + beta mean_k s[k] (the first
 * mean after create initialises z), the global update x <- x + alpha (z - s).
 * alpha = beta = 1 (the default) is Algorithm 1 exactly.
 * Errors: INVALID (a value outside [0, 1] or not a number).
 */
lasgd_status lasgd_set_elastic(lasgd_ctx *ctx, float alpha, float beta);

/*
 * The SGD All-Reduce comparator (Sec. 2; "SGD-AR" in Table 1): average the K
 * gradients (fp64 accumulate, one rounding) and let every replica take the local
 * update with the mean gradient, in one pass.  Main stream; touches x, v only.
 * Errors: as lasgd_local_step.
 */
lasgd_status lasgd_sgd_ar_step(lasgd_ctx *ctx, float lr);

/*
 * Parity probe: wait for both streams, then copy one array to host memory as
 * fp32.  tensor >= 0: that tensor of replica k, n must equal numel[tensor];
 * tensor == -1: all tensors of replica k back to back (no padding), n must
 * equal the sum of numel.  k is ignored for LASGD_STATE_Z.
 * Errors: INVALID (NULL, bad which / k / tensor / n), STATE (X of an unbound
 * replica), HIP.
 */
lasgd_status lasgd_read_state(lasgd_ctx *ctx, int32_t which, int32_t k, int32_t tensor,
                              float *host_dst, int64_t n);

/*
 * For callers that cannot allocate device memory (code under stream capture,
 * tight serving loops, harnesses that forbid hipMalloc): the All-Reduce and the
 * global update of lasgd_average + lasgd_merge in one context-free call on flat
 * fp32 vectors, with no allocation of any kind on the device.
 *     z = (1/K) sum_k sent[k]   (fp64 accumulation in replica order, one rounding)
 *     x[k] <- z + (x[k] - sent[k]);  resnapshot != 0: sent[k] <- x[k]
 * Same roundings as the context calls.  x, sent: host arrays [K] of device
 * pointers to n fp32 elements each, 16-byte aligned, no two overlapping; they are the
 * caller's, are read during the call (the arrays) and updated in place on the
 * device (the buffers).  stream: hipStream_t (NULL = default stream); both
 * kernels are enqueued on it, the call does not wait for them.  z is kept in a
 * device array built into the library, LASGD_STATIC_MAX_N elements (128 MiB)
 * per GPU for the life of the process; it is fully rewritten for [0, n) by every
 * call, so nothing needs clearing, and its contents are not an output.  All calls
 * on one GPU share that array: two calls whose kernels may overlap on the device
 * (different streams, no ordering) race.  Error text: lasgd_last_error(NULL).
 * Errors: INVALID (NULL, K outside 1..64, n < 1, NULL / misaligned / overlapping
 * buffer), UNSUPPORTED (n > LASGD_STATIC_MAX_N), HIP.  A failed call leaves the caller's
 * buffers untouched.
 */
#define LASGD_STATIC_MAX_N (32ll << 20)
lasgd_status lasgd_global_update_static(int32_t K, int64_t n, float *const *x, float *const *sent,
                                        int32_t resnapshot, void *stream);

/* Wait until both streams have finished everything this context enqueued. */
lasgd_status lasgd_sync(lasgd_ctx *ctx);

/* Change launch-shape knobs (waits for enqueued work first).  A graph captured
 * earlier keeps the shape it was recorded with and stays valid (the tile table
 * of every tile size used is kept until lasgd_destroy).
 * Errors: INVALID (NULL, a field outside its documented values), HIP, ALLOC. */
lasgd_status lasgd_set_tuning(lasgd_ctx *ctx, const lasgd_tuning *t);

/* The knobs currently in effect. */
lasgd_status lasgd_get_tuning(const lasgd_ctx *ctx, lasgd_tuning *out);

/* Text of the last failure on this context ("" if none); owned by the context.
 * With ctx == NULL: text of the last failure of a context-free call (lasgd_create,
 * lasgd_global_update_static) on this thread. */
const char *lasgd_last_error(const lasgd_ctx *ctx);

/* Wait for enqueued work, free library-owned memory.  NULL is allowed. */
void lasgd_destroy(lasgd_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* LASGD_H */
