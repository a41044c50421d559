/*
 * nups.h - C ABI of the MI355X-native minibatch step of sparse-parameter SGD for the
 * workloads of "NuPS: A Parameter Server for Machine Learning with Non-Uniform
 * Parameter Access" (SIGMOD '22): draw negative keys, pull rows, compute the
 * per-example gradients, aggregate per key and push the updates back.
 *
 * Conventions (all entry points):
 *  - Every call returns a nups_status; nothing throws across the boundary.
 *    nups_last_error() gives a thread-local description of the last failure.
 *  - "dev" pointers are device (HBM) addresses, "host" pointers are host addresses.
 *  - The library never owns table, state, batch or output memory: the caller
 *    allocates it and keeps it alive while the context uses it.  The library owns
 *    only its workspace and the opaque objects it hands out.
 *  - All device work is enqueued on the HIP stream given to nups_init; the library creates
 *    no stream, event or thread.  Preparatory work that only handles keys (drawing samples,
 *    building the per-key aggregation structure of a step; the "background" work of Section
 *    4.3) does not get launches of its own when steps are prepared ahead: it rides in spare
 *    workgroups of the gradient and update launches of the steps that run before (see
 *    nups_prepare_step).  Calls return without waiting unless they hand a value back to the
 *    host (stated per call).
 *  - A table is a dense [num_keys, row_stride] fp32 array; the first `dim` floats of
 *    a row are the parameter, the rest is padding that stays zero.  row_stride must be
 *    64, 128, 192, 256, 320, 384, 512 or 1024 floats (the row widths that kernels are
 *    built for; pad narrower rows up to the next of them); keys are uint32 row numbers.
 *    nups_step works on tables 0 and 1, which must have the same row_stride; for
 *    NUPS_TASK_KGE (complex rows: real parts from float 0, imaginary parts from float
 *    row_stride / 2) it must be 128, 256, 384 or 512.
 *  - Keys outside [0, num_keys) never cause an out-of-range access: the kernels skip
 *    or clamp them, raise a device-side flag, and the next call that synchronises
 *    (nups_step with a loss pointer, nups_debug_structure, nups_check) returns
 *    NUPS_ERR_KEY_RANGE.
 */
#ifndef NUPS_H
#define NUPS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct nups_ctx nups_ctx;        /* tables + workspace + stream      */
typedef struct nups_dist nups_dist;      /* a registered target distribution */
typedef struct nups_sample nups_sample;  /* handle returned by PrepareSample */
typedef struct nups_prepared nups_prepared; /* a step whose preparatory work has been enqueued */

typedef enum {
    NUPS_OK = 0,
    NUPS_ERR_ARG = -1,           /* null pointer, negative size, inconsistent shapes        */
    NUPS_ERR_KEY_RANGE = -2,     /* a key was >= num_keys                                   */
    NUPS_ERR_OVERPULL = -3,      /* PullSample asked for more than the handle still holds   */
    NUPS_ERR_STATE = -4,         /* call not valid in the object's current state            */
    NUPS_ERR_DEVICE = -5,        /* a HIP call failed                                       */
    NUPS_ERR_UNIMPLEMENTED = -6
} nups_status;

/* Sampling schemes of Section 4.4, named by the conformity level they provide (Section 4.1). */
typedef enum {
    NUPS_CONFORM = 1,      /* independent sampling: i.i.d. draws, each used once           */
    NUPS_BOUNDED = 2,      /* sample reuse: pools of G draws, each traversed U times       */
    NUPS_LONGTERM = 3,     /* sample reuse over a long-lived pool of P draws, R passes     */
    NUPS_NONCONFORM = 4    /* local sampling / direct-access repurposing within the batch  */
} nups_scheme;

/* The three tasks of Section 5.1. */
typedef enum { NUPS_TASK_SGNS = 1, NUPS_TASK_MF = 2, NUPS_TASK_KGE = 3 } nups_task;

/* ---- context ----------------------------------------------------------------------- */

/*
 * Creates a context over n_tables (1..4) caller-owned tables (the key -> value-vector
 * store of Section 3.1).  tables_dev[t] is the device address of table t,
 * num_keys[t] x row_stride[t] floats.  hip_stream is a hipStream_t (NULL = the
 * default stream).  Errors: NUPS_ERR_ARG on null pointers, dim <= 0, dim > row_stride,
 * a row_stride that is not one of the supported widths, num_keys outside 1..2^32-1;
 * NUPS_ERR_DEVICE if no device is usable.
 */
nups_status nups_init(nups_ctx **out, int n_tables, float *const *tables_dev, const int64_t *num_keys,
                      const int32_t *dim, const int32_t *row_stride, void *hip_stream);

/* Releases the workspace and every distribution and handle created from ctx. */
nups_status nups_destroy(nups_ctx *ctx);

/*
 * Attaches per-row optimiser state (AdaGrad accumulators, same shape as the table,
 * caller-owned, device).  Table 1 of the paper stores it with the value (1000 values
 * per key for dimension 500); here it is a second array with the same row numbering.
 */
nups_status nups_set_state(nups_ctx *ctx, int table, float *state_dev);

/*
 * Declares the hot keys of a table (Section 3.2: frequently accessed keys get the
 * technique for hot spots, the long tail the other one).  keys_host holds k distinct
 * keys, hottest first.  Without a declaration the library decides per step: a key whose
 * accesses in the step exceed a threshold has its updates summed by several workgroups
 * (LDS pre-aggregation, partial rows combined once), every other key by one row group.
 * With a declaration only declared keys can take the hot path; k = 0 switches it off
 * altogether (every key is summed by one row group, nothing extra is launched).  The set
 * changes how updates are aggregated, never the result beyond fp32 summation order.
 * Waits for the stream (the set is uploaded synchronously).  NUPS_ERR_STATE while prepared
 * steps are outstanding: their structures were begun under the previous set.
 */
nups_status nups_set_hot_keys(nups_ctx *ctx, int table, const uint32_t *keys_host, int64_t k);

/*
 * Stale replicas of the hot keys (Section 3.2: hot-spot keys are replicated on every node; a node's workers read
 * and update the node's replica through shared memory; replicas are synchronised periodically by exchanging the
 * updates accumulated since the last synchronisation; Section 5.7 varies how often).  On one device the nodes
 * become `replicas` contiguous parts of the minibatch (example e of B belongs to part e * replicas / B; with 8,
 * a part is what one of the eight dies works on).  With replicas > 0 every key of the declared hot sets of tables
 * 0 and 1 (nups_set_hot_keys, before this call) gets that many replica rows in a buffer of the library's, all
 * starting from the key's row; from then on NUPS_TASK_SGNS and NUPS_TASK_MF steps read a hot key from the
 * replica of the accessing example's part and add that part's summed gradient to that replica only, while the
 * key's row in the table keeps the value of the last synchronisation; keys that are not hot behave as always.
 * nups_sync_replicas (enqueued on the stream; call it every so many steps: the paper's staleness bound is a
 * time, 40 ms by default, here it is the caller's step count) adds every replica's difference from the row to
 * the row, in replica order, and sets row and replicas to the result.  With one replica, or when synchronising
 * after every step, the result is the plain step's (bit for bit with one replica, to rounding otherwise); in
 * between, a part does not see what the other parts did to a hot key.  replicas = 0 synchronises, frees the
 * replicas and returns to the plain step.  Waits for the stream.
 * While replicas are on: NUPS_TASK_KGE steps return NUPS_ERR_UNIMPLEMENTED (its AdaGrad state is not
 * replicated); nups_push / nups_push_static on a table with replicas, nups_set_hot_keys and
 * nups_set_update_clipping return NUPS_ERR_STATE; nups_pull returns the rows of the table (the last
 * synchronised values); nups_debug_structure lists the replica row r * H + s of hot key number s (of H) as
 * key num_keys + r * H + s.  NUPS_ERR_STATE while prepared steps are outstanding or clipping is on;
 * NUPS_ERR_ARG for replicas outside 0..64.
 */
nups_status nups_set_replicas(nups_ctx *ctx, int32_t replicas);
nups_status nups_sync_replicas(nups_ctx *ctx);

/* Device address and number of rows of a table's replica buffer ([replicas * hot keys][row_stride]; null and 0
 * without replicas), valid until the next nups_set_replicas or nups_destroy: for inspection. */
nups_status nups_replica_rows(nups_ctx *ctx, int table, float **rows_dev, int64_t *n_rows);

/*
 * Reproducible aggregation (the push of Section 3.1 sums the updates sent for a key; in which order is left
 * open).  By default the accesses of a key are listed in the order in which positions were handed out by
 * atomic operations, so the fp32 sum of a key's contributions can differ in its last bits from run to run and
 * with the declared hot set.  enable != 0: structures built from now on also list every key's accesses in
 * ascending order (two more phases of preparatory work: the pieces of a segment are sorted in blocks of 256
 * positions, then merged by binary search; prepare steps four ahead to hide them), and the update
 * kernels add them in a fixed tree over that order (blocks of 16, super-blocks of 256, then in order), whichever
 * technique a key gets: tables are then bit-identical between runs and between hot sets.  The reported loss and
 * the clipping statistics are still accumulated with atomic additions (their last bits may vary).
 * NUPS_ERR_STATE while prepared steps are outstanding.
 */
nups_status nups_set_deterministic(nups_ctx *ctx, int enable);

/*
 * Norm clipping of the updates of hot keys (Section 5.1, implementation paragraph: for the
 * replicated parameters of the word-vector and factorisation tasks, updates that exceed the
 * average norm by more than a factor, 2 in the paper, are clipped, to keep summed gradients of
 * hot keys from exploding).  factor > 0 switches it on for the SGD steps (NUPS_TASK_SGNS,
 * NUPS_TASK_MF) of tables 0 and 1, factor = 0 off (the default); steps with AdaGrad and
 * nups_push are never clipped.  It acts on the keys of a table's declared hot set
 * (nups_set_hot_keys) only.  Per table the library keeps the sum and the number of the Euclidean
 * norms, before clipping, of all hot-key updates (an update = the summed gradient of one key in
 * one step) since clipping was switched on.  A step compares against the mean of the steps
 * before it: a hot key's update of norm n > factor * mean is multiplied by factor * mean / n;
 * while no norm has been recorded nothing is clipped.  Switching on (from off) resets the
 * statistics; calling again with another factor keeps them.  Takes effect for steps run after
 * the call, including steps already prepared.  Waits for the stream when it allocates or resets.
 * NUPS_ERR_ARG: factor negative or not finite.
 */
nups_status nups_set_update_clipping(nups_ctx *ctx, float factor);

/* Reads a table's clipping statistics (waits for the stream): the sum of the recorded norms and
 * their number.  Either pointer may be null.  NUPS_ERR_STATE if clipping was never switched on. */
nups_status nups_get_update_clipping(nups_ctx *ctx, int table, double *norm_sum, double *norm_count);

/* ---- direct access (Section 3.1) ------------------------------------------------- */

/* pull: values_dev[i, :] = table[keys_dev[i], :] for i < n (whole stored rows, row_stride floats each).
 * A key that occurs twice is returned twice.  Out-of-range keys yield a zero row. */
nups_status nups_pull(nups_ctx *ctx, int table, const uint32_t *keys_dev, int64_t n, float *values_dev);

/* push: table[k, :] += sum of updates_dev[i, :] over all i with keys_dev[i] == k (additive; duplicates
 * within one call add up, each key is written once).  updates_dev is [n, row_stride]. */
nups_status nups_push(nups_ctx *ctx, int table, const uint32_t *keys_dev, int64_t n, const float *updates_dev);

/*
 * The same push for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid it): nups_push_static calls no hipMalloc / hipFree and no allocating
 * library routine.  Its workspace is one file-scope device array of fixed size (about 14 MB, held by every GPU the
 * library runs on until the process ends), which limits it to n <= NUPS_STATIC_MAX_PUSH keys per call and tables
 * of at most NUPS_STATIC_MAX_KEYS keys (any supported row_stride); beyond either, NUPS_ERR_ARG, and nups_push is
 * the call to use.  Same arguments, same result as nups_push (to fp32 summation order; identical bits in
 * deterministic mode); nups_debug_structure describes it afterwards like any push.  Every call on a GPU,
 * from whichever context, shares that GPU's array: calls whose kernels overlap on one GPU (different streams)
 * race; calls on one stream are ordered and safe.  The part of the array that must start at zero is cleared by a
 * kernel at the start of every call.
 */
#define NUPS_STATIC_MAX_PUSH 16384
#define NUPS_STATIC_MAX_KEYS 1048576
nups_status nups_push_static(nups_ctx *ctx, int table, const uint32_t *keys_dev, int64_t n, const float *updates_dev);

/* ---- sampling access (Sections 4.3, 4.4) ---------------------------------------- */

/*
 * Host-only helper: builds the alias table of pi_k = weights[k] / sum(weights) (fp64
 * weights, length num_keys).  Bucket b keeps itself when a uniform 32-bit word is
 * below thresh[b] and yields alias[b] otherwise.  Needs no GPU.
 * Errors: NUPS_ERR_ARG for null pointers, negative / NaN / infinite weights or a zero sum.
 */
nups_status nups_build_alias_table(const double *weights_host, int64_t num_keys,
                                   uint32_t *thresh_host, uint32_t *alias_host);

/*
 * register_distribution(pi, L) of Section 4.3: registers the target distribution over
 * the keys of `table` together with the scheme that serves it.  weights_host = NULL
 * means uniform.  Scheme parameters: U (use frequency) and G (pool size) for
 * NUPS_BOUNDED (1 <= G <= 1024); P (pool size) and R (passes per pool) for
 * NUPS_LONGTERM; ignored otherwise.  seed keys the counter-based generator: sample
 * i of the handle prepared for step t is a pure function of (seed, dist, t, i).
 */
nups_status nups_register_distribution(nups_ctx *ctx, int table, const double *weights_host,
                                       nups_scheme scheme, int32_t U, int32_t G, int64_t P, int32_t R,
                                       uint64_t seed, nups_dist **out);

/*
 * The same with a conformity level in place of a scheme (Section 4.1: L1 CONFORM, L2
 * BOUNDED, L3 LONG-TERM; a fourth value stands for "no guarantee asked", NON-CONFORM):
 * the library picks the cheapest scheme that the level admits (Table 2, Section 4.4) with
 * the parameters of the paper's untuned configuration (Section 5.1):
 *   NUPS_CONFORM    -> independent sampling;
 *   NUPS_BOUNDED    -> sample reuse, U = 16, pools of G = 250;
 *   NUPS_LONGTERM   -> sample reuse from a persistent pool of P = 1,000,000 draws, R = 16 passes;
 *   NUPS_NONCONFORM -> local sampling (the caller supplies the batch's keys, nups_set_local_keys).
 * The level is passed as the nups_scheme value of the same name.
 */
nups_status nups_register_distribution_at_level(nups_ctx *ctx, int table, const double *weights_host,
                                                nups_scheme level, uint64_t seed, nups_dist **out);

/*
 * Host-only helper, needs no GPU: the management-technique heuristic of the paper's untuned
 * configuration (Section 5.1): a key is hot (replicated there; given the hot path here) if its
 * access frequency exceeds `factor` (the paper: 100) times the mean access frequency over all
 * num_keys keys.  frequency_host holds one non-negative number per key (counts or relative
 * frequencies, from dataset statistics).  Writes the hot keys, most frequent first (ties: smaller
 * key first), to keys_out_host, at most `capacity` of them, and their total number to *k_out (which
 * may exceed capacity: call again with a larger array).  The result is what nups_set_hot_keys takes.
 * Errors: NUPS_ERR_ARG for null pointers, num_keys < 1, a negative capacity, factor not positive,
 * negative / NaN / infinite frequencies.
 */
nups_status nups_select_hot_keys(const double *frequency_host, int64_t num_keys, double factor,
                                 uint32_t *keys_out_host, int64_t capacity, int64_t *k_out);

/*
 * NUPS_NONCONFORM only: the keys the minibatch accesses anyway, from which samples are
 * taken.  Sample p belongs to example p / per_example; its first `split` samples come
 * from keys_a_dev, the others from keys_b_dev (both [n_examples], may be the same
 * array); candidates are the examples of the same tile of `tile` consecutive examples.
 * The arrays must stay valid until the handles prepared from them are released.
 */
nups_status nups_set_local_keys(nups_dist *dist, const uint32_t *keys_a_dev, const uint32_t *keys_b_dev,
                                int64_t n_examples, int32_t per_example, int32_t split, int32_t tile);

/*
 * NUPS_LONGTERM only: sample reuse WITH POSTPONING (Section 4.4, "Sample reuse with postponing").  The paper's
 * server walks through the prepared samples and moves one whose key is not local at that moment to the end, once,
 * while the key is relocated.  On one device "local" is read as "in the table's declared hot set" (the keys a
 * replication technique keeps resident everywhere; none declared: no key is resident at the start), and the
 * walk covers the N samples of one handle: handles prepared while postponing is on hold the pool's sequence with
 * the first occurrence (within the handle) of every non-resident key moved behind all other samples, the moved
 * samples in the order in which they were met, every other sample in its original order.  The hot set is read
 * when the handle is prepared.  enable = 0 switches back to the plain pool sequence.  Costs 4 bytes of device
 * memory per key of the table while on.  Steps take such samples through batch.sample (the handle); naming the
 * distribution in batch.dist instead returns NUPS_ERR_UNIMPLEMENTED.
 * Errors: NUPS_ERR_ARG for a null distribution, NUPS_ERR_STATE for another scheme, NUPS_ERR_DEVICE.
 */
nups_status nups_set_postponing(nups_dist *dist, int enable);

/*
 * PrepareSample(dist, N): enqueues the drawing of N sample keys for step `step` (one
 * launch on the stream) and returns at once.  For NUPS_LONGTERM the distribution's cursor advances by N (step
 * is ignored).  The handle must be released with nups_release_sample.
 */
nups_status nups_prepare_sample(nups_dist *dist, int64_t n, uint64_t step, nups_sample **out);

/*
 * PullSample(handle, n_j): hands out the next n_j samples of the handle: their keys
 * into keys_dev[n_j] and, if values_dev != NULL, their rows into values_dev[n_j,
 * row_stride].  Partial pulls may be repeated until the N samples are used up;
 * asking for more returns NUPS_ERR_OVERPULL and hands out nothing.  The copies are
 * enqueued on the stream (stream-ordered, not host-blocking).
 */
nups_status nups_pull_sample(nups_sample *handle, int64_t n_j, uint32_t *keys_dev, float *values_dev);

/* Device address of all N keys of the handle (valid until release).  Work enqueued on the stream
 * after nups_prepare_sample sees the keys. */
nups_status nups_sample_keys(nups_sample *handle, const uint32_t **keys_dev, int64_t *n);

/* Gives the handle back; releasing twice is NUPS_ERR_STATE. */
nups_status nups_release_sample(nups_sample *handle);

/* ---- one minibatch step (Section 5.1 tasks) ------------------------------------- */

typedef struct {
    int32_t task;          /* nups_task                                                          */
    int64_t B;             /* examples in the batch                                              */
    const uint32_t *k0;    /* dev [B]: SGNS center word | MF row    | KGE subject                 */
    const uint32_t *k1;    /* dev [B]: SGNS context word| MF column | KGE relation                */
    const uint32_t *k2;    /* dev [B]: KGE object (else NULL)                                     */
    const float *val;      /* dev [B]: MF cell value (else NULL)                                  */
    int32_t n_neg;         /* SGNS: negatives per pair; KGE: subject-replacing negatives per triple */
    int32_t n_neg2;        /* KGE: object-replacing negatives per triple (else 0)                 */
    float lr;              /* learning rate                                                       */
    float l2;              /* MF: L2 regularisation weight                                        */
    float eps;             /* KGE: AdaGrad epsilon                                                */
    const uint32_t *negs;  /* dev [B * (n_neg + n_neg2)] sampled keys, example-major (NULL if none or if
                              `sample` is given)                                                   */
    nups_sample *sample;   /* alternatively: the handle whose N >= B * (n_neg + n_neg2) keys are the
                              negatives.  NULL if `negs` is given or there are none.              */
    nups_dist *dist;       /* alternatively: the step draws its own B * (n_neg + n_neg2) negatives from
                              this distribution as PrepareSample(dist, N) for step `sample_step` would
                              (same keys), without a handle, as part of its preparatory work.  NULL
                              otherwise.                                                           */
    uint64_t sample_step;  /* step number of that drawing (ignored unless `dist` is given)        */
} nups_batch;

/*
 * One synchronous minibatch step on tables 0 and 1 of the context
 * (SGNS: input / output vectors; MF: row / column factors; KGE: entities / relations,
 * both with state attached).  All gradients are taken against the values at the start
 * of the step, contributions to one key are summed, and each touched row is updated
 * once (SGD, or AdaGrad for KGE).  If loss_sum_host != NULL the call waits for the
 * step and stores the batch loss (and reports pending key-range errors); with NULL it
 * only enqueues.
 */
nups_status nups_step(nups_ctx *ctx, const nups_batch *batch, double *loss_sum_host);

/*
 * The same step in two halves, in the manner of PrepareSample / PullSample (Section 4.3).
 * nups_prepare_step hands the batch to the library and returns at once, without enqueuing
 * anything: the work that depends only on the batch's keys (drawing the step's own negatives,
 * the per-key aggregation structure) is a chain of six short phases (seven for more than
 * 131,072 accesses to a table, two more in deterministic mode), and every gradient or update launch
 * of a step that runs afterwards carries one phase of each of the four oldest prepared steps in spare
 * workgroups.
 * nups_step_prepared first enqueues, as launches of their own, whatever phases of this step
 * have not been carried yet, then the step's two launches.  So with steps prepared three
 * ahead (prepare t+3, run t) a step costs two launches and its preparatory work hides inside
 * earlier steps; prepared less far ahead, part of it runs on its own; nups_step(batch) is
 * prepare followed by run and runs all of it on its own.  A NUPS_TASK_MF step that is prepared
 * while three others are still under construction (steps prepared four ahead) starts its chain
 * one launch later, which puts its long phases into the gradient launches (its update kernel is
 * short); that is the fastest arrangement for this task.  The results are the same in every
 * case.  The key arrays of the batch (and the sampled keys or batch-local key arrays it
 * points to) must stay valid and unchanged until the step has run; arrays written by work
 * enqueued on the stream before nups_prepare_step are seen complete.  A prepared step is
 * consumed by running it; running it twice is NUPS_ERR_STATE.
 */
nups_status nups_prepare_step(nups_ctx *ctx, const nups_batch *batch, nups_prepared **out);
nups_status nups_step_prepared(nups_ctx *ctx, nups_prepared *step, double *loss_sum_host);

/*
 * Aggregation structure of the last nups_step / nups_push on `table`: the distinct
 * keys in ascending order and how many accesses each received.  Buffers are device
 * arrays with room for as many entries as the call had accesses to that table.
 * Waits for the stream.
 */
nups_status nups_debug_structure(nups_ctx *ctx, int table, uint32_t *uniq_keys_dev, uint32_t *counts_dev,
                                 int64_t *n_uniq_host);

/* Waits for the stream and returns NUPS_ERR_KEY_RANGE if any kernel since the last check saw a bad key. */
nups_status nups_check(nups_ctx *ctx);

/* ---- measurement ------------------------------------------------------------------ */

/* Phases whose device time can be recorded with HIP events around their launches: drawing a step's
 * samples, building its aggregation structure, the gradient kernel, the update of both tables (APPLY0; APPLY1 is
 * kept for callers that number the phases and stays empty), pull, push. */
enum { NUPS_PHASE_SAMPLE = 0, NUPS_PHASE_PLAN = 1, NUPS_PHASE_GRAD = 2, NUPS_PHASE_APPLY0 = 3,
       NUPS_PHASE_APPLY1 = 4, NUPS_PHASE_PULL = 5, NUPS_PHASE_PUSH = 6, NUPS_PHASE_COUNT = 7 };

/* Switches per-phase event timing on or off (off by default; it adds event records to the stream).  While it
 * is on, nups_prepare_step enqueues the step's preparatory phases at once as launches of their own, so that
 * each phase is timed bare and the gradient and update launches carry nothing. */
nups_status nups_profile(nups_ctx *ctx, int enable);

/* Waits for the stream; returns accumulated milliseconds and launch count of a phase and resets them. */
nups_status nups_profile_read(nups_ctx *ctx, int phase, double *ms_total, int64_t *launches);

const char *nups_phase_name(int phase);

/* Description of the calling thread's last error ("" if none). */
const char *nups_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* NUPS_H */
