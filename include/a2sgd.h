/*
 * a2sgd.h — C ABI of the A2SGD (two-level gradient averaging) per-step hot path for one MI355X (gfx950).
 *
 * The method (arXiv 2006.07405): each of P data-parallel workers reduces its n-element gradient to two
 * numbers, the mean of the entries >= 0 and the mean magnitude of the entries < 0 (Sec. 3.1); the workers
 * average those two numbers (Algorithm 1 line 5); each rebuilds an update from the two global means at the
 * positions of its own two sign groups and keeps the difference to its own means as a local error vector
 * (Algorithm 1 lines 4 and 6; Eq. 2); the model takes w <- w - eta * update (line 7).
 *
 * Here the P workers are P (gradient, error) buffer pairs resident on one GPU plus one shared weight buffer,
 * which stands for the average of the P replicas: the applied update is the mean over the workers of their
 * rebuilt updates (Eq. 1 with each worker's gradient replaced by its rebuilt one).
 *
 * Notation: n parameters, P workers, g^p / e^p worker p's gradient / error, v^p = fl32(g^p + e^p) the vector
 * that is encoded.  All buffers are fp32.
 *
 * Conventions for every entry point
 *   - Pointers named g, e, w, workspace, mask are DEVICE pointers; `g` and `e` themselves are HOST arrays of
 *     P device pointers (copied into the kernel arguments at launch).  Everything else is host memory.
 *   - Ownership: the library never allocates, frees or keeps user device memory.  Buffers are borrowed until
 *     the work enqueued on `stream` has completed.  The plan is the only object the library owns.
 *   - Aliasing: g^p is read-only; e^p and w are updated in place.  A buffer that a call writes (e^p, w, w^p, the
 *     workspace) must not overlap any other buffer of that call (else A2SGD_ERR_INVALID_ARG); buffers that are
 *     only read may coincide.
 *   - Alignment: every device pointer must be 16-byte aligned (else A2SGD_ERR_ALIGNMENT).  n is arbitrary.
 *   - Asynchrony: the step calls only enqueue kernels on `stream` (a hipStream_t passed as void*; NULL is the
 *     default stream) and return.  Only a2sgd_read_stats synchronises.
 *   - Errors: a status code is returned; nothing is thrown or aborted.  Argument errors are found before any
 *     kernel is launched, so a failed call has enqueued nothing.
 *   - Determinism: no floating-point atomics; the same plan on the same inputs gives bit-identical outputs.
 *   - Inputs are expected finite.  A NaN in v^p belongs to neither sign group: it is counted in n_nan, adds to
 *     no sum, and turns only its own e and w entries into NaN.
 */
#ifndef A2SGD_H
#define A2SGD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define A2SGD_MAX_WORKERS 64u

typedef struct a2sgd_plan a2sgd_plan_t; /* opaque; host memory owned by the library */
typedef void *a2sgd_stream_t;           /* a hipStream_t */

typedef enum {
    A2SGD_OK = 0,
    A2SGD_ERR_INVALID_ARG = 1, /* NULL where a pointer is required, n == 0, P out of range, bad mode */
    A2SGD_ERR_ALIGNMENT = 2,   /* a device pointer is not 16-byte aligned */
    A2SGD_ERR_DEVICE = 3,      /* a HIP call or kernel launch failed */
    A2SGD_ERR_NOMEM = 4,       /* host allocation of the plan failed */
    A2SGD_ERR_WORKSPACE_TOO_SMALL = 5, /* a2sgd_workspace_check: fewer bytes than a2sgd_workspace_bytes */
    A2SGD_ERR_WORKSPACE_STATE = 6,     /* a plan with tensors found a workspace that a2sgd_workspace_init has not
                                          prepared for it; the calls since then have computed nothing */
    A2SGD_ERR_SCRATCH_LIMIT = 7        /* a2sgd_step_static: the plan needs more than A2SGD_STATIC_SCRATCH_BYTES */
} a2sgd_status_t;

typedef enum {
    /* v = fl32(g + e_old); the update applied is the global-mean vector alone; e_new = v - enc(v) is kept
     * for the next step.  (Abstract and Sec. 3: each worker keeps its errors in a local error vector.) */
    A2SGD_MODE_RETAINED_ERROR = 0,
    /* Algorithm 1 lines 4-7 as printed: the error is added back in the same step, update = e_new + global-mean
     * vector, which is Theorem 1's g + (net gain of the means).  e may be NULL (then v = g and no error is
     * stored); if e is given it is folded in and overwritten like in the other mode. */
    A2SGD_MODE_ALG1_LITERAL = 1
} a2sgd_mode_t;

typedef struct {
    uint64_t n;                 /* model size, 1 <= n <= 2^38 */
    uint32_t num_workers;       /* P, 1 <= P <= A2SGD_MAX_WORKERS */
    int32_t mode;               /* an a2sgd_mode_t */
    uint32_t blocks_per_worker; /* 0 = let the plan choose; else the first-level reduction's grid width */
    uint32_t num_segments;      /* 0: the whole range [0, n) is the model (the paper's method, one pair of means per
                                   worker).  S >= 1: the model consists of S tensors (segments) inside [0, n), see
                                   "Tensors" below.  At most 2^20. */
    const uint64_t *seg_length; /* HOST array of num_segments tensor sizes (each >= 1) in ascending address order; read
                                   during a2sgd_plan only; ignored (may be NULL) when num_segments is 0 */
    const uint64_t *seg_offset; /* HOST array of num_segments start indices, or NULL: the tensors are packed back to
                                   back from 0 and their sizes sum to n.  With offsets the tensors must not overlap
                                   and must end by n; elements outside every tensor are padding: neither counted nor
                                   read for the means nor written */
    uint32_t pooled_means;      /* with num_segments >= 1: 0 = one pair of means per worker and tensor; 1 = one pair
                                   per worker over all tensors together (the paper's whole-model means on a buffer
                                   that has padding).  Must be 0 when num_segments is 0 */
    int32_t device;             /* HIP device index the plan is made for: every call that enqueues work first checks
                                   that this device is the current one (else A2SGD_ERR_DEVICE, nothing enqueued).
                                   -1: no check, the calls run on whichever device is current */
} a2sgd_config_t;

/* Per-worker result of the reduction (Sec. 3.1; the pair (mu_pos, mu_neg) is the worker's 64-bit message of
 * Sec. 4.3).  An empty group has mean 0.  n_zero (entries == 0, a subset of n_pos) and n_nan are diagnostics. */
typedef struct {
    float mu_pos, mu_neg;
    uint64_t n_pos, n_neg, n_zero, n_nan;
} a2sgd_worker_stats_t;

/* The two global means of Algorithm 1 line 5: plain averages of the P workers' means. */
typedef struct {
    float gmu_pos, gmu_neg;
} a2sgd_global_stats_t;

/* Host only, launches nothing.  Validates cfg and fixes the launch geometry and the workspace layout.
 * *out_plan is written only on success and must be released with a2sgd_plan_destroy.
 * Thread safety: different plans may be used from different host threads at once.  One plan must not be used by
 * two host threads at the same time (a call notes in the plan what it enqueued), and must not be destroyed
 * while work enqueued with it is still running. */
a2sgd_status_t a2sgd_plan(const a2sgd_config_t *cfg, a2sgd_plan_t **out_plan);
a2sgd_status_t a2sgd_plan_destroy(a2sgd_plan_t *plan);

/* Bytes of device workspace the caller must provide (16-byte aligned) to the calls below.  Its contents need
 * no initialisation; it carries the block partials, the per-worker means and counts and the global means from
 * one call of a step to the next.  It includes the records of the lazy calls' reduction pass (40 bytes per 2048
 * elements and worker) and, in A2SGD_MODE_RETAINED_ERROR, one sign bit per element and worker for the lazy calls
 * and for the apply pass of plans with 8 workers or more: about 0.15 bytes per element and worker in all.
 * Returns 0 for a NULL plan. */
size_t a2sgd_workspace_bytes(const a2sgd_plan_t *plan);

/* Host only.  The step calls take a workspace pointer without a size; a caller that wants the size checked passes
 * the buffer here once: A2SGD_ERR_INVALID_ARG for a NULL plan or pointer, A2SGD_ERR_ALIGNMENT, and
 * A2SGD_ERR_WORKSPACE_TOO_SMALL if `bytes` is less than a2sgd_workspace_bytes(plan). */
a2sgd_status_t a2sgd_workspace_check(const a2sgd_plan_t *plan, const void *workspace, size_t bytes);

/* Algorithm 1 line 3.  For every worker p: one pass over v^p = fl32(g^p + e^p) giving n_pos = #{v >= 0},
 * n_neg = #{v < 0}, the two sums, and from them mu_pos = fl32(S_pos / n_pos), mu_neg = fl32(S_neg / n_neg)
 * (0 for an empty group).  Sums are accumulated in fp64 and combined in a fixed order.  Results stay in the
 * workspace.  e may be NULL only in A2SGD_MODE_ALG1_LITERAL (then v = g).  Reads g and e once. */
a2sgd_status_t a2sgd_local_averages(const a2sgd_plan_t *plan, const float *const *g, const float *const *e,
                                    void *workspace, a2sgd_stream_t stream);

/* Algorithm 1 line 5, the stand-in for the Allreduce(average) of two floats per worker: gmu_pos and gmu_neg
 * are the fp64 sums over p = 0..P-1 of the workers' fp32 means, divided by P and rounded to fp32.  Reads and
 * writes only the workspace; must follow a2sgd_local_averages on the same stream. */
a2sgd_status_t a2sgd_global_average(const a2sgd_plan_t *plan, void *workspace, a2sgd_stream_t stream);

/* Algorithm 1 lines 4, 6 and 7 in one pass.  For every i and p: v = fl32(g^p_i + e^p_i); if v >= 0 then
 * e^p_i <- v - mu_pos^p and u^p = +gmu_pos, else e^p_i <- v + mu_neg^p and u^p = -gmu_neg (literal mode:
 * u^p = new e^p_i + that).  Then w_i <- w_i - eta * (1/P) * sum_p u^p.  g, e and w are each read once, e and
 * w written once; the rebuilt gradient is never stored.  Must follow a2sgd_global_average on the same stream
 * with the same g and e that a2sgd_local_averages saw.  eta is the learning rate of this step. */
a2sgd_status_t a2sgd_apply_and_update_error(const a2sgd_plan_t *plan, const float *const *g, float *const *e,
                                            float *w, float eta, void *workspace, a2sgd_stream_t stream);

/* One whole step of Algorithm 1's loop body (lines 3-7) on one stream: the same result as the three calls above
 * in order (to the tolerance of the sums' grouping: the counts are identical, the fp64 sums are combined in
 * another fixed order).  When g, e and w together are small enough to stay in the on-chip caches (below 192 MiB)
 * the step is ONE kernel launch with a grid-wide barrier inside; larger models run the three passes.  The
 * barrier's cell is library-owned device memory, one of 64 cells: such a plan owns one from a2sgd_plan to
 * a2sgd_plan_destroy, so no two live plans share a cell; a plan made while all 64 are taken runs the three passes,
 * as does any plan on a device with fewer compute units than its grid has workgroups
 * (a2sgd_plan_single_launch_cell tells).  The launch needs its whole grid on the device at once, and the device
 * holds two such grids: single-launch steps of two plans may run at the same time on two streams; with more than two
 * in flight at once a grid may have to wait for another to drain, within the bounded wait described next.  Calls with the same plan must
 * not overlap (they share the workspace anyway).  The barrier's wait is bounded; should it ever run out, that
 * step's outputs are invalid and later single-launch steps of the plan do nothing, until a2sgd_read_stats reports
 * it once with A2SGD_ERR_DEVICE; from then on the plan runs the three passes. */
a2sgd_status_t a2sgd_step(const a2sgd_plan_t *plan, const float *const *g, float *const *e, float *w, float eta,
                          void *workspace, a2sgd_stream_t stream);

/* For callers that cannot allocate device memory or pass a workspace (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): a2sgd_step's three passes (never the single launch) with the header and
 * the block partial records in a fixed array inside the library's own device memory instead of a workspace.  The
 * array has A2SGD_STATIC_SCRATCH_BYTES on every GPU the library runs on, for the life of the process; a whole-model
 * plan fits if 4096 + 40 * P * a2sgd_plan_blocks_per_worker(plan) is no more than that (every plan made with
 * blocks_per_worker = 0 does), otherwise A2SGD_ERR_SCRATCH_LIMIT and nothing is enqueued; plans with tensors get
 * A2SGD_ERR_INVALID_ARG.  The call allocates and frees nothing, copies nothing and does not synchronise: it only
 * enqueues the same kernels as a2sgd_local_averages, a2sgd_global_average and a2sgd_apply_and_update_error, so e and
 * w come out bit-identical to those three calls.  Every pass rewrites what it reads from the array, so nothing in it
 * has to start at zero and what an earlier call left does not matter.  All calls on one GPU share the array: two
 * calls that may run at the same time on that GPU (two streams, two host threads) race and give wrong results;
 * calls ordered by one stream are safe.  The statistics are not readable after this call (a2sgd_read_stats needs
 * a workspace). */
#define A2SGD_STATIC_SCRATCH_BYTES (256u * 1024u)
a2sgd_status_t a2sgd_step_static(const a2sgd_plan_t *plan, const float *const *g, float *const *e, float *w, float eta,
                                 a2sgd_stream_t stream);

/* Copies the per-worker and global results of the last completed reduction out of the workspace into host
 * memory: out_workers[P] and *out_global (either may be NULL).  Synchronises `stream`.  For tests and logging. */
a2sgd_status_t a2sgd_read_stats(const a2sgd_plan_t *plan, const void *workspace, a2sgd_stream_t stream,
                                a2sgd_worker_stats_t *out_workers, a2sgd_global_stats_t *out_global);

/* Test aid: writes pos(v^p) of Eq. 2 as a bitmap, mask[p * ceil(n/64) + i/64] bit (i % 64) = (v^p_i >= 0),
 * bits beyond n are 0.  mask is a device buffer of P * ceil(n/64) uint64.  e may be NULL (v = g). */
a2sgd_status_t a2sgd_export_mask(const a2sgd_plan_t *plan, const float *const *g, const float *const *e,
                                 uint64_t *mask, a2sgd_stream_t stream);

/* Dense data-parallel SGD, Eq. 1, which is also the final synchronisation step of Algorithm 1 (lines 9-10):
 * w_i <- w_i - eta * (1/P) * sum_p g^p_i.  Reads every g^p and w once, writes w once. */
a2sgd_status_t a2sgd_dense_step(const a2sgd_plan_t *plan, const float *const *g, float *w, float eta,
                                a2sgd_stream_t stream);

/* ---- Tensors: per-tensor means, and buffers with padding -------------------------------------------------------
 * A plan made with num_segments = S >= 1 treats the flat buffers as S tensors (segments).  With pooled_means = 0 it
 * applies the operator of Eq. 2 and Algorithm 1 lines 3-7 to every tensor on its own: worker p has one pair of
 * local means per tensor, the global means are averaged over the workers per tensor, and each element is encoded
 * with the means of its tensor (2S scalars per worker and step instead of 2).  With pooled_means = 1 every worker
 * has one pair of means over all its tensors together, as in the paper, and the tensors only say which elements of
 * the buffers belong to the model.  Elements outside every tensor (possible with seg_offset) are left alone by every
 * call except a2sgd_dense_step and a2sgd_export_mask, which do not depend on the segments.
 * a2sgd_local_averages, a2sgd_global_average, a2sgd_apply_and_update_error and a2sgd_step work as described above
 * (a2sgd_step is one kernel launch for such a plan too, when the model stays in the caches, has at most about 4 M
 * elements and its means are not pooled: the paper's own FNN-3 and ResNet-20 with a pair of means per layer),
 * and so do the replica calls and the lazy calls further down, each element with the means of its tensor (the lazy
 * state carries one pair of means per worker and tensor, and the same bytes per step as on a whole-model plan).  Not available on such a plan (A2SGD_ERR_INVALID_ARG): a2sgd_step_static, the export/import pair, and
 * a2sgd_read_stats unless the means are pooled.  The workspace of such a plan holds static lookup tables: */

/* Uploads the plan's segment tables into the workspace, and last a tag that identifies them.  Required once per
 * workspace, before its first use, when the plan has num_segments >= 1; a no-op otherwise.  Enqueues on `stream`
 * and synchronises it before returning (a set-up call: the tables are copied from the plan's own host memory, which
 * may then be released at any time).  A step call on a workspace that does not carry this plan's tag reads
 * no table and writes no output: its kernels exit at once and leave a mark, which a2sgd_read_segment_stats (and
 * a2sgd_read_stats with pooled means) reports as A2SGD_ERR_WORKSPACE_STATE until a2sgd_workspace_init has run. */
a2sgd_status_t a2sgd_workspace_init(const a2sgd_plan_t *plan, void *workspace, a2sgd_stream_t stream);

/* Per-tensor results of the last completed reduction: out_workers[p * S + s] for worker p and tensor s (host array
 * of P * S records, may be NULL) and out_global[s] (host array of S, may be NULL).  Synchronises `stream`. */
a2sgd_status_t a2sgd_read_segment_stats(const a2sgd_plan_t *plan, const void *workspace, a2sgd_stream_t stream,
                                        a2sgd_worker_stats_t *out_workers, a2sgd_global_stats_t *out_global);

/* ---- One weight vector per worker: Algorithm 1 as each worker runs it on its own replica ------------------
 * `w` is a HOST array of P DEVICE pointers, like g and e; w^p is updated in place.  The same workspace serves. */

/* Algorithm 1 lines 4, 6 and 7 exactly as printed for worker p: e^p as in a2sgd_apply_and_update_error, and
 * w^p_i <- w^p_i - eta * u^p_i with that worker's own rebuilt update, no averaging over the workers.  The mean
 * of the P replicas then moves exactly as the single w of a2sgd_apply_and_update_error does.  Reads g, e, w^p
 * once, writes e and w^p once: 20 bytes per element and worker. */
a2sgd_status_t a2sgd_apply_and_update_error_replicas(const a2sgd_plan_t *plan, const float *const *g, float *const *e,
                                                     float *const *w, float eta, void *workspace,
                                                     a2sgd_stream_t stream);

/* a2sgd_local_averages, a2sgd_global_average and a2sgd_apply_and_update_error_replicas, in order. */
a2sgd_status_t a2sgd_step_replicas(const a2sgd_plan_t *plan, const float *const *g, float *const *e, float *const *w,
                                   float eta, void *workspace, a2sgd_stream_t stream);

/* The synchronisation step that ends Algorithm 1 (lines 9-10): every replica takes the dense averaged gradient,
 * w^p_i <- w^p_i - eta * (1/P) * sum_q g^q_i. */
a2sgd_status_t a2sgd_dense_step_replicas(const a2sgd_plan_t *plan, const float *const *g, float *const *w, float eta,
                                         a2sgd_stream_t stream);

/* How far the replicas have drifted apart: with wbar_i = (1/P) sum_p w^p_i, out_max_abs[p] = max_i |w^p_i -
 * wbar_i| and out_rms[p] = sqrt((1/n) sum_i (w^p_i - wbar_i)^2), both host arrays of P doubles (either may be
 * NULL).  Overwrites the workspace's partial records; synchronises `stream`.  A diagnostic, not on the step. */
a2sgd_status_t a2sgd_replica_drift(const a2sgd_plan_t *plan, const float *const *w, void *workspace,
                                   a2sgd_stream_t stream, double *out_max_abs, double *out_rms);

/* ---- Lazy error state: the same step with less traffic than a2sgd_step's 20nP + 8n bytes -------------------
 * Between lazy steps worker p's buffer s^p holds the folded vector v^p of the last step instead of the error,
 * and the workspace carries that step's local means; the error is e^p_i = fl32(s^p_i - enc(s^p)_i) with those
 * means (Eq. 2), and it is formed on the fly when the next step reads the buffer.  The reduction pass then reads
 * g and s and writes the new v into s (12 bytes per element and worker).  What the apply pass reads depends on
 * the plan's mode.  A2SGD_MODE_ALG1_LITERAL: s again, for the errors that enter the update (4 bytes per element
 * and worker plus 8 per parameter: 16nP + 8n in all).  A2SGD_MODE_RETAINED_ERROR: the update of a parameter
 * depends only on how many workers have it in the positive group, so the reduction pass also leaves pos(v) as one
 * bit per element and worker in the workspace and the apply pass reads those (12.25nP + 8n in all; if any worker
 * counted a NaN, which has no sign, it reads s instead).  The counts are the same as a2sgd_step's; the means may
 * differ from its in the last bit (the sums are grouped differently) and w by an ulp; the errors once
 * materialised are those of a2sgd_step within that.
 * A workspace in lazy use carries state: between a2sgd_lazy_reset and a2sgd_lazy_materialize it must see no other
 * calls than the a2sgd_lazy_* ones, a2sgd_global_average, the export/import pair and a2sgd_read_stats.  s is
 * required. */

/* Declares that the buffers that will be passed as s hold true errors (for a fresh run: zeros): clears the local
 * means carried in the workspace.  Call once before the first a2sgd_lazy_step on a workspace. */
a2sgd_status_t a2sgd_lazy_reset(const a2sgd_plan_t *plan, void *workspace, a2sgd_stream_t stream);

/* Algorithm 1 line 3 on the lazy state: forms every worker's pending error, folds it into the gradient, stores the
 * new v in s and leaves the local means, counts (and, in retained-error mode, sign bits) in the workspace.
 * a2sgd_global_average, or a2sgd_export_local_means / a2sgd_import_global_means, follows. */
a2sgd_status_t a2sgd_lazy_local_averages(const a2sgd_plan_t *plan, const float *const *g, float *const *s,
                                         void *workspace, a2sgd_stream_t stream);

/* Algorithm 1 lines 6-7 on the lazy state: updates w from the sign groups; s is only read. */
a2sgd_status_t a2sgd_lazy_apply(const a2sgd_plan_t *plan, const float *const *s, float *w, float eta, void *workspace,
                                a2sgd_stream_t stream);

/* One step of Algorithm 1's loop body (lines 3-7) on the lazy state: a2sgd_lazy_local_averages,
 * a2sgd_global_average and a2sgd_lazy_apply, in order. */
a2sgd_status_t a2sgd_lazy_step(const a2sgd_plan_t *plan, const float *const *g, float *const *s, float *w, float eta,
                               void *workspace, a2sgd_stream_t stream);

/* Turns the lazy state back into true errors, in place: s^p <- fl32(s^p - enc(s^p)), and clears the carried
 * means (so the buffers may go on as s, or be handed to a2sgd_step as e).  For checkpoints and hand-over. */
a2sgd_status_t a2sgd_lazy_materialize(const a2sgd_plan_t *plan, float *const *s, void *workspace,
                                      a2sgd_stream_t stream);

/* ---- Where a real collective goes: Algorithm 1 line 5 done by the caller ------------------------------------
 * When the workers live on different GPUs (one process per GPU, each with a plan of its own workers, typically
 * P = 1), the average of line 5 is the caller's collective over 2 floats per worker.  The two calls below replace
 * a2sgd_global_average for that: a2sgd_local_averages, a2sgd_export_local_means, the caller's all-reduce (average)
 * or all-gather of the pairs on the same stream, a2sgd_import_global_means, a2sgd_apply_and_update_error.  Both only
 * enqueue a small kernel; nothing comes to the host.  Whole-model plans only. */

/* Writes this plan's P pairs (mu_pos^p, mu_neg^p), as left by a2sgd_local_averages, to `out`: a DEVICE array of
 * 2 * P floats, out[2p] = mu_pos^p, out[2p + 1] = mu_neg^p. */
a2sgd_status_t a2sgd_export_local_means(const a2sgd_plan_t *plan, const void *workspace, float *out,
                                        a2sgd_stream_t stream);

/* Takes the global means from `gmu`, a DEVICE array of 2 floats (gmu_pos, gmu_neg: the average over ALL workers of
 * the job of their local means, formed by the caller), instead of averaging this plan's own workers. */
a2sgd_status_t a2sgd_import_global_means(const a2sgd_plan_t *plan, void *workspace, const float *gmu,
                                         a2sgd_stream_t stream);

/* Diagnostic: exercises the grid-wide barrier of the single-launch step on a cell of its own.  First 128
 * workgroups must all pass one barrier; then 128 workgroups wait, with a limit of 64 polls, for an arrival that
 * never comes: every one of them must give up, exit normally and leave the cell marked failed.  Returns A2SGD_OK
 * if both behaved, A2SGD_ERR_DEVICE otherwise.  `buffer` is at least 4 KiB of device memory (a workspace
 * will do; its contents are overwritten).  Synchronises `stream`. */
a2sgd_status_t a2sgd_selftest_barrier(void *buffer, a2sgd_stream_t stream);

/* Geometry the plan chose, for reports: blocks per worker of the first-level reduction. */
uint32_t a2sgd_plan_blocks_per_worker(const a2sgd_plan_t *plan);

/* The grid-barrier cell (0..63) that a2sgd_step's single launch uses with this plan, or -1 if the plan runs the
 * three passes (model too large for the caches, tensors with pooled means or more than about 4 M elements, no free
 * cell when it was made, or a step that gave up at its barrier).  Host call. */
int32_t a2sgd_plan_single_launch_cell(const a2sgd_plan_t *plan);

/* What the current HIP device reports about itself, for benchmark reports: compute units, memory clock (kHz) and
 * bus width (bits), total device memory and L2 size in bytes.  (An MI355X reports 2,000,000 kHz and 8192 bits; its
 * HBM3E moves 4 bits per pin and reported clock, 8192 GB/s, which the published 8000 GB/s rounds.)  Host call;
 * `out` is host memory. */
typedef struct {
    uint32_t compute_units;
    uint32_t memory_clock_khz;
    uint32_t memory_bus_bits;
    uint32_t reserved;
    uint64_t total_memory_bytes;
    uint64_t l2_bytes;
} a2sgd_device_info_t;
a2sgd_status_t a2sgd_device_info(a2sgd_device_info_t *out);

const char *a2sgd_status_string(a2sgd_status_t status);

#ifdef __cplusplus
}
#endif
#endif /* A2SGD_H */
