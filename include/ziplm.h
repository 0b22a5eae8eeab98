/*
 * ziplm.h -- C ABI of the MI355X (gfx950) structured Optimal-Brain-Surgeon pruning library.
 *
 * The library implements the layer-wise pruner of ZipLM (Section 3.1, Eq. 1-4, Algorithm 1):
 *
 *   1. ziplm_hessian_accumulate   H += scale * X X^T over batches of calibration inputs
 *   2. ziplm_hinv                 Hinv = (H + lambda I)^-1 through a Cholesky factorisation
 *   3. ziplm_structured_obs_prune the greedy loop: score every remaining structure (Eq. 2),
 *                                 remove the cheapest, compensate the remaining weights (Eq. 3),
 *                                 eliminate the structure from Hinv (Eq. 4), k times; then mask.
 *   and, for the sparsity search that consumes the pruned layers (Section 3.2):
 *      ziplm_module_error         error of dropping the whole module, tr(W (H + lambda I) W^T)
 *      ziplm_prior                p_s after every removal of a run
 *      ziplm_search_select/mutate the search itself, on the host
 *
 * Conventions
 *   - Every matrix is row-major.  W is d_row x d_col; a structure is a set of COLUMNS of W
 *     (input features).  Structure s = columns [s*group_size, (s+1)*group_size): one column for a
 *     feed-forward neuron, d_head = 64 consecutive columns for an attention head ("Pruned
 *     structures", Section 3.1).
 *   - Pointers are DEVICE pointers unless the name ends in _host.  The caller owns every buffer.
 *     Scratch space is passed in as `workspace` (256-byte aligned, size from the matching
 *     *_workspace_bytes call) and may be reused or freed as soon as the work enqueued by the
 *     call has finished.  No entry point allocates or frees device memory except
 *     ziplm_exchange_alloc, whose only purpose is to allocate.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue work
 *     on that stream and return without waiting, except where a *_host output is requested.
 *   - Return value: ZIPLM_OK or a negative ziplm_status.  Argument errors are detected before
 *     anything is enqueued and leave all buffers untouched.  No exception crosses this boundary.
 *   - The library keeps no state between calls and reads no environment variable.  Calls on
 *     different streams are independent as long as every buffer they write (outputs, workspace,
 *     exchange area) is theirs alone.  One rule per device: a greedy loop over single columns
 *     (group_size == 1) is one persistent launch that takes a workgroup slot on every compute unit, so
 *     two such loops never run side by side; enqueue them on one stream or order them with events.
 *     The runtime would run them one after the other anyway, but in an order of its choosing.
 */
#ifndef ZIPLM_H
#define ZIPLM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ZIPLM_OK = 0,
    ZIPLM_ERR_INVALID_ARG = -1, /* null pointer, bad size, d_col % group_size != 0, ... */
    ZIPLM_ERR_NOT_PD = -2,      /* a Cholesky pivot (of H + lambda I or of a block of Hinv) was <= 0 */
    ZIPLM_ERR_WORKSPACE = -3,   /* workspace null, misaligned or smaller than *_workspace_bytes */
    ZIPLM_ERR_DEVICE = -4,      /* a HIP call failed, or the device-side loop gave up waiting */
    ZIPLM_ERR_UNSUPPORTED = -5  /* valid request that this build does not cover */
} ziplm_status;

typedef enum {
    ZIPLM_X_FEATURE_MAJOR = 0, /* X[d_col][n_tok], ldx >= n_tok: the paper's X (Eq. 1)      */
    ZIPLM_X_TOKEN_MAJOR = 1    /* X[n_tok][d_col], ldx >= d_col: how activations are captured */
} ziplm_xlayout;

/* Library version: major*10000 + minor*100 + patch. */
int ziplm_version(void);

/* Static, human-readable name of a status code. */
const char *ziplm_status_string(int status);

/*
 * Calibration Hessian (Section 3.1 "Saliency scores and weight update": H = X X^T; the caption
 * of Algorithm 1 uses 2 X X^T, hence `scale`).
 *
 *   H (d_col x d_col, leading dimension d_col, fp32)  +=  scale * X X^T
 *
 * X holds n_tok calibration inputs of d_col features each, fp32, in the given layout with
 * leading dimension ldx.  The caller zero-fills H before the first batch and may call this once
 * per batch.  Both triangles of H are valid on return.  Products and sums are fp32 (matrix-core
 * fp32 multiply-accumulate); no reduced-precision input format is used.
 * n_tok == 0 is a no-op.  `workspace` may be NULL only if ziplm_hessian_workspace_bytes
 * returns 0 for these sizes.  The result does not depend on run-to-run scheduling (partial sums
 * are combined in a fixed order).
 */
int ziplm_hessian_accumulate(float *H, const float *X, int d_col, int64_t n_tok, int64_t ldx,
                             int layout, float scale, void *workspace, size_t workspace_bytes,
                             void *stream);
size_t ziplm_hessian_workspace_bytes(int d_col, int64_t n_tok);

/*
 * Dampened inverse (caption of Algorithm 1: H^-1 = (2 X X^T + lambda I)^-1).
 *
 *   lambda = damp_rel * mean(diag H);   Hinv = (H + lambda I)^-1
 *
 * computed as H + lambda I = L L^T (blocked Cholesky), T = L^-1, X0 = T^T T in fp32, followed by
 * one Newton step Hinv = X0 + X0 (I - (H + lambda I) X0) whose residual is formed on the fp64
 * matrix cores: the result is the fp64 inverse of the fp32 H rounded to fp32, as long as fp32
 * arithmetic gets X0 to within a few 1e-4 (conditioning up to about 1e4).  H and Hinv are
 * d_col x d_col fp32 with leading dimension d_col; H is only read, and Hinv may alias H.  Both
 * triangles of Hinv are written, bit-identical.
 * lambda_out_host / info_host (host pointers, each may be NULL): if either is given the call
 * waits for the stream and stores lambda and, in *info_host, 0; or 1 + the index of the first
 * non-positive pivot (-> ZIPLM_ERR_NOT_PD); or -1 when H + lambda I is too ill conditioned for
 * the fp32 factorisation to be refined (-> ZIPLM_ERR_UNSUPPORTED: use more dampening).  The
 * refinement takes a second step when the residual I - (H + lambda I) X the first one starts from
 * has an entry above 2.5e-4 (condition numbers up to about 1e5 need one step and reach a relative
 * error below 5e-7), and is refused when the last step started above 1.5e-3 (a relative error
 * beyond about 1e-5; condition numbers of a few 1e6 and more, where the rounding of an fp32 H
 * already moves its exact inverse by tens of per cent).  Either failure is also
 * marked on the device, for callers that do not wait: every diagonal entry of Hinv is set to
 * NaN, which ziplm_structured_obs_prune reports as ZIPLM_ERR_NOT_PD at its first step.
 */
int ziplm_hinv(const float *H, float *Hinv, int d_col, float damp_rel, float *lambda_out_host,
               int *info_host, void *workspace, size_t workspace_bytes, void *stream);
size_t ziplm_hinv_workspace_bytes(int d_col);

/*
 * Greedy structured OBS pruning (Algorithm 1).
 *
 *   W        d_row x d_col fp32, in/out.  On return the removed columns are exactly zero and
 *            the remaining ones carry the accumulated updates of Eq. 3.
 *   Hinv     d_col x d_col fp32, in/out, symmetric positive definite on the live columns.  On
 *            return the live x live block is the inverse Hessian of the surviving columns
 *            (Eq. 4 applied n_remove times); removed rows and columns are exactly zero.
 *   group_size  columns per structure; d_col % group_size == 0; 1 <= group_size <= 64 in this
 *            build (ZIPLM_ERR_UNSUPPORTED above that).
 *   n_remove number of structures to remove, 0 <= n_remove <= number of live structures.
 *   order_out   int32[n_remove]: index of the structure removed at each step.
 *   err_out     double[n_remove]: its Eq. 2 score at that step (the layer-wise error the removal
 *            adds; the factor convention follows Eq. 2, i.e. no 1/2).
 *   alive_in    optional uint8[d_col/group_size]; 0 marks structures removed by an earlier call
 *            (their columns of W and rows/columns of Hinv are ignored and zeroed on return).
 *   n_snap, snapshot_steps_host, W_snap   optional per-layer database (Section 3.2): after
 *            snapshot_steps_host[i] removals (0..n_remove, host int32 array, read before the
 *            call returns) the masked W is copied to W_snap + i*d_row*d_col.
 *   info_host   optional host int: when given, the call waits for the stream and stores the device's
 *            status word: 0; or 1 + the step at which a block of Hinv was not positive definite
 *            (-> ZIPLM_ERR_NOT_PD); or -1 if a device-side wait gave up after its 4 s limit
 *            (-> ZIPLM_ERR_DEVICE); or -(2 + t) if no live structure was left at step t, i.e. n_remove
 *            exceeds the structures alive under alive_in (-> ZIPLM_ERR_INVALID_ARG, the one argument
 *            error that only the device can see).  After any of the three, order_out and err_out hold
 *            the steps completed so far; W and Hinv are unchanged (single columns) or partly updated
 *            (larger structures), and must not be used.
 *   exchange, exchange_bytes   optional separate area for the words the loop's workgroups wait on
 *            (group_size == 1 only; size from ziplm_prune_exchange_bytes, 256-byte aligned).  NULL: they
 *            live in the workspace.  Results are identical either way; in uncached device memory
 *            (ziplm_exchange_alloc) a store reaches the other workgroups' loads sooner, which makes the
 *            loop about 3% faster.  The area is scratch like the workspace: cleared on entry, and two
 *            calls in flight must not share it.
 *
 * The state is held in fp64 for Hinv and fp32 for W inside the call; scores are reduced in
 * fp64.  Ties in the argmin go to the lowest structure index.  Eq. 3 and Eq. 4 of one step use
 * the rows of Hinv as they were before that step.
 */
int ziplm_structured_obs_prune(float *W, float *Hinv, int d_row, int d_col, int group_size,
                               int n_remove, int32_t *order_out, double *err_out,
                               const uint8_t *alive_in, int n_snap,
                               const int32_t *snapshot_steps_host, float *W_snap,
                               int *info_host, void *exchange, size_t exchange_bytes,
                               void *workspace, size_t workspace_bytes, void *stream);
size_t ziplm_prune_workspace_bytes(int d_row, int d_col, int group_size, int n_snap);

/*
 * Size of a separate exchange area for ziplm_structured_obs_prune (n_layers = 1) or
 * ziplm_structured_obs_prune_batch; 0 when the loop has no use for one (group_size > 1, or a shape
 * that runs on the eager kernel).
 */
size_t ziplm_prune_exchange_bytes(int n_layers, int d_row, int d_col, int group_size);

/*
 * Allocates `bytes` of uncached device memory on the current device for use as an exchange area and
 * stores its address in *exchange_out (host pointer).  The caller owns it.  It is meant to be kept
 * for the life of the process and reused by every call: memory of this kind must not be returned to
 * the driver once a kernel has read it (later allocations have been seen holding wrong values), so
 * the library offers no call that frees it.
 */
int ziplm_exchange_alloc(size_t bytes, void **exchange_out);

/*
 * The same loop for several layers of one shape in one sequence of launches (Section 3.2: every layer
 * is treated independently).  Meant for the layers of a model: their loops are latency bound, whether a
 * sequence of small launches (heads) or one persistent launch (single columns); layers do not interact.
 *
 *   W        n_layers matrices d_row x d_col, layer l at W + l*stride_w (stride_w >= d_row*d_col), in/out
 *   Hinv     n_layers matrices d_col x d_col, layer l at Hinv + l*stride_hinv, in/out
 *   order_out, err_out   [n_layers][n_remove]
 *   W_snap   [n_layers][n_snap][d_row][d_col]; snapshot_steps_host is shared by all layers
 *   info_host   optional host int[n_layers], as in the single-layer call; the return value is
 *            ZIPLM_ERR_NOT_PD / ZIPLM_ERR_DEVICE if any layer reported it (the other layers are complete)
 *
 * 1 <= group_size <= 64 in this build.  Every layer starts with all structures alive.
 * group_size >= 2: one sequence of launches covers all layers; results are identical to n_layers
 * single-layer calls.
 * group_size == 1: the layers are taken up to four at a time; the loops of one such set run side by side
 * in one launch, each on its share of the compute units, and the sets follow one another on the stream
 * (a single loop is bound by the hand-off between its workgroups, so four loops on a quarter of the device each
 * finish in 55% of the time of four loops one after another).  The columns are spread over fewer
 * workgroups than in the single-layer call, so the deferred eliminations are summed in another order: same
 * removal order wherever the scores differ by more than rounding, W, Hinv and err equal to rounding, not bit
 * for bit.  With info_host the call waits for the stream after every set.  exchange: as in the
 * single-layer call, sized by ziplm_prune_exchange_bytes(n_layers, ...).
 */
int ziplm_structured_obs_prune_batch(float *W, float *Hinv, int n_layers, int64_t stride_w,
                                     int64_t stride_hinv, int d_row, int d_col, int group_size,
                                     int n_remove, int32_t *order_out, double *err_out, int n_snap,
                                     const int32_t *snapshot_steps_host, float *W_snap,
                                     int *info_host, void *exchange, size_t exchange_bytes,
                                     void *workspace, size_t workspace_bytes, void *stream);
size_t ziplm_prune_batch_workspace_bytes(int n_layers, int d_row, int d_col, int group_size,
                                         int n_snap);

/*
 * The same greedy loop over single columns (Algorithm 1 with |S| = 1) on the eager kernel: every step
 * reads and writes the whole live state, the O(d_col^2) elimination of Eq. 4 included, exactly as the
 * algorithm is printed.  ziplm_structured_obs_prune uses it for shapes whose per-workgroup state does
 * not fit on chip; this entry point runs it for any shape -- a cross-check of the deferred-update
 * kernel and the baseline its time is quoted against.  Arguments as in ziplm_structured_obs_prune
 * with group_size = 1 and no exchange area.
 */
int ziplm_structured_obs_prune_eager(float *W, float *Hinv, int d_row, int d_col, int n_remove,
                                     int32_t *order_out, double *err_out, const uint8_t *alive_in,
                                     int n_snap, const int32_t *snapshot_steps_host, float *W_snap,
                                     int *info_host, void *workspace, size_t workspace_bytes,
                                     void *stream);
size_t ziplm_prune_eager_workspace_bytes(int d_row, int d_col, int n_snap);

/*
 * Self-test of the single-column loop's bounded waits.  The loop's workgroups wait for one another's
 * candidates (Algorithm 1: the argmin of a step needs every score); every such wait gives up after
 * 4 s, raises the status word, and the launch drains.  This call runs the loop of
 * ziplm_structured_obs_prune (group_size 1, every column to be removed, workspace of that call) with
 * one workgroup held back, so that the others wait for a candidate that never comes.  It takes a
 * little over 4 s and is expected to return ZIPLM_ERR_DEVICE with *info_host = -1 and W, Hinv
 * unchanged; ZIPLM_ERR_UNSUPPORTED for shapes that run on the eager kernel.
 */
int ziplm_selftest_bounded_wait(float *W, float *Hinv, int d_row, int d_col, int32_t *order_out,
                                double *err_out, int *info_host, void *workspace,
                                size_t workspace_bytes, void *stream);

/*
 * Hand-off latency between two workgroups on this device: what the serial chain of Algorithm 1 costs
 * at the very least per removal when the columns are spread over the whole chip (the argmin of a step
 * needs a value from every workgroup).  Workgroup 0 and workgroup `partner` (1..15; workgroup i of the
 * launch runs on XCD i % 8, so 1 is another XCD and 8 the same one) pass a word back and forth
 * `rounds` times with the device-scope store and polling load the loop uses; *us_out_host (host
 * pointer) receives the mean one-way time in microseconds.  Waits for the stream.  workspace: 1 KiB,
 * 256-byte aligned, ordinary or uncached device memory -- the time depends on which.
 */
int ziplm_selftest_handoff_latency(int rounds, int partner, double *us_out_host, void *workspace,
                                   size_t workspace_bytes, void *stream);

/*
 * Error of dropping a whole module ("Pruned structures", Section 3.1: besides heads and
 * feed-forward columns, an entire attention or feed-forward module may be removed).  With every
 * column pruned nothing is left to compensate, so the layer-wise error in the quadratic form of
 * Eq. 2 is
 *
 *   *err_out = tr(W (H + lambda I) W^T) = sum_i W_i (H + lambda I) W_i^T
 *
 * which for H = scale X X^T is scale ||W X||^2 + lambda ||W||^2, and equals the sum of err_out of
 * a ziplm_structured_obs_prune run that removes every structure.  It is also the squared
 * denominator of the prior below.
 * W d_row x d_col and H d_col x d_col (symmetric; the UNdampened Hessian, both triangles), fp32,
 * row-major, only read.  lambda >= 0 is the dampening constant that ziplm_hinv reports.
 * err_out: one DEVICE double.  Products are fp32 matrix-core multiply-accumulates, the final sums
 * fp64 in a fixed order.
 */
int ziplm_module_error(const float *W, const float *H, int d_row, int d_col, float lambda,
                       double *err_out, void *workspace, size_t workspace_bytes, void *stream);
size_t ziplm_module_error_workspace_bytes(int d_row, int d_col);

/*
 * ziplm_module_error for callers that cannot allocate or carry a workspace: code running under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same result bit for bit;
 * the per-tile partial sums go to a scratch array built into the library's device image (32 KiB, one copy
 * on every GPU the library runs on, held until the process ends) instead of a workspace.  The call
 * allocates and frees nothing.
 * Limit: ceil(d_row / 128) * ceil(d_col / 128) <= ziplm_module_error_static_max_tiles() (4096); larger
 * layers get ZIPLM_ERR_UNSUPPORTED and must use ziplm_module_error.
 * All calls on one GPU share that array: calls whose work may overlap in time (different streams without
 * an ordering between them) race on it and must be ordered by the caller.
 */
int ziplm_module_error_static(const float *W, const float *H, int d_row, int d_col, float lambda,
                              double *err_out, void *stream);
int ziplm_module_error_static_max_tiles(void);

/*
 * Prior of the sparsity search (Section 3.2, "Structured SPDY search"):
 * p_s = ||W_s X - W X|| / ||W X|| for the layer after each removal of a greedy run,
 *
 *   prior_out[t] = sqrt((err[0] + ... + err[t]) / *total),   t = 0 .. n-1
 *
 * err: the err_out of ziplm_structured_obs_prune (device, double[n]); the running sum is the
 * layer-wise error of the pruned layer because every intermediate W is the least-squares optimum
 * on its support.  total: one device double, the whole-module error from ziplm_module_error (with
 * the same lambda the pruner's Hinv was built with); a fully dropped layer gets 1.
 * prior_out: device double[n].  n == 0 is a no-op.  *total must be positive and finite; the value
 * is on the device, so a violation cannot be returned as a status: every prior_out[t] is then NaN.
 */
int ziplm_prior(const double *err, int n, const double *total, double *prior_out, void *stream);

/*
 * Host-side search for a per-layer sparsity configuration under a runtime budget (Section 3.2, "Runtime
 * awareness", "Finding the optimal sparsity configuration", "Structured SPDY search").  No device work: every
 * pointer is a HOST pointer.  A configuration picks one level (a pruned version from the per-layer database of
 * a greedy run) per layer; the flat arrays list the levels of layer 0, then of layer 1, ...: n_levels_host[l]
 * entries each, ordered by increasing sparsity.
 *
 * ziplm_search_select: the configuration of least  sum_l cost[l][s_l]  with  sum_l time[l][s_l] <= budget, by
 * dynamic programming on a time axis of `buckets` equal steps (1 .. 2^24).  Times are rounded up to whole steps,
 * so the result always meets the budget in the unrounded times (at the price of leaving up to n_layers steps of
 * it unused).  Equal costs go to the lower level.  choice_out_host[n_layers]; cost_out_host / time_out_host
 * (optional): the sum of the chosen costs / unrounded times.  ZIPLM_ERR_UNSUPPORTED if no configuration fits.
 *
 * ziplm_search_mutate: the outer loop of the structured SPDY search.  cost[l][s] = c_l * prior[l][s] (prior: the
 * p_s of ziplm_prior at the level's number of removals; 0 for the dense level, 1 for a dropped module) with one
 * sensitivity coefficient c_l per layer, all 1 at the start.  n_steps times (the paper: 1000): every coefficient is
 * redrawn with probability mutate_prob (the paper: 0.1) as a uniform number in (0, 1], ziplm_search_select picks the
 * configuration, score(choice, user) rates it (lower is better: the caller evaluates the stitched model), and the
 * trial replaces the incumbent if its score is not worse.  uniform_host[n_steps][n_layers][2]: the caller's
 * uniform numbers in [0, 1) (decision, value), so a run can be reproduced.  Outputs: the best configuration, its
 * coefficients and score (the last two optional).  What the paper leaves to the SPDY method it adapts -- the
 * starting coefficients, the distribution of a redrawn one, the acceptance of equal scores -- is this library's
 * reading.
 */
typedef double (*ziplm_score_fn)(const int32_t *choice, void *user);
int ziplm_search_select(int n_layers, const int32_t *n_levels_host, const double *time_host,
                        const double *cost_host, double budget, int buckets, int32_t *choice_out_host,
                        double *cost_out_host, double *time_out_host);
int ziplm_search_mutate(int n_layers, const int32_t *n_levels_host, const double *time_host,
                        const double *prior_host, double budget, int buckets, int n_steps,
                        double mutate_prob, const double *uniform_host, ziplm_score_fn score, void *user,
                        int32_t *choice_out_host, double *coef_out_host, double *score_out_host);

#ifdef __cplusplus
}
#endif
#endif /* ZIPLM_H */
