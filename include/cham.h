/*
 * cham.h -- C ABI of libcham: the data-parallel core of Adaptive Sampling
 * (Chameleon, arXiv 2001.08743, Sec. 3.3 and Algorithm 1) for AMD MI355X (gfx950).
 *
 * One call of Algorithm 1 takes the candidate configurations s_Theta of a tuning
 * task and the visited configurations v_Theta and returns the configurations to
 * measure.  The library runs that for a batch of independent tasks on one GPU:
 *
 *   cham_kmeans_sweep     k-means for every k of a sweep (Algorithm 1, first loop body)
 *   cham_select_k         threshold test on the loss curve (Algorithm 1, knee exit)
 *   cham_snap_centroids   member configuration nearest to each centroid of the chosen k
 *   cham_synthesize       per-knob mode replacement of redundant / invalid picks and
 *                         dedupe against the visited set (Algorithm 1, second loop)
 *
 * Conventions
 *   - A configuration is one small integer per knob (Sec. 2.2): a uint8 knob index.  Design
 *     spaces whose knobs have more than 256 choices, or more than 32 knobs, go through the
 *     *_u16 entry points at the end of this header.
 *   - X is a structure-of-arrays matrix in DEVICE memory: knob j of row i is X[j*ld + i].
 *     ld >= total rows, ld % 4 == 0, X 4-byte aligned.  All tasks share X; task t owns
 *     rows [task_off[t], task_off[t+1]).
 *   - "DEVICE" pointers are hipMalloc'd (or torch) device memory, "HOST" pointers ordinary
 *     host memory that is read before the call returns.  The caller owns every buffer and
 *     keeps device buffers alive until the stream has run the call.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = default
 *     stream); calls do not synchronise.  Small HOST arrays are read before the call
 *     returns: they travel to the workspace inside the arguments of small staging kernels
 *     launched on that stream (no host buffer has to outlive the call).
 *   - Every function returns CHAM_OK or a negative error; on an argument error nothing
 *     is enqueued and no output is written.  Functions never throw or abort; the only
 *     host memory they may take is a malloc'd table for batches of more than about a
 *     thousand tasks (CHAM_E_NOMEM if that fails).
 *   - The library keeps no state between calls except the code of the last failed HIP call,
 *     which is thread-local (cham_last_hip_error), and the static scratch buffer of
 *     cham_kmeans_sweep_static.
 *   - ks is strictly increasing, 1 <= k <= 256.  Ksum = sum(ks), koff[i] = ks[0]+..+ks[i-1],
 *     k_max = ks[n_k-1].
 *   - Integer outputs are exact and reproducible run to run; floating-point outputs are
 *     IEEE doubles computed in a fixed order (see each function).
 */
#ifndef CHAM_H
#define CHAM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CHAM_OK              0
#define CHAM_E_NULL         (-1)   /* a required pointer is NULL */
#define CHAM_E_BAD_DIM      (-2)   /* d outside [1,32] ([1,64] for *_u16), ld < rows, ld % 4 != 0, misaligned X, n_iter < 0, T < 1 */
#define CHAM_E_BAD_K        (-3)   /* ks empty, not strictly increasing, k < 1 or k > 256; *_u16: k_max too large for d */
#define CHAM_E_BAD_OFFSETS  (-4)   /* task_off not non-decreasing from >= 0, a task larger than 2^23 rows */
#define CHAM_E_CARD         (-5)   /* a cardinality is 0 or above 256 (above 16384 for *_u16) */
#define CHAM_E_WORKSPACE    (-6)   /* workspace NULL or smaller than cham_*_workspace_bytes says */
#define CHAM_E_HIP          (-7)   /* a HIP runtime call failed; see cham_last_hip_error() */
#define CHAM_E_BAD_FLAG     (-8)   /* unknown bits in flags / unknown init_mode */
#define CHAM_E_NOMEM        (-9)   /* host memory for the call's small tables could not be had */
#define CHAM_E_TOO_LARGE    (-10)  /* cham_kmeans_sweep_static: the input needs more scratch than the static buffer holds */

/* values of out_flag (cham_synthesize) */
#define CHAM_OUT_EMPTY   0   /* cluster has no member (or index >= chosen k) */
#define CHAM_OUT_KEPT    1   /* the cluster's pick is valid and not visited: kept as is */
#define CHAM_OUT_SYNTH   2   /* pick replaced by the per-knob mode of the cluster */
#define CHAM_OUT_DROPPED 3   /* pick flagged and no usable replacement exists */

/* flags of cham_kmeans_sweep / cham_snap_centroids */
#define CHAM_F_FORCE_EXACT   1   /* evaluate every distance in double (slow; verification aid) */
#define CHAM_F_STREAMING     2   /* force the multi-workgroup-per-task path */
#define CHAM_F_RESIDENT      4   /* force the one-workgroup-per-(task,k) path */
#define CHAM_F_NO_MFMA       8   /* never use the matrix-core distance path */
#define CHAM_F_VALUES_BELOW_2048 16  /* *_u16 sweeps: the caller promises that every knob value is below 2048 (as it
                                        is whenever every cardinality is at most 2048); tasks of at most 2048 rows
                                        with k <= 32 (4096 rows and k <= 64 up to 31 knobs) then run on the
                                        matrix cores.  A value of 2048 or more found on the way gives status 4
                                        for every (task, k) and zero outputs.  Ignored by the byte entry points. */

int32_t     cham_version(void);
const char *cham_strerror(int32_t code);
/* Last HIP error code seen by this thread's library calls (0 = none). */
int32_t     cham_last_hip_error(void);

/* Bytes of DEVICE workspace cham_kmeans_sweep needs for these arguments (all HOST),
 * or a negative error code. */
int64_t cham_sweep_workspace_bytes(int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                                   const int32_t *ks, int32_t n_k, int32_t n_iter, int32_t flags);

/*
 * K-means sweep (Algorithm 1, "K-means.run(s_Theta, k)" for every k; Sec. 3.3: centroids and
 * the L2 loss per number of clusters).  The whole list ks is run (no early exit; the knee
 * test is cham_select_k).
 *
 * For each task t and each k = ks[ki]:
 *   start:  init_mode 0: the first k distinct rows of the task, in row order;
 *           init_mode 1: init_centroids[(t*Ksum + koff[ki] + c)*d + j]  (DEVICE, doubles);
 *   n_iter times: label every row with its nearest centroid (squared Euclidean distance on
 *           the raw knob indices, lowest cluster index on ties); move every non-empty
 *           centroid to the mean of its rows (an empty cluster keeps its centroid);
 *   then one more labelling with the final centroids, which fixes labels, counts and loss.
 * Distances are screened in fp32 with a proven error bound; every decision inside that
 * bound is re-evaluated in double as sum_j ((double)x_j - mu_j)^2 (j ascending, no fused
 * multiply-add), so labels are those of a plain double-precision implementation.
 * Cluster sums are integers; centroids are (double)sum / (double)count.
 *
 * Outputs (all DEVICE):
 *   centroids [T][Ksum][d] double  final centroids, row (t,ki,c) at t*Ksum + koff[ki] + c
 *   counts    [T][Ksum]    int32   final cluster sizes
 *   inertia   [T][n_k]     double  loss: sum over rows of the squared distance to the row's
 *                                  final centroid (double terms, fixed summation tree)
 *   status    [T][n_k]     int32   0 ok; 1 = task has fewer than k distinct rows (init_mode 0):
 *                                  centroids, counts, loss and labels of that (t,k) are zero
 *                                  (4: see CHAM_F_VALUES_BELOW_2048)
 *   labels    [n_k][ld]    uint8   final labels per k (optional, may be NULL)
 *   inertia_trace [T][n_k][n_iter+1] double  loss seen by every labelling pass (optional); a
 *                                  kernel that stops at the fixed point (see cham_sweep_passes)
 *                                  repeats the final loss for the passes it did not run
 * workspace: DEVICE scratch of at least cham_sweep_workspace_bytes(...) bytes, 256-byte aligned.
 */
int32_t cham_kmeans_sweep(const uint8_t *X, int64_t ld, int32_t d,
                          const int64_t *task_off, int32_t T,
                          const int32_t *ks, int32_t n_k,
                          int32_t n_iter, int32_t init_mode, const double *init_centroids,
                          double *centroids, int32_t *counts, double *inertia, int32_t *status,
                          uint8_t *labels, double *inertia_trace,
                          void *workspace, int64_t workspace_bytes, int32_t flags, void *stream);

/*
 * Which kernel family cham_kmeans_sweep runs for these arguments (all HOST), or a negative error:
 * the choice depends only on d, the largest task, the largest k and flags (Sec. 3.3's k-means,
 * "K-means.run" of Algorithm 1, is the same computation on every path).
 *   CHAM_PATH_RESIDENT_MFMA    one workgroup per (task, k), distances on the matrix cores
 *                              (d <= 31, tasks of at most 4096 rows, k <= 64)
 *   CHAM_PATH_STREAM_MFMA      several workgroups per (task, k), one launch pair per pass (d <= 31)
 *   CHAM_PATH_RESIDENT_VECTOR  one workgroup per (task, k), vector ALU
 * cham_sweep_path_kernel gives the name of the family's dominant kernel (a static string).
 */
#define CHAM_PATH_RESIDENT_MFMA   0
#define CHAM_PATH_STREAM_MFMA     1
#define CHAM_PATH_RESIDENT_VECTOR 2
int32_t     cham_sweep_path(int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                            const int32_t *ks, int32_t n_k, int32_t flags);
const char *cham_sweep_path_kernel(int32_t path);

/*
 * Labelling passes the last sweep that used `workspace` really ran, per (task, k): passes
 * [T][n_k] int32 DEVICE.  Algorithm 1's K-means.run is n_iter update steps plus the final
 * labelling, n_iter + 1 passes; a pass that changes no label leaves sums, centroids and every
 * later pass unchanged, so a kernel may stop there with the results of the full iteration
 * (the matrix-core resident kernel does; the figure is what a throughput in executed distance
 * evaluations is computed from).  0 for a (task, k) that was skipped (status 1 or 3).  The
 * arguments other than passes are those of the sweep call; works for both knob widths.
 */
int32_t cham_sweep_passes(const void *workspace, int64_t workspace_bytes, int64_t ld, int32_t d,
                          const int64_t *task_off, int32_t T, const int32_t *ks, int32_t n_k, int32_t flags,
                          int32_t *passes, void *stream);

/*
 * cham_kmeans_sweep for callers that cannot allocate device memory or pass a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments
 * (minus the workspace), same results bit for bit, same kernels; the scratch memory is a static
 * device array of CHAM_STATIC_SCRATCH_BYTES inside the library, one per GPU, held until the
 * process ends.  The call allocates nothing, on the device or on the host.
 *   - Limit: cham_sweep_workspace_bytes(...) for the arguments must not exceed
 *     CHAM_STATIC_SCRATCH_BYTES and T + n_k must stay below about a thousand (the host tables
 *     live on the stack); beyond: CHAM_E_TOO_LARGE, nothing is enqueued.
 *   - The array's device address is looked up on the first call on each GPU (with that GPU
 *     current); cham_static_init() does the lookup ahead of time, e.g. before a graph capture.
 *   - All calls on one GPU share that GPU's array, whatever the stream: calls that overlap in
 *     time on one GPU race.  Nothing in it has to be cleared between calls: every word a call
 *     reads it has written first.
 */
#define CHAM_STATIC_SCRATCH_BYTES (8 * 1024 * 1024)
int32_t cham_static_init(void);
int32_t cham_kmeans_sweep_static(const uint8_t *X, int64_t ld, int32_t d,
                                 const int64_t *task_off, int32_t T,
                                 const int32_t *ks, int32_t n_k,
                                 int32_t n_iter, int32_t init_mode, const double *init_centroids,
                                 double *centroids, int32_t *counts, double *inertia, int32_t *status,
                                 uint8_t *labels, double *inertia_trace, int32_t flags, void *stream);

/*
 * K-means sweep that stops at the knee, the loop of Algorithm 1 as printed: for k in the list,
 * run k-means, and leave the loop at the first k with threshold * loss(k) >= previous_loss.
 * The list is run in chunks of `chunk` consecutive entries of ks (all tasks at once); after every
 * chunk the knee test runs on the device and the later chunks skip the tasks that have stopped,
 * so at most chunk - 1 values of k beyond the knee are computed per task.  Arguments and outputs
 * as for cham_kmeans_sweep, plus
 *   threshold            the factor of the test (the paper's value is 2.5)
 *   chunk                >= 1; values above n_k mean one chunk (the whole list)
 *   chosen_idx [T]       DEVICE int32: index into ks of the k the loop stopped at (the last usable
 *                        k if it never stopped, -1 if none is usable), as cham_select_k on the
 *                        full curve would give
 *   status               3 = not computed: the task had stopped before this k (outputs of that
 *                        (t,k) are zero); every entry up to and including the chosen one is 0 or 1
 * Every computed entry is identical to the one cham_kmeans_sweep produces.  Workspace:
 * cham_sweep_knee_workspace_bytes(...) bytes.  Errors: as cham_kmeans_sweep; CHAM_E_BAD_K for
 * chunk < 1, CHAM_E_NULL for a missing chosen_idx.
 */
int64_t cham_sweep_knee_workspace_bytes(int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                                        const int32_t *ks, int32_t n_k, int32_t n_iter, int32_t flags);
int32_t cham_kmeans_sweep_knee(const uint8_t *X, int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                               const int32_t *ks, int32_t n_k, int32_t n_iter, int32_t init_mode,
                               const double *init_centroids, double threshold, int32_t chunk,
                               double *centroids, int32_t *counts, double *inertia, int32_t *status,
                               int32_t *chosen_idx, uint8_t *labels, double *inertia_trace,
                               void *workspace, int64_t workspace_bytes, int32_t flags, void *stream);

/*
 * Knee selection (Algorithm 1: previous_loss = infinity; for each k in order: stop at the
 * first k with threshold * loss(k) >= previous_loss, and that k is the result; if no k
 * stops the loop the last k is the result).  Entries with status != 0 are skipped as if
 * absent.  chosen_idx[t] (DEVICE int32 [T]) receives the index into ks, -1 if none usable.
 * The paper's threshold is 2.5 (hyper-parameter table, threshold_meta).
 */
int32_t cham_select_k(const double *inertia, const int32_t *status, int32_t T, int32_t n_k,
                      double threshold, int32_t *chosen_idx, void *stream);
/* The same rule on HOST arrays (status may be NULL); returns the index or -1. */
int32_t cham_select_k_host(const double *curve, const int32_t *status, int32_t n_k, double threshold);

int64_t cham_snap_workspace_bytes(int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                                  const int32_t *ks, int32_t n_k);
/*
 * Representatives of the chosen clustering (Sec. 3.3: centroids stand for their clusters; a
 * centroid is real-valued, so the representative is the member configuration nearest to it).
 * For task t with k* = ks[chosen_idx[t]] and its centroids from cham_kmeans_sweep:
 *   labels_sel [ld] uint8          nearest-centroid label of every row (same rule as the sweep)
 *   pick_row [T][k_max] int32      row (relative to the task's first row) of the member with the
 *                                  smallest distance to centroid c, lowest row on ties;
 *                                  -1 for an empty cluster and for c >= k*
 *   pick_cfg [T][k_max][d] uint8   that row's knob values (zeros where pick_row = -1)
 * chosen_idx = -1 leaves the task's picks at -1.  All pointers DEVICE except task_off, ks.
 */
int32_t cham_snap_centroids(const uint8_t *X, int64_t ld, int32_t d,
                            const int64_t *task_off, int32_t T, const int32_t *ks, int32_t n_k,
                            const int32_t *chosen_idx, const double *centroids,
                            uint8_t *labels_sel, int32_t *pick_row, uint8_t *pick_cfg,
                            void *workspace, int64_t workspace_bytes, int32_t flags, void *stream);

int64_t cham_synth_workspace_bytes(int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                                   const int32_t *ks, int32_t n_k);
/*
 * Sample Synthesis and dedupe (Algorithm 1, second loop; Sec. 3.3 "most frequent = mode,
 * non-invalid choice for each knob").
 *   cards [T][d] HOST uint16     cardinality of each knob.  Precondition: every value of X is below its
 *                                knob's cardinality; a value that is not is never counted for the mode
 *   valid [ld] DEVICE uint8      1 = valid configuration, 0 = known invalid; NULL = all valid
 *   visited DEVICE uint64        hashes (cham_hash_config) of measured configurations, sorted
 *                                ascending; membership is by hash
 *   task_salt [T] HOST uint64    hash salt per task; NULL = task index
 * A pick is flagged if its row is invalid or its hash is in visited.  Unflagged picks are
 * KEPT.  Flagged clusters, in ascending order, are replaced by the per-knob mode over the
 * cluster's valid members (smallest value on ties); the replacement is DROPPED if the cluster
 * has no valid member, if its hash is visited, if it equals a kept pick or a replacement
 * accepted for a lower cluster; otherwise SYNTH.
 *   out_cfg [T][k_max][d] uint8, out_flag [T][k_max] uint8 (CHAM_OUT_*), out_count [T] int32
 *   (number of KEPT + SYNTH); rows of out_cfg that are not KEPT / SYNTH are zero.
 */
int32_t cham_synthesize(const uint8_t *X, int64_t ld, int32_t d,
                        const int64_t *task_off, int32_t T, const uint16_t *cards,
                        const uint8_t *valid, const int32_t *ks, int32_t n_k,
                        const int32_t *chosen_idx, const uint8_t *labels_sel,
                        const int32_t *pick_row, const uint8_t *pick_cfg,
                        const uint64_t *visited, int64_t n_visited, const uint64_t *task_salt,
                        uint8_t *out_cfg, uint8_t *out_flag, int32_t *out_count,
                        void *workspace, int64_t workspace_bytes, void *stream);

/*
 * Visited set kept on the device across calls (the outer loop of the search calls the sampling
 * step again and again with a growing set of measured configurations; Sec. 3.1 / 4.1, 16
 * iterations per task): an open-addressing table of `slots` uint64 (a power of two, >= 2; DEVICE,
 * 8-byte aligned, caller-owned, slots * 8 bytes).  Membership is by the same 64-bit hash as in
 * cham_synthesize; an empty slot holds all ones and the one hash with that value is stored as
 * the value below it.  Keep the load below about one half.
 *   cham_visited_table_clear            empties the table
 *   cham_visited_table_insert_hashes    inserts n hashes (DEVICE); duplicates are no-ops
 *   cham_visited_table_insert_configs   hashes and inserts rows of cfgs (DEVICE row-major [n][d]):
 *                                       row i iff flags is NULL or flags[i] is CHAM_OUT_KEPT or
 *                                       CHAM_OUT_SYNTH (so out_cfg / out_flag of cham_synthesize,
 *                                       n = T * k_max, go in directly); its salt is
 *                                       salts[i / rows_per_salt] (DEVICE; NULL: i / rows_per_salt)
 *   overflow (DEVICE int32, may be NULL) is set to 1 if an insert finds no free slot; it is never
 *   cleared by the library.
 *   cham_synthesize_table               cham_synthesize with the table in place of the sorted array
 * Errors: CHAM_E_NULL for a missing table / input, CHAM_E_BAD_DIM for slots not a power of two,
 * a misaligned table, n < 0, d outside [1,32], rows_per_salt < 1.
 */
int32_t cham_visited_table_clear(uint64_t *table, int64_t slots, void *stream);
int32_t cham_visited_table_insert_hashes(uint64_t *table, int64_t slots, const uint64_t *hashes, int64_t n,
                                         int32_t *overflow, void *stream);
int32_t cham_visited_table_insert_configs(uint64_t *table, int64_t slots, const uint8_t *cfgs, int64_t n, int32_t d,
                                          const uint8_t *flags, const uint64_t *salts, int64_t rows_per_salt,
                                          int32_t *overflow, void *stream);
int32_t cham_synthesize_table(const uint8_t *X, int64_t ld, int32_t d,
                              const int64_t *task_off, int32_t T, const uint16_t *cards,
                              const uint8_t *valid, const int32_t *ks, int32_t n_k,
                              const int32_t *chosen_idx, const uint8_t *labels_sel,
                              const int32_t *pick_row, const uint8_t *pick_cfg,
                              const uint64_t *table, int64_t slots, const uint64_t *task_salt,
                              uint8_t *out_cfg, uint8_t *out_flag, int32_t *out_count,
                              void *workspace, int64_t workspace_bytes, void *stream);

/*
 * Configuration updater of the exploration step that feeds the sampling step (Sec. 3.2, the
 * action figure: the agent emits increment / decrement / stay per knob, the updater applies it;
 * hyper-parameter table: 128 episodes of up to 500 steps).  The policy network is not part of this
 * library: the actions are an input.
 *   theta   DEVICE uint8 [B][d]           configurations, updated in place through n_steps steps:
 *                                         theta <- clip(theta + a, 0, card - 1) per knob
 *   actions DEVICE int8 [n_steps][B][d]   each -1, 0 or +1
 *   cards   DEVICE uint16 [d]             cardinalities (one design space for the whole batch)
 *   seen_table / slots                    table as for cham_visited_table_* (NULL: no bookkeeping);
 *                                         every configuration reached is entered under `salt`
 *   unique_rows DEVICE uint8 [capacity][d], n_unique DEVICE int32 (caller zeroes it, or keeps it
 *                                         running across calls): the distinct configurations in
 *                                         the order in which they were first entered (unspecified
 *                                         between threads) - the set S_Theta handed to the
 *                                         sampling step
 *   overflow DEVICE int32 (may be NULL)   set to 1 if the table or the list is full
 * Errors: CHAM_E_NULL, CHAM_E_BAD_DIM (B < 0, d outside [1,32], n_steps < 0, bad table).
 */
int32_t cham_update_configs(uint8_t *theta, const int8_t *actions, int64_t B, int32_t d, int32_t n_steps,
                            const uint16_t *cards, uint64_t salt, uint64_t *seen_table, int64_t slots,
                            uint8_t *unique_rows, int64_t capacity, int32_t *n_unique, int32_t *overflow,
                            void *stream);

/*
 * Configuration hash used for the visited set: 64-bit FNV-1a over the d knob values, the
 * offset basis first XORed with salt * 0x9E3779B97F4A7C15 (mod 2^64).  salt 0 gives plain
 * FNV-1a.  cfg is HOST memory.
 */
uint64_t cham_hash_config(const uint8_t *cfg, int32_t d, uint64_t salt);
/* Batch version on the device: rows is DEVICE row-major [n][d]; salts DEVICE [n] or NULL
 * (then salt_all is used for every row); out DEVICE [n]. */
int32_t cham_hash_rows(const uint8_t *rows, int64_t n, int32_t d, const uint64_t *salts,
                       uint64_t salt_all, uint64_t *out, void *stream);

/*
 * Two-byte knobs.  The design spaces of Sec. 2 are products of the knobs' choice lists (10^10
 * points and more); a split knob of a large loop alone has hundreds of choices, and templates
 * with many loops have more than 32 knobs.  Every entry point above that reads or writes
 * configurations has a twin that takes uint16 knob values and up to 64 knobs; what is computed,
 * every rule, tie-break, output layout and error code is that of the function without the
 * suffix, with these differences:
 *   - X is uint16 [d][ld] (DEVICE), 8-byte aligned, ld % 4 == 0; pick_cfg, out_cfg, cfgs and
 *     rows are uint16; 1 <= d <= 64; knob values up to 65535.
 *   - The sweep and the snap run one workgroup per (task, k) whatever the task size (built for
 *     tasks of up to some ten thousand rows; larger ones are correct but slow).  Cluster sums
 *     are 64-bit integers.  flags: CHAM_F_FORCE_EXACT is honoured, CHAM_F_RESIDENT is accepted
 *     (it names what these paths do anyway), CHAM_F_STREAMING gives CHAM_E_BAD_FLAG.
 *   - Without CHAM_F_VALUES_BELOW_2048 the sweep runs on the vector ALU.  With it (values below
 *     2048 are exact in the f16 operands of the matrix cores; Sec. 3.3's k-means is the same
 *     computation either way, and the results are the same bit for bit) the sweep runs the
 *     matrix-core kernel when d <= 63 and either d <= 31, tasks have at most 4096 rows and
 *     k <= 64, or tasks have at most 2048 rows and k <= 32; otherwise, and under
 *     CHAM_F_FORCE_EXACT or CHAM_F_NO_MFMA, the flag changes nothing.  cham_sweep_path_u16 tells
 *     which one a call runs.  The promise is checked on the device: a value of 2048 or more
 *     makes every (task, k) of the call report status 4 with zero outputs.
 *   - k_max * (20 * dp + 20) + 4 * dp + 192 must not exceed 160 KiB, dp = d rounded up to a
 *     multiple of 8 (k_max up to 256 for d <= 24, 247 for d <= 32, 199 for d <= 40, 166 for
 *     d <= 48, 143 for d <= 56, 125 for d <= 64); beyond that: CHAM_E_BAD_K, also from the
 *     sweep's workspace queries.
 *   - cham_synthesize*_u16: cardinalities up to 16384 (the value histogram of one knob of one
 *     cluster has to fit in LDS); above: CHAM_E_CARD.
 *   - The hash takes one FNV-1a step per knob value, the whole value in the step: equal to the
 *     byte hash for a configuration whose values are all below 256, so a visited set can be
 *     shared between the two families.
 */
int64_t cham_sweep_workspace_bytes_u16(int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                                       const int32_t *ks, int32_t n_k, int32_t n_iter, int32_t flags);
int32_t cham_sweep_path_u16(int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                            const int32_t *ks, int32_t n_k, int32_t flags);
int32_t cham_kmeans_sweep_u16(const uint16_t *X, int64_t ld, int32_t d,
                              const int64_t *task_off, int32_t T,
                              const int32_t *ks, int32_t n_k,
                              int32_t n_iter, int32_t init_mode, const double *init_centroids,
                              double *centroids, int32_t *counts, double *inertia, int32_t *status,
                              uint8_t *labels, double *inertia_trace,
                              void *workspace, int64_t workspace_bytes, int32_t flags, void *stream);
int64_t cham_sweep_knee_workspace_bytes_u16(int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                                            const int32_t *ks, int32_t n_k, int32_t n_iter, int32_t flags);
int32_t cham_kmeans_sweep_knee_u16(const uint16_t *X, int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                                   const int32_t *ks, int32_t n_k, int32_t n_iter, int32_t init_mode,
                                   const double *init_centroids, double threshold, int32_t chunk,
                                   double *centroids, int32_t *counts, double *inertia, int32_t *status,
                                   int32_t *chosen_idx, uint8_t *labels, double *inertia_trace,
                                   void *workspace, int64_t workspace_bytes, int32_t flags, void *stream);
int64_t cham_snap_workspace_bytes_u16(int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                                      const int32_t *ks, int32_t n_k);
int32_t cham_snap_centroids_u16(const uint16_t *X, int64_t ld, int32_t d,
                                const int64_t *task_off, int32_t T, const int32_t *ks, int32_t n_k,
                                const int32_t *chosen_idx, const double *centroids,
                                uint8_t *labels_sel, int32_t *pick_row, uint16_t *pick_cfg,
                                void *workspace, int64_t workspace_bytes, int32_t flags, void *stream);
int64_t cham_synth_workspace_bytes_u16(int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                                       const int32_t *ks, int32_t n_k);
int32_t cham_synthesize_u16(const uint16_t *X, int64_t ld, int32_t d,
                            const int64_t *task_off, int32_t T, const uint16_t *cards,
                            const uint8_t *valid, const int32_t *ks, int32_t n_k,
                            const int32_t *chosen_idx, const uint8_t *labels_sel,
                            const int32_t *pick_row, const uint16_t *pick_cfg,
                            const uint64_t *visited, int64_t n_visited, const uint64_t *task_salt,
                            uint16_t *out_cfg, uint8_t *out_flag, int32_t *out_count,
                            void *workspace, int64_t workspace_bytes, void *stream);
int32_t cham_synthesize_table_u16(const uint16_t *X, int64_t ld, int32_t d,
                                  const int64_t *task_off, int32_t T, const uint16_t *cards,
                                  const uint8_t *valid, const int32_t *ks, int32_t n_k,
                                  const int32_t *chosen_idx, const uint8_t *labels_sel,
                                  const int32_t *pick_row, const uint16_t *pick_cfg,
                                  const uint64_t *table, int64_t slots, const uint64_t *task_salt,
                                  uint16_t *out_cfg, uint8_t *out_flag, int32_t *out_count,
                                  void *workspace, int64_t workspace_bytes, void *stream);
int32_t cham_visited_table_insert_configs_u16(uint64_t *table, int64_t slots, const uint16_t *cfgs, int64_t n,
                                              int32_t d, const uint8_t *flags, const uint64_t *salts,
                                              int64_t rows_per_salt, int32_t *overflow, void *stream);
uint64_t cham_hash_config_u16(const uint16_t *cfg, int32_t d, uint64_t salt);
int32_t cham_hash_rows_u16(const uint16_t *rows, int64_t n, int32_t d, const uint64_t *salts,
                           uint64_t salt_all, uint64_t *out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* CHAM_H */
