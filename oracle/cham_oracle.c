/*
 * cham_oracle.c -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * Plain, slow, double-precision CPU statement of what the Adaptive Sampling
 * hot path computes (paper Sec. 3.3 and Algorithm 1):
 *   k-means over integer knob vectors for every k of a sweep, the "L2 loss"
 *   per k, threshold selection of k (knee), the member closest to each
 *   centroid, the per-knob mode of a cluster for redundant / invalid picks,
 *   and the membership test against the visited set.
 * Only tests, the smoke check and the bench's cpu_baseline leg may call it.
 * It shares no code, header, table or helper with the GPU library.
 *
 * Arithmetic: IEEE double, no fused multiply-add (build with
 * -ffp-contract=off), loops in the order written.  Rows are row-major
 * knob_t [n][d]; knob values are non-negative integers (indices into each
 * knob's list of choices; Sec. 2: a design space is the product of such lists,
 * and a split-factor knob can have hundreds of choices), held in 16 bits.
 *
 * Where the paper is silent the readings are (each repeated at its function):
 *   - feature space: raw knob indices, unscaled squared Euclidean distance;
 *   - "L2 loss": sum over rows of the squared distance to the assigned
 *     centroid, after one extra assignment with the final centroids;
 *   - initial centroids: the first k distinct rows in row order;
 *   - a fixed number of Lloyd steps, no tolerance, no restarts;
 *   - a cluster that loses all members keeps its previous centroid;
 *   - every tie goes to the smallest index (cluster, row, knob value).
 *
 * Pins (tests/test_oracle_*.py): brute-force optimal partitions on tiny
 * inputs, the k = 1 closed form (N * population variance), zero loss when
 * k equals the number of distinct rows, monotone loss over Lloyd steps,
 * conservation of counts and sums, metamorphic relations, a library Lloyd
 * run from the same start, hand-worked knee / snap / mode / dedupe cases,
 * published FNV-1a test vectors for the hash.
 * Full-size workloads (1M rows; 256 tasks) have no pin beyond these:
 * parity unpinned there except through the small-case pins.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef uint16_t knob_t;

enum { ORC_EMPTY = 0, ORC_KEPT = 1, ORC_SYNTH = 2, ORC_DROPPED = 3 };

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Squared Euclidean distance between an integer row and a real centroid,
 * knobs in ascending order (Sec. 3.3: clustering of configurations; the
 * distance itself is the k-means one). */
static double sqdist(const knob_t *x, const double *mu, int d)
{
    double s = 0.0;
    for (int j = 0; j < d; ++j) {
        double t = (double)x[j] - mu[j];
        s = s + t * t;
    }
    return s;
}

/* Nearest centroid of one row; ties go to the smallest cluster index. */
static int nearest(const knob_t *x, const double *mu, int k, int d, double *dmin)
{
    int best = 0;
    double bd = sqdist(x, mu, d);
    for (int c = 1; c < k; ++c) {
        double v = sqdist(x, mu + (size_t)c * d, d);
        if (v < bd) { bd = v; best = c; }
    }
    *dmin = bd;
    return best;
}

/* Indices of the first kmax distinct rows, scanning rows in order; a row equal
 * to one already taken is skipped.  Returns how many were found (<= kmax).
 * (The paper does not say how k-means is started; this is the benchmark's rule.) */
int orc_first_distinct(const knob_t *x, int64_t n, int d, int kmax, int64_t *rows_out)
{
    int found = 0;
    for (int64_t i = 0; i < n && found < kmax; ++i) {
        int dup = 0;
        for (int q = 0; q < found && !dup; ++q)
            if (memcmp(x + (size_t)rows_out[q] * d, x + (size_t)i * d, sizeof(knob_t) * (size_t)d) == 0) dup = 1;
        if (!dup) rows_out[found++] = i;
    }
    return found;
}

/* One assignment pass: label and distance of every row (rows are independent). */
static void assign_all(const knob_t *x, int64_t n, int d, int k, const double *mu,
                       int32_t *lab, double *dmin)
{
#pragma omp parallel for schedule(static) if (n >= 32768)
    for (int64_t i = 0; i < n; ++i)
        lab[i] = nearest(x + (size_t)i * d, mu, k, d, &dmin[i]);
}

static double sum_in_order(const double *v, int64_t n)
{
    double s = 0.0;
    for (int64_t i = 0; i < n; ++i) s = s + v[i];
    return s;
}

/* K-means for one k (Algorithm 1, the K-means.run call): n_iter times
 * { assign every row to its nearest centroid; move every non-empty centroid to
 * the mean of its rows }, then one more assignment that fixes the labels, the
 * cluster sizes and the loss.  mu holds the start on entry and the final
 * centroids on return.  trace (optional, n_iter + 1 values) receives the loss
 * seen by every assignment pass; the last one is the returned loss. */
void orc_kmeans(const knob_t *x, int64_t n, int d, int k, int n_iter, double *mu,
                int64_t *counts, int32_t *labels, double *inertia, double *trace)
{
    double *dmin = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
    int64_t *S = (int64_t *)malloc(sizeof(int64_t) * (size_t)k * d);
    int64_t *cnt = (int64_t *)malloc(sizeof(int64_t) * (size_t)k);
    for (int it = 0; it < n_iter; ++it) {
        assign_all(x, n, d, k, mu, labels, dmin);
        if (trace) trace[it] = sum_in_order(dmin, n);
        memset(S, 0, sizeof(int64_t) * (size_t)k * d);
        memset(cnt, 0, sizeof(int64_t) * (size_t)k);
        for (int64_t i = 0; i < n; ++i) {
            int c = labels[i];
            cnt[c] += 1;
            for (int j = 0; j < d; ++j) S[(size_t)c * d + j] += x[(size_t)i * d + j];
        }
        for (int c = 0; c < k; ++c) {
            if (cnt[c] == 0) continue;            /* empty cluster keeps its centroid */
            for (int j = 0; j < d; ++j)
                mu[(size_t)c * d + j] = (double)S[(size_t)c * d + j] / (double)cnt[c];
        }
    }
    assign_all(x, n, d, k, mu, labels, dmin);
    memset(cnt, 0, sizeof(int64_t) * (size_t)k);
    for (int64_t i = 0; i < n; ++i) cnt[labels[i]] += 1;
    for (int c = 0; c < k; ++c) counts[c] = cnt[c];
    *inertia = sum_in_order(dmin, n);
    if (trace) trace[n_iter] = *inertia;
    free(dmin); free(S); free(cnt);
}

/* The sweep over k (Algorithm 1's for-loop, run in full: no early break) for a
 * batch of independent tasks.  Task t owns rows [task_off[t], task_off[t+1]).
 * Outputs, with Ksum = sum of ks and koff = running sum of ks:
 *   centroids [T][Ksum][d]   row (t, ki, c) at (t*Ksum + koff[ki] + c)
 *   counts    [T][Ksum]      final cluster sizes
 *   inertia   [T][n_k]       loss per k
 *   status    [T][n_k]       0 ok, 1 = the task has fewer than k distinct rows
 *                            (then centroids, counts and loss of that k are zero)
 *   labels    [n_k][N_total] final labels (optional)
 *   trace     [T][n_k][n_iter+1] (optional)
 * init_mode 0: centroids start at the first k distinct rows;
 * init_mode 1: they start at init[...] (same layout as centroids). */
void orc_sweep(const knob_t *x, int d, const int64_t *task_off, int T, const int32_t *ks,
               int n_k, int n_iter, int init_mode, const double *init, double *centroids,
               int64_t *counts, double *inertia, int32_t *status, int32_t *labels,
               double *trace)
{
    int64_t Ksum = 0, n_total = task_off[T];
    int kmax = 0;
    int64_t *koff = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n_k + 1));
    for (int i = 0; i < n_k; ++i) { koff[i] = Ksum; Ksum += ks[i]; if (ks[i] > kmax) kmax = ks[i]; }
    koff[n_k] = Ksum;
    int64_t *first = (int64_t *)malloc(sizeof(int64_t) * (size_t)T * kmax);
    int *nfirst = (int *)malloc(sizeof(int) * (size_t)T);
    int64_t nmax = 0;
    for (int t = 0; t < T; ++t) {
        int64_t n = task_off[t + 1] - task_off[t];
        if (n > nmax) nmax = n;
        nfirst[t] = orc_first_distinct(x + (size_t)task_off[t] * d, n, d, kmax,
                                       first + (size_t)t * kmax);
    }
    int64_t units = (int64_t)T * n_k;
    int outer_parallel = 1;
#ifdef _OPENMP
    if (units < 2 * (int64_t)omp_get_max_threads() && nmax >= 32768) outer_parallel = 0;
#endif
    /* units in descending-k order so that dynamic scheduling balances */
#pragma omp parallel for schedule(dynamic, 1) if (outer_parallel)
    for (int64_t u = 0; u < units; ++u) {
        int ki = n_k - 1 - (int)(u / T);
        int t = (int)(u % T);
        int k = ks[ki];
        int64_t r0 = task_off[t], n = task_off[t + 1] - task_off[t];
        const knob_t *xt = x + (size_t)r0 * d;
        double *mu = centroids + ((size_t)t * Ksum + koff[ki]) * d;
        int64_t *cn = counts + (size_t)t * Ksum + koff[ki];
        size_t slot = (size_t)t * n_k + ki;
        int32_t *lab = labels ? labels + (size_t)ki * n_total + r0
                              : (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
        double *tr = trace ? trace + slot * (size_t)(n_iter + 1) : NULL;
        if (init_mode == 0 && nfirst[t] < k) {
            status[slot] = 1;
            inertia[slot] = 0.0;
            memset(mu, 0, sizeof(double) * (size_t)k * d);
            memset(cn, 0, sizeof(int64_t) * (size_t)k);
            if (labels) memset(lab, 0, sizeof(int32_t) * (size_t)n);
            if (tr) memset(tr, 0, sizeof(double) * (size_t)(n_iter + 1));
        } else {
            status[slot] = 0;
            if (init_mode == 0) {
                for (int c = 0; c < k; ++c)
                    for (int j = 0; j < d; ++j)
                        mu[(size_t)c * d + j] =
                            (double)xt[(size_t)first[(size_t)t * kmax + c] * d + j];
            } else {
                memcpy(mu, init + ((size_t)t * Ksum + koff[ki]) * d, sizeof(double) * (size_t)k * d);
            }
            orc_kmeans(xt, n, d, k, n_iter, mu, cn, lab, &inertia[slot], tr);
        }
        if (!labels) free(lab);
    }
    free(koff); free(first); free(nfirst);
}

/* Threshold-based choice of k (Algorithm 1: previous_loss starts at infinity;
 * walking the sweep in order, stop at the first k with
 * threshold * loss >= previous_loss, and that k is the one returned because its
 * result has already replaced the previous one; without a stop the last k is
 * returned).  Entries whose status is non-zero are skipped as if absent.
 * Returns the index into ks, or -1 if no entry is usable. */
int orc_select_k(const double *loss, const int32_t *status, int n_k, double threshold)
{
    int have_prev = 0, last = -1;
    double prev = 0.0;
    for (int i = 0; i < n_k; ++i) {
        if (status && status[i] != 0) continue;
        if (have_prev && threshold * loss[i] >= prev) return i;
        prev = loss[i];
        have_prev = 1;
        last = i;
    }
    return last;
}

/* Representative configuration of each cluster: labels are the nearest-centroid
 * labels under mu; the pick of a non-empty cluster is its member closest to the
 * centroid, smallest row index on ties; pick_row = -1 for an empty cluster.
 * (Sec. 3.3 uses the centroids as representatives; a centroid is real-valued,
 * so the benchmark's rule is to take the nearest member configuration.) */
void orc_snap(const knob_t *x, int64_t n, int d, int k, const double *mu,
              int32_t *labels, int64_t *pick_row)
{
    double *dmin = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
    double *bd = (double *)malloc(sizeof(double) * (size_t)k);
    assign_all(x, n, d, k, mu, labels, dmin);
    for (int c = 0; c < k; ++c) pick_row[c] = -1;
    for (int64_t i = 0; i < n; ++i) {
        int c = labels[i];
        if (pick_row[c] < 0 || dmin[i] < bd[c]) { pick_row[c] = i; bd[c] = dmin[i]; }
    }
    free(dmin); free(bd);
}

/* 64-bit FNV-1a over the knob values, one xor-multiply step per knob; the
 * offset basis is first mixed with the task salt so that equal vectors of
 * different tasks hash apart.  With salt 0 and every value below 256 this is
 * exactly FNV-1a of the byte string; a larger value enters its step whole. */
uint64_t orc_hash(const knob_t *cfg, int d, uint64_t salt)
{
    uint64_t h = 0xCBF29CE484222325ULL ^ (salt * 0x9E3779B97F4A7C15ULL);
    for (int j = 0; j < d; ++j) {
        h ^= (uint64_t)cfg[j];
        h *= 0x100000001B3ULL;
    }
    return h;
}

void orc_hash_rows(const knob_t *x, int64_t n, int d, const uint64_t *salt_per_row,
                   uint64_t salt_all, uint64_t *out)
{
    for (int64_t i = 0; i < n; ++i)
        out[i] = orc_hash(x + (size_t)i * d, d, salt_per_row ? salt_per_row[i] : salt_all);
}

static int in_sorted(const uint64_t *v, int64_t n, uint64_t key)
{
    int64_t lo = 0, hi = n;
    while (lo < hi) {
        int64_t mid = lo + (hi - lo) / 2;
        if (v[mid] < key) lo = mid + 1; else hi = mid;
    }
    return lo < n && v[lo] == key;
}

/* Sample Synthesis with dedupe (Algorithm 1's second loop; Sec. 3.3 "most
 * frequent ... non-invalid choice for each knob").
 * A pick is flagged when its row is invalid or its hash is in the visited set.
 * Unflagged picks are KEPT.  For each flagged cluster in ascending order the
 * replacement takes, per knob, the value most frequent among the cluster's
 * valid members (smallest value on ties); it is DROPPED when the cluster has no
 * valid member, when its hash is visited, when it equals a kept pick, or when it
 * equals a replacement accepted for a lower cluster; otherwise it is SYNTH.
 * Empty clusters are EMPTY.  Rows of out_cfg for DROPPED / EMPTY are zero. */
void orc_synthesize(const knob_t *x, int64_t n, int d, const uint16_t *cards,
                    const uint8_t *valid, int k, const int32_t *labels,
                    const int64_t *pick_row, const uint64_t *visited, int64_t n_visited,
                    uint64_t salt, knob_t *out_cfg, uint8_t *out_flag, int32_t *out_count)
{
    int cmax = 0;
    for (int j = 0; j < d; ++j) if (cards[j] > cmax) cmax = cards[j];
    int64_t *hist = (int64_t *)malloc(sizeof(int64_t) * (size_t)d * (size_t)(cmax > 0 ? cmax : 1));
    uint8_t *flagged = (uint8_t *)calloc((size_t)k, 1);
    knob_t *m = (knob_t *)malloc(sizeof(knob_t) * (size_t)d);
    memset(out_cfg, 0, sizeof(knob_t) * (size_t)k * d);
    int count = 0;
    for (int c = 0; c < k; ++c) {
        if (pick_row[c] < 0) { out_flag[c] = ORC_EMPTY; continue; }
        const knob_t *p = x + (size_t)pick_row[c] * d;
        int bad = (valid && !valid[pick_row[c]]) || in_sorted(visited, n_visited, orc_hash(p, d, salt));
        if (bad) { flagged[c] = 1; out_flag[c] = ORC_DROPPED; }
        else { out_flag[c] = ORC_KEPT; memcpy(out_cfg + (size_t)c * d, p, sizeof(knob_t) * (size_t)d); ++count; }
    }
    for (int c = 0; c < k; ++c) {
        if (!flagged[c]) continue;
        memset(hist, 0, sizeof(int64_t) * (size_t)d * cmax);
        int64_t members = 0;
        for (int64_t i = 0; i < n; ++i) {
            if (labels[i] != c || (valid && !valid[i])) continue;
            ++members;
            for (int j = 0; j < d; ++j) {
                /* a choice index at or above the knob's cardinality (outside the design space of
                 * Sec. 2.2; the caller's precondition) can never be the mode: it is not counted */
                const int v = (int)x[(size_t)i * d + j];
                if (v < (int)cards[j]) hist[(size_t)j * cmax + v] += 1;
            }
        }
        if (members == 0) continue;                          /* stays DROPPED */
        for (int j = 0; j < d; ++j) {
            int bv = 0;
            for (int v = 1; v < cards[j]; ++v)
                if (hist[(size_t)j * cmax + v] > hist[(size_t)j * cmax + bv]) bv = v;
            m[j] = (knob_t)bv;
        }
        int dup = in_sorted(visited, n_visited, orc_hash(m, d, salt));
        for (int q = 0; q < k && !dup; ++q) {
            int use = (out_flag[q] == ORC_KEPT) || (q < c && out_flag[q] == ORC_SYNTH);
            if (use && memcmp(out_cfg + (size_t)q * d, m, sizeof(knob_t) * (size_t)d) == 0) dup = 1;
        }
        if (dup) continue;
        out_flag[c] = ORC_SYNTH;
        memcpy(out_cfg + (size_t)c * d, m, sizeof(knob_t) * (size_t)d);
        ++count;
    }
    *out_count = count;
    free(hist); free(flagged); free(m);
}
