/* Driver for a sanitizer build of the oracle (test infrastructure): runs every entry point of
 * cham_oracle.c on small seeded inputs, including the degenerate ones (an empty task, fewer
 * distinct rows than k, an empty visited set, a knob value at or above its cardinality), so that
 * AddressSanitizer and UndefinedBehaviorSanitizer see each of its loops.  Built and run by
 * tests/test_sanitizers.py:
 *   gcc -O1 -g -std=c11 -fsanitize=address,undefined -fno-sanitize-recover=all -static-libasan \
 *       oracle/cham_oracle.c oracle/sanitize_check.c -lm -o sanitize_check
 * Prints "sanitize_check ok" and exits 0 when nothing was reported. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef uint16_t knob_t;
int orc_num_threads(void);
int orc_first_distinct(const knob_t *x, int64_t n, int d, int kmax, int64_t *rows_out);
void orc_kmeans(const knob_t *x, int64_t n, int d, int k, int n_iter, double *mu, int64_t *counts,
                int32_t *labels, double *inertia, double *trace);
void orc_sweep(const knob_t *x, int d, const int64_t *task_off, int T, const int32_t *ks, int n_k, int n_iter,
               int init_mode, const double *init, double *centroids, int64_t *counts, double *inertia,
               int32_t *status, int32_t *labels, double *trace);
int orc_select_k(const double *loss, const int32_t *status, int n_k, double threshold);
void orc_snap(const knob_t *x, int64_t n, int d, int k, const double *mu, int32_t *labels, int64_t *pick_row);
uint64_t orc_hash(const knob_t *cfg, int d, uint64_t salt);
void orc_hash_rows(const knob_t *x, int64_t n, int d, const uint64_t *salt_per_row, uint64_t salt_all,
                   uint64_t *out);
void orc_synthesize(const knob_t *x, int64_t n, int d, const uint16_t *cards, const uint8_t *valid, int k,
                    const int32_t *labels, const int64_t *pick_row, const uint64_t *visited, int64_t n_visited,
                    uint64_t salt, knob_t *out_cfg, uint8_t *out_flag, int32_t *out_count);

static uint64_t rng_state = 0x243F6A8885A308D3ULL;
static uint32_t rnd(void)
{
    rng_state = rng_state * 6364136223846793005ULL + 1442695040888963407ULL;
    return (uint32_t)(rng_state >> 33);
}

static int cmp_u64(const void *a, const void *b)
{
    const uint64_t x = *(const uint64_t *)a, y = *(const uint64_t *)b;
    return x < y ? -1 : (x > y ? 1 : 0);
}

static void one_case(int64_t n0, int64_t n1, int d, int card, int n_iter, int shrink_all)
{
    /* three tasks: n0 rows, none, n1 rows (the last with few distinct rows) */
    const int64_t off[4] = {0, n0, n0, n0 + n1};
    const int64_t n = off[3];
    const int32_t ks[3] = {1, 3, 7};
    const int n_k = 3, Ksum = 11, T = 3;
    knob_t *x = (knob_t *)malloc(sizeof(knob_t) * (size_t)(n > 0 ? n : 1) * d);
    for (int64_t i = 0; i < n0; ++i)
        for (int j = 0; j < d; ++j) x[i * d + j] = (knob_t)(rnd() % (uint32_t)card);
    for (int64_t i = n0; i < n; ++i)
        for (int j = 0; j < d; ++j) x[i * d + j] = (knob_t)((i - n0) % 2);      /* two distinct rows */

    double *cent = (double *)malloc(sizeof(double) * (size_t)T * Ksum * d);
    int64_t *counts = (int64_t *)malloc(sizeof(int64_t) * (size_t)T * Ksum);
    double *inertia = (double *)malloc(sizeof(double) * (size_t)T * n_k);
    int32_t *status = (int32_t *)malloc(sizeof(int32_t) * (size_t)T * n_k);
    int32_t *labels = (int32_t *)malloc(sizeof(int32_t) * (size_t)n_k * (size_t)(n > 0 ? n : 1));
    double *trace = (double *)malloc(sizeof(double) * (size_t)T * n_k * (n_iter + 1));
    orc_sweep(x, d, off, T, ks, n_k, n_iter, 0, NULL, cent, counts, inertia, status, labels, trace);
    /* the same again from the centroids just found (init_mode 1), without the optional outputs */
    double *cent2 = (double *)malloc(sizeof(double) * (size_t)T * Ksum * d);
    orc_sweep(x, d, off, T, ks, n_k, 1, 1, cent, cent2, counts, inertia, status, NULL, NULL);

    for (int t = 0; t < T; ++t) {
        const int ki = orc_select_k(inertia + t * n_k, status + t * n_k, n_k, 2.5);
        if (ki < 0) continue;
        const int k = ks[ki];
        const int64_t nt = off[t + 1] - off[t];
        const knob_t *xt = x + off[t] * d;
        int64_t koff = 0;
        for (int i = 0; i < ki; ++i) koff += ks[i];
        int32_t *lab = (int32_t *)malloc(sizeof(int32_t) * (size_t)(nt > 0 ? nt : 1));
        int64_t *pick = (int64_t *)malloc(sizeof(int64_t) * (size_t)k);
        orc_snap(xt, nt, d, k, cent2 + ((size_t)t * Ksum + koff) * d, lab, pick);
        /* visited: hashes of every third row, sorted; validity: every fifth row invalid */
        const int64_t nv = nt / 3;
        uint64_t *vis = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)(nv > 0 ? nv : 1));
        for (int64_t i = 0; i < nv; ++i) vis[i] = orc_hash(xt + 3 * i * d, d, (uint64_t)t);
        qsort(vis, (size_t)nv, sizeof(uint64_t), cmp_u64);
        uint8_t *valid = (uint8_t *)malloc((size_t)(nt > 0 ? nt : 1));
        for (int64_t i = 0; i < nt; ++i) valid[i] = (uint8_t)(i % 5 != 0);
        uint16_t *cards = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)d);
        for (int j = 0; j < d; ++j) cards[j] = (uint16_t)((j == 0 || shrink_all) && card > 1 ? card - 1 : card);   /* values may reach the cardinality */
        knob_t *out_cfg = (knob_t *)malloc(sizeof(knob_t) * (size_t)k * d);
        uint8_t *out_flag = (uint8_t *)malloc((size_t)k);
        int32_t out_count = -1;
        orc_synthesize(xt, nt, d, cards, valid, k, lab, pick, vis, nv, (uint64_t)t, out_cfg, out_flag, &out_count);
        orc_synthesize(xt, nt, d, cards, NULL, k, lab, pick, vis, 0, (uint64_t)t, out_cfg, out_flag, &out_count);
        if (out_count < 0 || out_count > k) { fprintf(stderr, "bad count\n"); exit(2); }
        uint64_t *hh = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)(nt > 0 ? nt : 1));
        orc_hash_rows(xt, nt, d, NULL, 7, hh);
        free(hh); free(out_flag); free(out_cfg); free(cards); free(valid); free(vis); free(pick); free(lab);
    }
    int64_t first[8];
    (void)orc_first_distinct(x, n, d, 8, first);
    free(cent2); free(trace); free(labels); free(status); free(inertia); free(counts); free(cent); free(x);
}

int main(void)
{
    (void)orc_num_threads();
    one_case(300, 40, 5, 9, 4, 0);
    one_case(300, 40, 5, 9, 4, 1);    /* every knob: values up to the cardinality itself (precondition broken) */
    one_case(1, 2, 1, 2, 0, 0);
    one_case(0, 0, 3, 4, 2, 0);          /* every task empty */
    one_case(64, 9, 24, 256, 3, 0);
    one_case(50, 5, 40, 1000, 2, 0);     /* wide design space: values above 255 */
    printf("sanitize_check ok\n");
    return 0;
}
