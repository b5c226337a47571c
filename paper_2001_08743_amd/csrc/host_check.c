/* Driver for a sanitizer build of the library's host code (development check, built and run by
 * tests/test_sanitizers.py; not part of libcham).  It calls the entry points of cham.h with
 * invalid arguments of every kind and with well-formed arguments that stop at the workspace
 * check, i.e. it walks the argument validation, the planning of a call (tables of task offsets,
 * k lists, workspace layout, kernel family) and the host-side helpers under AddressSanitizer and
 * UndefinedBehaviorSanitizer.  Nothing here reaches a kernel launch, so no GPU is needed and the
 * device pointers can be placeholders that are never dereferenced. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "cham.h"

static int fails = 0;
#define EXPECT(cond)                                                       \
    do {                                                                   \
        if (!(cond)) {                                                     \
            fprintf(stderr, "host_check: line %d: %s\n", __LINE__, #cond); \
            ++fails;                                                       \
        }                                                                  \
    } while (0)

int main(void)
{
    EXPECT(cham_version() > 0);
    for (int c = -14; c <= 2; ++c) EXPECT(cham_strerror(c) != NULL);
    for (int p = -1; p <= 4; ++p) EXPECT(cham_sweep_path_kernel(p) != NULL);
    (void)cham_last_hip_error();

    /* placeholders for device memory: aligned, non-null, never dereferenced by host code */
    uint8_t *dev8 = (uint8_t *)(uintptr_t)0x10000;
    uint16_t *dev16 = (uint16_t *)(uintptr_t)0x10000;
    double *devd = (double *)(uintptr_t)0x20000;
    int32_t *devi = (int32_t *)(uintptr_t)0x30000;

    /* task tables of several sizes: the inline table of a call and the one that needs the heap */
    const int sizes[4] = {1, 3, 700, 2500};
    for (int si = 0; si < 4; ++si) {
        const int T = sizes[si];
        int64_t *off = (int64_t *)malloc(sizeof(int64_t) * (size_t)(T + 1));
        off[0] = 0;
        for (int t = 0; t < T; ++t) off[t + 1] = off[t] + (t % 3 == 1 ? 0 : 50 + 7 * (t % 11));   /* some tasks empty */
        const int64_t rows = off[T], ld = (rows + 63) / 64 * 64 + 64;
        int32_t ks[64];
        for (int i = 0; i < 64; ++i) ks[i] = i + 1;
        for (int d = 1; d <= 32; d += 5) {
            for (int flags = 0; flags <= 8; flags = flags ? flags * 2 : 1) {
                const int64_t need = cham_sweep_workspace_bytes(ld, d, off, T, ks, 64, 10, flags);
                EXPECT(need > 0);
                EXPECT(cham_sweep_knee_workspace_bytes(ld, d, off, T, ks, 64, 10, flags) >= need);
                const int path = cham_sweep_path(ld, d, off, T, ks, 64, flags);
                EXPECT(path >= 0 && path <= 2);
                /* a well-formed call without workspace: everything up to the workspace check runs */
                EXPECT(cham_kmeans_sweep(dev8, ld, d, off, T, ks, 64, 10, 0, NULL, devd, devi, devd, devi, NULL, NULL,
                                         NULL, 0, flags, NULL) == CHAM_E_WORKSPACE);
                EXPECT(cham_kmeans_sweep_knee(dev8, ld, d, off, T, ks, 64, 10, 0, NULL, 2.5, 8, devd, devi, devd,
                                              devi, devi, NULL, NULL, NULL, 0, flags, NULL) == CHAM_E_WORKSPACE);
            }
            EXPECT(cham_snap_workspace_bytes(ld, d, off, T, ks, 64) > 0);
            EXPECT(cham_synth_workspace_bytes(ld, d, off, T, ks, 64) > 0);
        }
        EXPECT(cham_sweep_workspace_bytes_u16(ld, 40, off, T, ks, 16, 10, 0) > 0);
        EXPECT(cham_kmeans_sweep_u16(dev16, ld, 40, off, T, ks, 16, 10, 0, NULL, devd, devi, devd, devi, NULL, NULL,
                                     NULL, 0, 0, NULL) == CHAM_E_WORKSPACE);
        /* the entry point without allocations: too large for its scratch, or no device at all */
        {
            const int32_t rc = cham_kmeans_sweep_static(dev8, ld, 8, off, T, ks, 64, 10, 0, NULL, devd, devi, devd, devi,
                                                        NULL, NULL, 0, NULL);
            EXPECT(rc == CHAM_E_TOO_LARGE || rc == CHAM_E_HIP || rc == CHAM_E_BAD_DIM);
        }

        /* invalid arguments */
        EXPECT(cham_sweep_workspace_bytes(ld, 0, off, T, ks, 64, 10, 0) == CHAM_E_BAD_DIM);
        EXPECT(cham_sweep_workspace_bytes(ld, 33, off, T, ks, 64, 10, 0) == CHAM_E_BAD_DIM);
        EXPECT(cham_sweep_workspace_bytes(rows > 4 ? rows - 4 : -4, 8, off, T, ks, 64, 10, 0) == CHAM_E_BAD_DIM);
        EXPECT(cham_sweep_workspace_bytes(ld + 1, 8, off, T, ks, 64, 10, 0) == CHAM_E_BAD_DIM);
        EXPECT(cham_sweep_workspace_bytes(ld, 8, NULL, T, ks, 64, 10, 0) == CHAM_E_NULL);
        EXPECT(cham_sweep_workspace_bytes(ld, 8, off, T, NULL, 64, 10, 0) == CHAM_E_NULL);
        EXPECT(cham_sweep_workspace_bytes(ld, 8, off, 0, ks, 64, 10, 0) == CHAM_E_BAD_DIM);
        EXPECT(cham_sweep_workspace_bytes(ld, 8, off, T, ks, 0, 10, 0) == CHAM_E_BAD_K);
        EXPECT(cham_kmeans_sweep(dev8, ld, 8, off, T, ks, 64, 10, 0, NULL, devd, devi, devd, devi, NULL, NULL, NULL, 0,
                                 1 << 9, NULL) == CHAM_E_BAD_FLAG);
        {
            int32_t bad[3] = {4, 4, 9};
            EXPECT(cham_sweep_workspace_bytes(ld, 8, off, T, bad, 3, 10, 0) == CHAM_E_BAD_K);
            bad[0] = 0;
            EXPECT(cham_sweep_workspace_bytes(ld, 8, off, T, bad, 1, 10, 0) == CHAM_E_BAD_K);
            bad[0] = 257;
            EXPECT(cham_sweep_workspace_bytes(ld, 8, off, T, bad, 1, 10, 0) == CHAM_E_BAD_K);
        }
        if (T >= 3) {
            const int64_t keep = off[2];
            off[2] = off[1] - 1;
            EXPECT(cham_sweep_workspace_bytes(ld, 8, off, T, ks, 64, 10, 0) == CHAM_E_BAD_OFFSETS);
            off[2] = keep;
        }
        EXPECT(cham_kmeans_sweep(NULL, ld, 8, off, T, ks, 64, 10, 0, NULL, devd, devi, devd, devi, NULL, NULL, NULL, 0, 0,
                                 NULL) == CHAM_E_NULL);
        EXPECT(cham_kmeans_sweep(dev8, ld, 8, off, T, ks, 64, 10, 0, NULL, NULL, devi, devd, devi, NULL, NULL, NULL, 0, 0,
                                 NULL) == CHAM_E_NULL);
        EXPECT(cham_kmeans_sweep(dev8, ld, 8, off, T, ks, 64, -1, 0, NULL, devd, devi, devd, devi, NULL, NULL, NULL, 0, 0,
                                 NULL) == CHAM_E_BAD_DIM);
        EXPECT(cham_kmeans_sweep(dev8, ld, 8, off, T, ks, 64, 10, 1, NULL, devd, devi, devd, devi, NULL, NULL, NULL, 0, 0,
                                 NULL) == CHAM_E_NULL);
        EXPECT(cham_kmeans_sweep(dev8, ld, 8, off, T, ks, 64, 10, 2, NULL, devd, devi, devd, devi, NULL, NULL, NULL, 0, 0,
                                 NULL) == CHAM_E_BAD_FLAG);
        EXPECT(cham_kmeans_sweep(dev8 + 1, ld, 8, off, T, ks, 64, 10, 0, NULL, devd, devi, devd, devi, NULL, NULL, NULL, 0,
                                 0, NULL) == CHAM_E_BAD_DIM);
        /* synthesis: cardinalities are checked on the host */
        {
            uint16_t *cards = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)T * 8);
            for (int i = 0; i < T * 8; ++i) cards[i] = (uint16_t)(2 + i % 200);
            EXPECT(cham_synthesize(dev8, ld, 8, off, T, cards, NULL, ks, 64, devi, dev8, devi, dev8, NULL, 0, NULL, dev8,
                                   dev8, devi, NULL, 0, NULL) == CHAM_E_WORKSPACE);
            cards[T * 8 - 1] = 0;
            EXPECT(cham_synthesize(dev8, ld, 8, off, T, cards, NULL, ks, 64, devi, dev8, devi, dev8, NULL, 0, NULL, dev8,
                                   dev8, devi, NULL, 0, NULL) == CHAM_E_CARD);
            cards[T * 8 - 1] = 257;
            EXPECT(cham_synthesize(dev8, ld, 8, off, T, cards, NULL, ks, 64, devi, dev8, devi, dev8, NULL, 0, NULL, dev8,
                                   dev8, devi, NULL, 0, NULL) == CHAM_E_CARD);
            free(cards);
        }
        EXPECT(cham_snap_centroids(dev8, ld, 8, off, T, ks, 64, devi, devd, dev8, devi, dev8, NULL, 0, 0, NULL) ==
               CHAM_E_WORKSPACE);
        free(off);
    }

    /* the knee rule on host arrays */
    {
        const double curve[6] = {100.0, 30.0, 10.0, 9.0, 8.5, 8.4};
        const int32_t st[6] = {0, 0, 1, 0, 0, 0};
        EXPECT(cham_select_k_host(curve, NULL, 6, 2.5) == 3);
        EXPECT(cham_select_k_host(curve, st, 6, 2.5) == 4);
        EXPECT(cham_select_k_host(curve, NULL, 0, 2.5) == -1);
        EXPECT(cham_select_k_host(curve, NULL, 1, 2.5) == 0);
    }
    if (fails) return 1;
    printf("host_check ok\n");
    return 0;
}
