/*
 * Drives the host side of every entry point of the C ABI in a process that has
 * no GPU: argument checking, code construction, rebuild matrices, RDP plans
 * and all the launch preparation (tables, row plans, grids) run for real, and
 * the launch itself fails in the runtime with GS_EHIP.  Built together with
 * the library's sources (host code only) under AddressSanitizer and UBSan by
 * tests/test_host_sanitize.py; any out-of-bounds access or undefined
 * arithmetic on the way to a launch aborts the program.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../include/ghostserve_ec.h"

#define EXPECT(cond) do { if (!(cond)) { printf("FAIL line %d: %s\n", __LINE__, #cond); return 1; } } while (0)

enum { MAXN = 256 };

static void *fake[MAXN];  /* aligned, never dereferenced: no launch can succeed here */

static int encode_and_rebuild(gs_code *code, int k, int m)
{
    static const size_t sizes[] = {1, 15, 16, 17, 4096 + 5, (size_t)1 << 20, ((size_t)1 << 33) + 48, (size_t)1 << 40};
    for (size_t si = 0; si < sizeof sizes / sizeof sizes[0]; si++) {
        const int rc = gs_encode(code, (const void *const *)fake, fake + k, sizes[si], NULL);
        EXPECT(rc == GS_EHIP || rc == GS_EINVAL);  /* EINVAL: RDP needs whole stripes */
        int er[4] = {0, k, 1, k + 1};
        for (int e = 0; e <= m && e <= 4; e++) {
            if (k == 1 && e > 1) {
                er[1] = 1;
                er[2] = 2;
                er[3] = 3;
            }
            const int rr = gs_reconstruct(code, fake, er, e, sizes[si], NULL);
            EXPECT(e == 0 ? rr == GS_OK : (rr == GS_EHIP || rr == GS_EINVAL));
        }
    }
    EXPECT(gs_encode(code, (const void *const *)fake, fake + k, 0, NULL) == GS_OK);
    return 0;
}

int main(void)
{
    /* far enough apart that no two of them overlap at the largest size tried below */
    for (int i = 0; i < MAXN; i++) fake[i] = (void *)(uintptr_t)(((uint64_t)1 << 42) + ((uint64_t)(unsigned)i << 41));

    /* every code kind over a range of widths, all launch shapes */
    static const int shapes[][4] = {{0, 0, -1, -1}, {1, 1, 1, 5}, {2, 3, 0, 0}, {4, 1, 1, 10}, {1, 7, 1, 3}};
    for (size_t sh = 0; sh < sizeof shapes / sizeof shapes[0]; sh++) {
        EXPECT(gs_set_launch_shape(shapes[sh][0], shapes[sh][1], shapes[sh][2], shapes[sh][3]) == GS_OK);
        for (int kind = GS_CAUCHY; kind <= GS_POWER; kind++) {
            static const int km[][2] = {{1, 1}, {4, 1}, {4, 2}, {8, 2}, {8, 3}, {16, 4}, {17, 2}, {40, 6}, {3, 3}, {250, 6}, {1, 255}};
            for (size_t c = 0; c < sizeof km / sizeof km[0]; c++) {
                const int k = km[c][0], m = km[c][1];
                gs_code *code = NULL;
                const int rc = gs_make_code(k, m, kind, &code);
                const int rdp_ok = kind == GS_RDP && m == 2 && k <= 16;
                const int pow_ok = kind == GS_POWER && m <= 3;
                if ((kind == GS_RDP && !rdp_ok) || (kind == GS_POWER && !pow_ok)) {
                    EXPECT(rc == GS_EINVAL && code == NULL);
                    continue;
                }
                EXPECT(rc == GS_OK && code != NULL);
                int kk = 0, mm = 0;
                EXPECT(gs_code_params(code, &kk, &mm) == GS_OK && kk == k && mm == m);
                for (int horner = 0; horner <= 1; horner++) {
                    EXPECT(gs_set_power_horner(horner) == GS_OK);
                    if (encode_and_rebuild(code, k, m)) return 1;
                }
                if (kind != GS_RDP) {
                    static uint8_t P[MAXN * MAXN], R[8 * MAXN];
                    int surv[MAXN];
                    EXPECT(gs_code_matrix(code, P) == GS_OK);
                    for (int j = 0; j < k; j++) EXPECT(P[j] == 1);
                    int er[8];
                    const int e = m < 6 ? m : 6;
                    for (int x = 0; x < e; x++) er[x] = (x % 2) ? k + x / 2 : (k - 1 - x / 2 >= 0 ? k - 1 - x / 2 : 0);
                    if (k == 1) for (int x = 0; x < e; x++) er[x] = x;
                    EXPECT(gs_decode_matrix(code, er, e, R, surv) == GS_OK);
                    er[0] = k + m;
                    EXPECT(gs_decode_matrix(code, er, 1, R, surv) == GS_EINVAL);
                    /* paged forms, table rows and dense buffers on both sides */
                    int rp = gs_encode_paged(code, (const void *const *)fake[0], 3, 2048, 64, (const int32_t *)fake[1], 5, fake + k, NULL);
                    EXPECT(rp == GS_EHIP);
                    rp = gs_encode_paged(code, (const void *const *)fake[0], 3, 48, 64, (const int32_t *)fake[1], 5, fake + k, NULL);
                    EXPECT(rp == GS_EHIP);
                    er[0] = 0;
                    er[1] = k;
                    rp = gs_reconstruct_paged(code, (const void *const *)fake[0], 3, 2048, 64, (const int32_t *)fake[1], 5, fake + k, er,
                                              m >= 2 ? 2 : 1, NULL);
                    EXPECT(rp == GS_EHIP);
                } else {
                    int p = 0, read[18], n_read = 0;
                    uint32_t masks[32];
                    size_t cell = 0;
                    EXPECT(gs_rdp_prime(code, &p) == GS_OK && p >= k + 1);
                    EXPECT(gs_rdp_cell_bytes(code, &cell) == GS_OK && cell == GS_RDP_DEFAULT_CELL);
                    EXPECT(gs_rdp_plan(code, NULL, 0, read, &n_read, masks) == GS_OK && n_read == k);
                    for (int a = 0; a < k + 2; a++)
                        for (int b = a + 1; b < k + 2; b++) {
                            const int miss[2] = {a, b};
                            EXPECT(gs_rdp_plan(code, miss, 2, read, &n_read, masks) == GS_OK && n_read == k);
                        }
                    const size_t stripe = cell * (size_t)(p - 1);
                    EXPECT(gs_encode(code, (const void *const *)fake, fake + k, 3 * stripe, NULL) == GS_EHIP);
                    const int miss[2] = {0, k + 1};
                    EXPECT(gs_reconstruct(code, fake, miss, 2, 3 * stripe, NULL) == GS_EHIP);
                    EXPECT(gs_reconstruct(code, fake, miss, 2, stripe + 16, NULL) == GS_EINVAL);
                    uint8_t dummy[4];
                    EXPECT(gs_code_matrix(code, dummy) == GS_EINVAL);
                    /* paged RDP: a cell must be a page and the shard whole stripes of slots */
                    EXPECT(gs_encode_paged(code, (const void *const *)fake[0], 3, cell, 1 << 20, (const int32_t *)fake[1], 4 * (p - 1),
                                           fake + k, NULL) == GS_EHIP);
                    EXPECT(gs_encode_paged(code, (const void *const *)fake[0], 3, cell, 1 << 20, (const int32_t *)fake[1], 4 * (p - 1) + 1,
                                           fake + k, NULL) == GS_EINVAL);
                    EXPECT(gs_encode_paged(code, (const void *const *)fake[0], 3, 2048, 1 << 20, (const int32_t *)fake[1], 4 * (p - 1),
                                           fake + k, NULL) == GS_EINVAL);
                    EXPECT(gs_reconstruct_paged(code, (const void *const *)fake[0], 3, cell, 1 << 20, (const int32_t *)fake[1],
                                                4 * (p - 1), fake + k, miss, 2, NULL) == GS_EHIP);
                }
                /* objects that need device memory cannot be made here, and must not leak or crash */
                gs_pipe *pipe = (gs_pipe *)fake[0];
                gs_batch *batch = (gs_batch *)fake[0];
                EXPECT(gs_pipe_create(code, 1 << 20, 2, &pipe) != GS_OK && pipe == NULL);
                EXPECT(gs_batch_create(code, 8, &batch) != GS_OK && batch == NULL);
                gs_step_graph *graph = (gs_step_graph *)fake[0];
                EXPECT(gs_step_graph_create(code, (const void *const *)fake[0], 2, 2048, 64, (const int32_t *)fake[1], 4, fake + k, NULL,
                                            &graph) != GS_OK && graph == NULL);
                gs_free_code(code);
            }
        }
    }
    EXPECT(gs_set_launch_shape(0, 0, -1, -1) == GS_OK);
    EXPECT(gs_set_power_horner(1) == GS_OK);
    EXPECT(gs_set_size_forms(3) == GS_EINVAL && gs_set_size_forms(-1) == GS_EINVAL);
    EXPECT(gs_set_size_forms(2) == GS_OK && gs_set_size_forms(0) == GS_OK && gs_set_size_forms(1) == GS_OK);

    gs_code *rdp = NULL;
    EXPECT(gs_make_rdp_code(6, 4096, &rdp) == GS_OK);
    EXPECT(gs_encode(rdp, (const void *const *)fake, fake + 6, 4096 * 6 * 5, NULL) == GS_EHIP);
    gs_free_code(rdp);
    EXPECT(gs_make_rdp_code(6, 100, &rdp) == GS_EINVAL && rdp == NULL);

    gs_pool *pool = (gs_pool *)fake[0];
    EXPECT(gs_pool_create(4, &pool) != GS_OK && pool == NULL);
    EXPECT(gs_pool_create(0, &pool) == GS_EINVAL);

    for (int c = 0; c < 256; c++) {
        uint32_t w[5];
        EXPECT(gs_coef_words(c, w) == GS_OK);
    }
    EXPECT(gs_coef_words(256, (uint32_t *)fake) == GS_EINVAL);

    for (int n = 0; n <= 1000; n += 37) {
        const gs_recovery_costs costs = {0.02, 0.001, 0.003, 0.018, 0.0005, 0.004};
        int r = -1;
        double t = -1;
        EXPECT(gs_recompute_units(n, &costs, &r, &t) == GS_OK && r >= 0 && r <= n && t >= 0);
    }
    /* an output that shares bytes with an input or with another output of the same call is refused
     * before anything is enqueued; buffers that merely touch end to end are fine */
    {
        gs_code *code = NULL;
        EXPECT(gs_make_code(4, 2, GS_CAUCHY, &code) == GS_OK);
        void *p[6];
        const size_t S = 4096;
        for (int i = 0; i < 6; i++) p[i] = (void *)(uintptr_t)(((uint64_t)1 << 42) + S * (unsigned)i);
        EXPECT(gs_encode(code, (const void *const *)p, p + 4, S, NULL) == GS_EHIP);         /* adjacent: accepted */
        EXPECT(gs_encode(code, (const void *const *)p, p + 4, S + 16, NULL) == GS_EINVAL);  /* every buffer runs into the next */
        void *q[6];
        memcpy(q, p, sizeof q);
        q[4] = p[2];                                                                        /* parity 0 on top of data 2 */
        EXPECT(gs_encode(code, (const void *const *)q, q + 4, S, NULL) == GS_EINVAL);
        memcpy(q, p, sizeof q);
        q[5] = (char *)p[4] + S - 16;                                                       /* the two parities overlap */
        EXPECT(gs_encode(code, (const void *const *)q, q + 4, S, NULL) == GS_EINVAL);
        const int er[2] = {1, 4};
        EXPECT(gs_reconstruct(code, p, er, 2, S, NULL) == GS_EHIP);
        memcpy(q, p, sizeof q);
        q[1] = p[3];                                                                        /* erased shard 1 = survivor 3 */
        EXPECT(gs_reconstruct(code, q, er, 2, S, NULL) == GS_EINVAL);
        memcpy(q, p, sizeof q);
        q[5] = p[1];                          /* with only shard 1 lost, shard 5 is neither read nor written: it may point anywhere */
        EXPECT(gs_reconstruct(code, q, er, 1, S, NULL) == GS_EHIP);
        EXPECT(gs_reconstruct(code, q, er, 2, S, NULL) == GS_EINVAL);   /* with shard 4 lost as well it is read */
        gs_free_code(code);
        gs_code *rdp2 = NULL;
        EXPECT(gs_make_rdp_code(4, 64, &rdp2) == GS_OK);   /* p = 5: stripes of 256 bytes */
        for (int i = 0; i < 6; i++) p[i] = (void *)(uintptr_t)(((uint64_t)1 << 42) + 1024u * (unsigned)i);
        EXPECT(gs_encode(rdp2, (const void *const *)p, p + 4, 1024, NULL) == GS_EHIP);
        EXPECT(gs_encode(rdp2, (const void *const *)p, p + 4, 1280, NULL) == GS_EINVAL);
        const int er2[2] = {0, 5};
        memcpy(q, p, sizeof q);
        q[0] = p[2];
        EXPECT(gs_reconstruct(rdp2, q, er2, 2, 1024, NULL) == GS_EINVAL);
        gs_free_code(rdp2);
    }
    /* the grouped encode that allocates nothing: refusals, and the host side up to the first launch */
    {
        gs_code *code = NULL;
        EXPECT(gs_make_code(8, 2, GS_CAUCHY, &code) == GS_OK);
        static const void *data[8 * 40];
        static void *par[2 * 40];
        static size_t sizes[GS_STATIC_MAX_CHUNKS + 1];
        for (int c = 0; c < 40; c++) {
            for (int j = 0; j < 8; j++) data[c * 8 + j] = fake[(c * 10 + j) % MAXN];
            for (int i = 0; i < 2; i++) par[c * 2 + i] = fake[(c * 10 + 8 + i) % MAXN];
            sizes[c] = 4096 + 7 * (size_t)c;
        }
        EXPECT(gs_encode_batch_static(code, GS_STATIC_MAX_CHUNKS + 1, data, par, sizes, NULL) == GS_ELIMIT);
        EXPECT(gs_encode_batch_static(code, 0, data, par, sizes, NULL) == GS_OK);
        EXPECT(gs_encode_batch_static(code, -1, data, par, sizes, NULL) == GS_EINVAL);
        EXPECT(gs_encode_batch_static(code, 25, data, par, sizes, NULL) == GS_EHIP);   /* no device: the first runtime call fails */
        sizes[3] = (size_t)1 << 34;   /* the first length one tile per workgroup does not cover */
        EXPECT(gs_encode_batch_static(code, 25, data, par, sizes, NULL) == GS_ELIMIT);
        sizes[3] = 64;
        par[2 * 3] = (void *)data[8 * 3 + 1];
        EXPECT(gs_encode_batch_static(code, 25, data, par, sizes, NULL) == GS_EINVAL);  /* output on top of an input */
        gs_free_code(code);
        gs_code *wide = NULL;
        EXPECT(gs_make_code(17, 2, GS_CAUCHY, &wide) == GS_OK);
        EXPECT(gs_encode_batch_static(wide, 1, data, par, sizes, NULL) == GS_EINVAL);
        gs_free_code(wide);
        EXPECT(strlen(gs_strerror(GS_ELIMIT)) > 0);
    }
    EXPECT(gs_last_hip_error() != 0);
    EXPECT(strlen(gs_strerror(GS_EHIP)) > 0 && strlen(gs_strerror(12345)) > 0);
    gs_pipe_destroy(NULL);
    gs_batch_destroy(NULL);
    gs_pool_destroy(NULL);
    gs_step_graph_destroy(NULL);
    gs_free_code(NULL);
    printf("OK\n");
    return 0;
}
