/*
 * Per-step latency of the streaming-decode checkpoint, measured from plain C
 * (no interpreter in the loop): Section 4.2's "parity is updated once the KV
 * cache for a chunk of tokens is generated", at the decode-step shape of the
 * paged pool (one pool plane per layer and K/V, 16-token blocks of 2 KiB token
 * slots, 64 sequences in k = 4 shards, m = 1).
 *
 * Every step rewrites the device block table (the engine moved each sequence
 * to its next slot), then times  launch -> stream idle  on the host clock for
 *   eager          gs_encode_paged into a device parity buffer
 *   eager_d2h      the same plus hipMemcpyAsync of the parity to pinned memory
 *   eager_pinned   gs_encode_paged straight into the pinned buffer
 *   graph          the captured step (gs_step_graph_launch), encode only
 *   graph_d2h      the captured step with the D2H copy in the graph
 * and prints one JSON object.  Pool contents do not matter for timing (the
 * code is data-independent); the pool is filled with a byte pattern.
 *
 * usage: gs_step_latency [steps] [layers]
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <time.h>

#include "../../include/ghostserve_ec.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "HIP error %d at line %d\n", (int)e_, __LINE__); return 2; } } while (0)
#define CHECK_GS(x) do { int r_ = (x); if (r_ != GS_OK) { fprintf(stderr, "gs error %d (%s) at line %d\n", r_, gs_strerror(r_), __LINE__); return 3; } } while (0)

enum { K = 4, M = 1, SEQS = 64, SEQS_PER_SHARD = SEQS / K, BLOCK_TOKENS = 16, SLOT_BYTES = 8 * 128 * 2 };

static double now_us(void)
{
    struct timespec ts;
    clock_gettime(CLOCK_MONOTONIC, &ts);
    return ts.tv_sec * 1e6 + ts.tv_nsec * 1e-3;
}

static int cmp_double(const void *a, const void *b)
{
    const double x = *(const double *)a, y = *(const double *)b;
    return x < y ? -1 : x > y;
}

static uint32_t rng_state = 0x67530102u;
static uint32_t next_u32(void)
{
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 17;
    rng_state ^= rng_state << 5;
    return rng_state;
}

struct step_ctx {
    gs_code *code;
    void **plane_base_dev;
    int n_planes;
    int64_t pages_per_plane;
    int32_t *table_dev;
    void *par_dev[M];
    void *par_host[M];
    size_t out_bytes;
    hipStream_t stream;
    gs_step_graph *g0, *g1;
};

typedef int (*step_fn)(struct step_ctx *);

static int eager(struct step_ctx *c)
{
    return gs_encode_paged(c->code, (const void *const *)c->plane_base_dev, c->n_planes, SLOT_BYTES, c->pages_per_plane,
                           c->table_dev, SEQS_PER_SHARD, c->par_dev, c->stream);
}

static int eager_d2h(struct step_ctx *c)
{
    const int rc = eager(c);
    if (rc != GS_OK) return rc;
    for (int i = 0; i < M; i++)
        if (hipMemcpyAsync(c->par_host[i], c->par_dev[i], c->out_bytes, hipMemcpyDeviceToHost, c->stream) != hipSuccess)
            return GS_EHIP;
    return GS_OK;
}

static int eager_pinned(struct step_ctx *c)
{
    return gs_encode_paged(c->code, (const void *const *)c->plane_base_dev, c->n_planes, SLOT_BYTES, c->pages_per_plane,
                           c->table_dev, SEQS_PER_SHARD, c->par_host, c->stream);
}

static int graph(struct step_ctx *c) { return gs_step_graph_launch(c->g0, c->stream); }
static int graph_d2h(struct step_ctx *c) { return gs_step_graph_launch(c->g1, c->stream); }

int main(int argc, char **argv)
{
    const int steps = argc > 1 ? atoi(argv[1]) : 1000;
    const int layers = argc > 2 ? atoi(argv[2]) : 32;
    const int warm = 50;
    if (steps < 1 || steps > 100000 || layers < 1 || layers > 512) {
        fprintf(stderr, "usage: gs_step_latency [steps 1..100000] [layers 1..512]\n");
        return 1;
    }
    struct step_ctx c;
    memset(&c, 0, sizeof c);
    c.n_planes = 2 * layers;
    const int blocks_per_seq = (steps + warm + BLOCK_TOKENS - 1) / BLOCK_TOKENS;
    const int64_t n_blocks = (int64_t)SEQS * blocks_per_seq;
    c.pages_per_plane = n_blocks * BLOCK_TOKENS;
    const size_t plane_bytes = (size_t)c.pages_per_plane * SLOT_BYTES;
    c.out_bytes = (size_t)c.n_planes * SEQS_PER_SHARD * SLOT_BYTES;

    CHECK_GS(gs_make_code(K, M, GS_CAUCHY, &c.code));
    CHECK_HIP(hipStreamCreateWithFlags(&c.stream, hipStreamNonBlocking));

    /* the pool: one allocation, plane p at offset p * plane_bytes */
    uint8_t *pool = NULL;
    CHECK_HIP(hipMalloc((void **)&pool, plane_bytes * c.n_planes));
    CHECK_HIP(hipMemset(pool, 0x5B, plane_bytes * c.n_planes));
    void **base_host = (void **)malloc(sizeof(void *) * c.n_planes);
    for (int p = 0; p < c.n_planes; p++) base_host[p] = pool + (size_t)p * plane_bytes;
    CHECK_HIP(hipMalloc((void **)&c.plane_base_dev, sizeof(void *) * c.n_planes));
    CHECK_HIP(hipMemcpy(c.plane_base_dev, base_host, sizeof(void *) * c.n_planes, hipMemcpyHostToDevice));

    /* block ownership: a shuffled list of all blocks, blocks_per_seq for each sequence */
    int32_t *perm = (int32_t *)malloc(sizeof(int32_t) * n_blocks);
    for (int64_t i = 0; i < n_blocks; i++) perm[i] = (int32_t)i;
    for (int64_t i = n_blocks - 1; i > 0; i--) {
        const int64_t j = next_u32() % (uint32_t)(i + 1);
        const int32_t t = perm[i];
        perm[i] = perm[j];
        perm[j] = t;
    }
    /* tables of all steps in pinned memory; step s is copied to the device table before it runs */
    int32_t *tables = NULL;
    const size_t table_bytes = sizeof(int32_t) * SEQS;
    CHECK_HIP(hipHostMalloc((void **)&tables, table_bytes * (steps + warm), hipHostMallocDefault));
    for (int s = 0; s < steps + warm; s++)
        for (int q = 0; q < SEQS; q++)
            tables[(size_t)s * SEQS + q] = perm[(size_t)(s / BLOCK_TOKENS) * SEQS + q] * BLOCK_TOKENS + s % BLOCK_TOKENS;
    CHECK_HIP(hipMalloc((void **)&c.table_dev, table_bytes));

    for (int i = 0; i < M; i++) {
        CHECK_HIP(hipMalloc(&c.par_dev[i], c.out_bytes));
        CHECK_HIP(hipHostMalloc(&c.par_host[i], c.out_bytes, hipHostMallocDefault));
    }
    CHECK_HIP(hipMemcpy(c.table_dev, tables, table_bytes, hipMemcpyHostToDevice));
    CHECK_GS(gs_step_graph_create(c.code, (const void *const *)c.plane_base_dev, c.n_planes, SLOT_BYTES, c.pages_per_plane,
                                  c.table_dev, SEQS_PER_SHARD, c.par_dev, NULL, &c.g0));
    CHECK_GS(gs_step_graph_create(c.code, (const void *const *)c.plane_base_dev, c.n_planes, SLOT_BYTES, c.pages_per_plane,
                                  c.table_dev, SEQS_PER_SHARD, c.par_dev, c.par_host, &c.g1));

    static const char *names[] = {"eager", "eager_d2h", "eager_pinned", "graph", "graph_d2h"};
    const step_fn fns[] = {eager, eager_d2h, eager_pinned, graph, graph_d2h};
    double *lat = (double *)malloc(sizeof(double) * steps);
    printf("{\"steps\": %d, \"layers\": %d, \"new_kv_bytes_per_step\": %zu, \"parity_bytes_per_step\": %zu",
           steps, layers, (size_t)K * c.out_bytes, (size_t)M * c.out_bytes);
    for (int v = 0; v < 5; v++) {
        for (int s = 0; s < steps + warm; s++) {
            CHECK_HIP(hipMemcpyAsync(c.table_dev, tables + (size_t)s * SEQS, table_bytes, hipMemcpyHostToDevice, c.stream));
            CHECK_HIP(hipStreamSynchronize(c.stream));
            const double t0 = now_us();
            CHECK_GS(fns[v](&c));
            CHECK_HIP(hipStreamSynchronize(c.stream));
            const double t1 = now_us();
            if (s >= warm) lat[s - warm] = t1 - t0;
        }
        qsort(lat, steps, sizeof(double), cmp_double);
        double sum = 0;
        for (int s = 0; s < steps; s++) sum += lat[s];
        printf(", \"%s\": {\"p50_us\": %.1f, \"p99_us\": %.1f, \"mean_us\": %.1f}", names[v], lat[steps / 2],
               lat[(int)(0.99 * steps) < steps ? (int)(0.99 * steps) : steps - 1], sum / steps);
    }
    printf("}\n");
    fflush(stdout);

    gs_step_graph_destroy(c.g0);
    gs_step_graph_destroy(c.g1);
    for (int i = 0; i < M; i++) {
        (void)hipFree(c.par_dev[i]);
        (void)hipHostFree(c.par_host[i]);
    }
    (void)hipFree(c.table_dev);
    (void)hipHostFree(tables);
    (void)hipFree(c.plane_base_dev);
    (void)hipFree(pool);
    (void)hipStreamDestroy(c.stream);
    gs_free_code(c.code);
    free(lat);
    free(perm);
    free(base_host);
    return 0;
}
