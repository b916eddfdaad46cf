/*
 * Measurements of the erasure-code library taken from plain C, with no
 * interpreter in the timed loops.  bench.py runs this program as a child
 * process and copies its JSON into the benchmark line; it can also be run by
 * hand or under rocprofv3 (the program itself goes directly after "--").
 *
 *   bench_native decode [steps] [layers]
 *       The streaming-decode checkpoint (Section 4.2: parity is updated as the
 *       KV cache of new tokens is generated; Section 5: streams and graphs) at
 *       the decode-step shape of the paged pool: one plane per layer and K/V,
 *       16-token blocks of 2 KiB token slots, 64 sequences in k = 4 shards,
 *       m = 1.  Two kinds of figures:
 *       (a) launch -> stream-idle latency of ONE step on the host clock, for the
 *           eager launch, eager + D2H copy, eager straight into pinned memory,
 *           and graph replays built several ways;
 *       (b) the step as a STREAM: all steps enqueued back to back with no host
 *           wait, parity going through a ring of device buffers and a ring of
 *           pinned host buffers, the D2H copy of step s on a copy stream beside
 *           the encode of step s+1; sustained time per step from the host
 *           clock, completion latency of each step from events.
 *   bench_native many
 *       Many small chunks at once (Section 5: one stream per chunk): enqueue ->
 *       stream-idle time of one launch per chunk, the stream pool and the
 *       grouped launch, for three shapes.
 *
 * Pool contents do not matter for timing (the code is data-independent); the
 * buffers are filled with a byte pattern.
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <time.h>

#include "include/ghostserve_ec.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "HIP error %d (%s) at line %d\n", (int)e_, hipGetErrorString(e_), __LINE__); return 2; } } while (0)
#define CHECK_GS(x) do { int r_ = (x); if (r_ != GS_OK) { fprintf(stderr, "gs error %d (%s) at line %d\n", r_, gs_strerror(r_), __LINE__); return 3; } } while (0)

enum { K = 4, M = 1, SEQS = 64, SEQS_PER_SHARD = SEQS / K, BLOCK_TOKENS = 16, SLOT_BYTES = 8 * 128 * 2 };
enum { RING = 4, GRAPH_STEPS = 8 };

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

static void print_stats(const char *name, double *lat, int n)
{
    qsort(lat, n, sizeof(double), cmp_double);
    double sum = 0;
    for (int s = 0; s < n; s++) sum += lat[s];
    const int i99 = (int)(0.99 * n) < n ? (int)(0.99 * n) : n - 1;
    printf(", \"%s\": {\"p50_us\": %.1f, \"p99_us\": %.1f, \"mean_us\": %.1f}", name, lat[n / 2], lat[i99], sum / n);
}

static uint32_t rng_state = 0x67530102u;
static uint32_t next_u32(void)
{
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 17;
    rng_state ^= rng_state << 5;
    return rng_state;
}

/* Pseudo-random bytes for a device buffer (a 16 MiB block repeated): the HBM rate depends on the data,
 * buffers of one constant byte run about 2 points faster than real ones. */
static int fill_random(void *dev, size_t bytes)
{
    const size_t block = (size_t)16 << 20;
    uint32_t *h = (uint32_t *)malloc(block);
    if (h == NULL) return 1;
    for (size_t i = 0; i < block / 4; i++) h[i] = next_u32() * 2654435761u ^ next_u32() << 16;
    for (size_t off = 0; off < bytes; off += block)
        if (hipMemcpy((char *)dev + off, h, bytes - off < block ? bytes - off : block, hipMemcpyHostToDevice) != hipSuccess) {
            free(h);
            return 1;
        }
    free(h);
    return 0;
}

struct step_ctx {
    gs_code *code;
    void **plane_base_dev;
    int n_planes;
    int64_t pages_per_plane;
    int32_t *table_dev;          /* the table the single-step variants read (rewritten before every step) */
    int32_t *table_ahead_dev;    /* GRAPH_STEPS tables the multi-step graph reads                         */
    void *par_dev[M];
    void *par_host[M];
    size_t out_bytes;
    hipStream_t stream;
    gs_step_graph *g0, *g1;
    hipGraphExec_t own, own_uploaded, multi;
};

typedef int (*step_fn)(struct step_ctx *);

static int encode_into(struct step_ctx *c, const int32_t *table, void *const *parity, hipStream_t s)
{
    return gs_encode_paged(c->code, (const void *const *)c->plane_base_dev, c->n_planes, SLOT_BYTES, c->pages_per_plane,
                           table, SEQS_PER_SHARD, parity, s);
}

static int eager(struct step_ctx *c) { return encode_into(c, c->table_dev, c->par_dev, c->stream); }

static int eager_d2h(struct step_ctx *c)
{
    const int rc = eager(c);
    if (rc != GS_OK) return rc;
    for (int i = 0; i < M; i++)
        if (hipMemcpyAsync(c->par_host[i], c->par_dev[i], c->out_bytes, hipMemcpyDeviceToHost, c->stream) != hipSuccess)
            return GS_EHIP;
    return GS_OK;
}

static int eager_pinned(struct step_ctx *c) { return encode_into(c, c->table_dev, c->par_host, c->stream); }
static int graph(struct step_ctx *c) { return gs_step_graph_launch(c->g0, c->stream); }
static int graph_d2h(struct step_ctx *c) { return gs_step_graph_launch(c->g1, c->stream); }
static int graph_own(struct step_ctx *c) { return hipGraphLaunch(c->own, c->stream) == hipSuccess ? GS_OK : GS_EHIP; }
static int graph_uploaded(struct step_ctx *c) { return hipGraphLaunch(c->own_uploaded, c->stream) == hipSuccess ? GS_OK : GS_EHIP; }

/* capture `n` encodes on the measuring stream itself (tables table + i*SEQS) and instantiate */
static int capture_steps(struct step_ctx *c, const int32_t *table, int n, hipGraphExec_t *exec)
{
    hipGraph_t g = NULL;
    CHECK_HIP(hipStreamBeginCapture(c->stream, hipStreamCaptureModeThreadLocal));
    int rc = GS_OK;
    for (int i = 0; i < n && rc == GS_OK; i++) rc = encode_into(c, table + (size_t)i * SEQS, c->par_dev, c->stream);
    const hipError_t e = hipStreamEndCapture(c->stream, &g);
    CHECK_GS(rc);
    CHECK_HIP(e);
    CHECK_HIP(hipGraphInstantiateWithFlags(exec, g, 0));
    CHECK_HIP(hipGraphDestroy(g));
    return 0;
}

static int run_decode(int steps, int layers)
{
    const int warm = 50;
    struct step_ctx c;
    memset(&c, 0, sizeof c);
    c.n_planes = 2 * layers;
    const int total_steps = steps + warm + GRAPH_STEPS;
    const int blocks_per_seq = (total_steps + BLOCK_TOKENS - 1) / BLOCK_TOKENS;
    const int64_t n_blocks = (int64_t)SEQS * blocks_per_seq;
    c.pages_per_plane = n_blocks * BLOCK_TOKENS;
    const size_t plane_bytes = (size_t)c.pages_per_plane * SLOT_BYTES;
    c.out_bytes = (size_t)c.n_planes * SEQS_PER_SHARD * SLOT_BYTES;

    CHECK_GS(gs_make_code(K, M, GS_CAUCHY, &c.code));
    CHECK_HIP(hipStreamCreateWithFlags(&c.stream, hipStreamNonBlocking));

    /* the pool: one allocation, plane p at offset p * plane_bytes */
    uint8_t *pool = NULL;
    CHECK_HIP(hipMalloc((void **)&pool, plane_bytes * c.n_planes));
    if (fill_random(pool, plane_bytes * c.n_planes)) return 3;
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
    int32_t *tables = NULL, *tables_all_dev = NULL;
    const size_t table_bytes = sizeof(int32_t) * SEQS;
    CHECK_HIP(hipHostMalloc((void **)&tables, table_bytes * total_steps, hipHostMallocDefault));
    for (int s = 0; s < total_steps; s++)
        for (int q = 0; q < SEQS; q++)
            tables[(size_t)s * SEQS + q] = perm[(size_t)(s / BLOCK_TOKENS) * SEQS + q] * BLOCK_TOKENS + s % BLOCK_TOKENS;
    CHECK_HIP(hipMalloc((void **)&c.table_dev, table_bytes));
    CHECK_HIP(hipMalloc((void **)&c.table_ahead_dev, table_bytes * GRAPH_STEPS));
    CHECK_HIP(hipMalloc((void **)&tables_all_dev, table_bytes * total_steps));
    CHECK_HIP(hipMemcpy(tables_all_dev, tables, table_bytes * total_steps, hipMemcpyHostToDevice));

    for (int i = 0; i < M; i++) {
        CHECK_HIP(hipMalloc(&c.par_dev[i], c.out_bytes));
        CHECK_HIP(hipHostMalloc(&c.par_host[i], c.out_bytes, hipHostMallocDefault));
    }
    CHECK_HIP(hipMemcpy(c.table_dev, tables, table_bytes, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(c.table_ahead_dev, tables, table_bytes * GRAPH_STEPS, hipMemcpyHostToDevice));
    CHECK_GS(gs_step_graph_create(c.code, (const void *const *)c.plane_base_dev, c.n_planes, SLOT_BYTES, c.pages_per_plane,
                                  c.table_dev, SEQS_PER_SHARD, c.par_dev, NULL, &c.g0));
    CHECK_GS(gs_step_graph_create(c.code, (const void *const *)c.plane_base_dev, c.n_planes, SLOT_BYTES, c.pages_per_plane,
                                  c.table_dev, SEQS_PER_SHARD, c.par_dev, c.par_host, &c.g1));
    if (capture_steps(&c, c.table_dev, 1, &c.own)) return 4;
    if (capture_steps(&c, c.table_dev, 1, &c.own_uploaded)) return 4;
    CHECK_HIP(hipGraphUpload(c.own_uploaded, c.stream));
    if (capture_steps(&c, c.table_ahead_dev, GRAPH_STEPS, &c.multi)) return 4;
    CHECK_HIP(hipStreamSynchronize(c.stream));

    /* ---- (a) one step at a time: launch -> stream idle on the host clock */
    /* the last one is the eager step again with the kernel form of small launches switched off */
    static const char *names[] = {"eager", "eager_d2h", "eager_pinned", "graph", "graph_d2h", "graph_captured_on_launch_stream",
                                  "graph_uploaded", "eager_bulk_kernel_form"};
    const step_fn fns[] = {eager, eager_d2h, eager_pinned, graph, graph_d2h, graph_own, graph_uploaded, eager};
    double *lat = (double *)malloc(sizeof(double) * steps);
    printf("{\"steps\": %d, \"layers\": %d, \"new_kv_bytes_per_step\": %zu, \"parity_bytes_per_step\": %zu",
           steps, layers, (size_t)K * c.out_bytes, (size_t)M * c.out_bytes);
    for (int v = 0; v < 8; v++) {
        CHECK_GS(gs_set_size_forms(v != 7));
        for (int s = 0; s < steps + warm; s++) {
            CHECK_HIP(hipMemcpyAsync(c.table_dev, tables + (size_t)s * SEQS, table_bytes, hipMemcpyHostToDevice, c.stream));
            CHECK_HIP(hipStreamSynchronize(c.stream));
            const double t0 = now_us();
            CHECK_GS(fns[v](&c));
            CHECK_HIP(hipStreamSynchronize(c.stream));
            const double t1 = now_us();
            if (s >= warm) lat[s - warm] = t1 - t0;
        }
        print_stats(names[v], lat, steps);
    }
    CHECK_GS(gs_set_size_forms(1));
    /* a graph that holds GRAPH_STEPS steps: the engine writes that many tables ahead, one replay
     * encodes them all; time per step = replay -> idle / GRAPH_STEPS */
    {
        const int reps = steps / GRAPH_STEPS > 8 ? steps / GRAPH_STEPS : 8;
        for (int r = 0; r < reps + 8; r++) {
            const int s0 = (r * GRAPH_STEPS) % (total_steps - GRAPH_STEPS);
            CHECK_HIP(hipMemcpyAsync(c.table_ahead_dev, tables + (size_t)s0 * SEQS, table_bytes * GRAPH_STEPS,
                                     hipMemcpyHostToDevice, c.stream));
            CHECK_HIP(hipStreamSynchronize(c.stream));
            const double t0 = now_us();
            CHECK_HIP(hipGraphLaunch(c.multi, c.stream));
            CHECK_HIP(hipStreamSynchronize(c.stream));
            const double t1 = now_us();
            if (r >= 8) lat[r - 8] = (t1 - t0) / GRAPH_STEPS;
        }
        char name[64];
        snprintf(name, sizeof name, "graph_of_%d_steps_per_step", GRAPH_STEPS);
        print_stats(name, lat, reps);
    }

    /* ---- (b) the step as a stream: no host wait between steps */
    {
        void *ring_dev[RING], *ring_host[RING];
        hipEvent_t filled[RING], drained[RING];
        hipStream_t copy_stream;
        CHECK_HIP(hipStreamCreateWithFlags(&copy_stream, hipStreamNonBlocking));  /* default priority */
        for (int i = 0; i < RING; i++) {
            CHECK_HIP(hipMalloc(&ring_dev[i], c.out_bytes));
            CHECK_HIP(hipHostMalloc(&ring_host[i], c.out_bytes, hipHostMallocDefault));
            CHECK_HIP(hipEventCreateWithFlags(&filled[i], hipEventDisableTiming));
            CHECK_HIP(hipEventCreateWithFlags(&drained[i], hipEventDisableTiming));
        }
        hipEvent_t *t_begin = (hipEvent_t *)malloc(sizeof(hipEvent_t) * steps);
        hipEvent_t *t_end = (hipEvent_t *)malloc(sizeof(hipEvent_t) * steps);
        for (int s = 0; s < steps; s++) {
            CHECK_HIP(hipEventCreate(&t_begin[s]));
            CHECK_HIP(hipEventCreate(&t_end[s]));
        }
        /* plain pinned D2H rate of one step's parity, back to back, for the PCIe fraction */
        double plain_us;
        {
            for (int s = 0; s < 20; s++)
                CHECK_HIP(hipMemcpyAsync(ring_host[s % RING], ring_dev[s % RING], c.out_bytes, hipMemcpyDeviceToHost, copy_stream));
            CHECK_HIP(hipStreamSynchronize(copy_stream));
            const double t0 = now_us();
            for (int s = 0; s < steps; s++)
                CHECK_HIP(hipMemcpyAsync(ring_host[s % RING], ring_dev[s % RING], c.out_bytes, hipMemcpyDeviceToHost, copy_stream));
            CHECK_HIP(hipStreamSynchronize(copy_stream));
            plain_us = (now_us() - t0) / steps;
        }
        double total_us = 0, enqueue_us = 0;
        for (int pass = 0; pass < 2; pass++) {  /* pass 0 warms up */
            const int n = pass == 0 ? warm : steps, first = pass == 0 ? 0 : warm;
            CHECK_HIP(hipStreamSynchronize(c.stream));
            CHECK_HIP(hipStreamSynchronize(copy_stream));
            const double t0 = now_us();
            for (int s = 0; s < n; s++) {
                const int slot = s % RING;
                /* the device buffer of this slot is free once its previous copy has finished */
                if (s >= RING) CHECK_HIP(hipStreamWaitEvent(c.stream, drained[slot], 0));
                if (pass) CHECK_HIP(hipEventRecord(t_begin[s], c.stream));
                CHECK_GS(encode_into(&c, tables_all_dev + (size_t)(first + s) * SEQS, &ring_dev[slot], c.stream));
                CHECK_HIP(hipEventRecord(filled[slot], c.stream));
                CHECK_HIP(hipStreamWaitEvent(copy_stream, filled[slot], 0));
                CHECK_HIP(hipMemcpyAsync(ring_host[slot], ring_dev[slot], c.out_bytes, hipMemcpyDeviceToHost, copy_stream));
                if (pass) CHECK_HIP(hipEventRecord(t_end[s], copy_stream));
                CHECK_HIP(hipEventRecord(drained[slot], copy_stream));
            }
            const double t1 = now_us();
            CHECK_HIP(hipStreamSynchronize(c.stream));
            CHECK_HIP(hipStreamSynchronize(copy_stream));
            const double t2 = now_us();
            if (pass) {
                total_us = t2 - t0;
                enqueue_us = t1 - t0;
            }
        }
        for (int s = 0; s < steps; s++) {
            float ms = 0;
            CHECK_HIP(hipEventElapsedTime(&ms, t_begin[s], t_end[s]));
            lat[s] = ms * 1e3;
        }
        printf(", \"stream_ring\": {\"ring\": %d, \"sustained_us_per_step\": %.2f, \"host_enqueue_us_per_step\": %.2f, "
               "\"plain_pinned_d2h_us_per_step\": %.2f, \"frac_of_plain_d2h\": %.3f, \"parity_GBps\": %.2f",
               RING, total_us / steps, enqueue_us / steps, plain_us, plain_us / (total_us / steps),
               M * c.out_bytes / (total_us / steps) / 1e3);
        print_stats("completion_latency_from_events", lat, steps);
        printf("}");
        /* the same stream with the kernel writing its parity straight into the pinned ring: one stream,
         * no copy, no events */
        for (int pass = 0; pass < 2; pass++) {
            const int n = pass == 0 ? warm : steps, first = pass == 0 ? 0 : warm;
            CHECK_HIP(hipStreamSynchronize(c.stream));
            const double t0 = now_us();
            for (int s = 0; s < n; s++)
                CHECK_GS(encode_into(&c, tables_all_dev + (size_t)(first + s) * SEQS, &ring_host[s % RING], c.stream));
            const double t1 = now_us();
            CHECK_HIP(hipStreamSynchronize(c.stream));
            const double t2 = now_us();
            if (pass)
                printf(", \"stream_into_pinned_ring\": {\"ring\": %d, \"sustained_us_per_step\": %.2f, "
                       "\"host_enqueue_us_per_step\": %.2f, \"parity_GBps\": %.2f}",
                       RING, (t2 - t0) / steps, (t1 - t0) / steps, M * c.out_bytes / ((t2 - t0) / steps) / 1e3);
        }
        /* encode and D2H copy on ONE stream, no events: nothing overlaps, but the host makes two calls per step */
        for (int pass = 0; pass < 2; pass++) {
            const int n = pass == 0 ? warm : steps, first = pass == 0 ? 0 : warm;
            CHECK_HIP(hipStreamSynchronize(c.stream));
            const double t0 = now_us();
            for (int s = 0; s < n; s++) {
                CHECK_GS(encode_into(&c, tables_all_dev + (size_t)(first + s) * SEQS, &ring_dev[s % RING], c.stream));
                CHECK_HIP(hipMemcpyAsync(ring_host[s % RING], ring_dev[s % RING], c.out_bytes, hipMemcpyDeviceToHost, c.stream));
            }
            const double t1 = now_us();
            CHECK_HIP(hipStreamSynchronize(c.stream));
            const double t2 = now_us();
            if (pass)
                printf(", \"stream_one_stream_encode_then_copy\": {\"sustained_us_per_step\": %.2f, "
                       "\"host_enqueue_us_per_step\": %.2f, \"parity_GBps\": %.2f}",
                       (t2 - t0) / steps, (t1 - t0) / steps, M * c.out_bytes / ((t2 - t0) / steps) / 1e3);
        }
        /* and encode only, back to back, into the device ring: what the GPU side of a step costs */
        for (int pass = 0; pass < 2; pass++) {
            const int n = pass == 0 ? warm : steps, first = pass == 0 ? 0 : warm;
            CHECK_HIP(hipStreamSynchronize(c.stream));
            const double t0 = now_us();
            for (int s = 0; s < n; s++)
                CHECK_GS(encode_into(&c, tables_all_dev + (size_t)(first + s) * SEQS, &ring_dev[s % RING], c.stream));
            const double t1 = now_us();
            CHECK_HIP(hipStreamSynchronize(c.stream));
            const double t2 = now_us();
            if (pass)
                printf(", \"stream_encode_only\": {\"sustained_us_per_step\": %.2f, \"host_enqueue_us_per_step\": %.2f}",
                       (t2 - t0) / steps, (t1 - t0) / steps);
        }
        /* graph replays back to back, no host wait: the one-step graph and the graph of GRAPH_STEPS steps */
        for (int v = 0; v < 2; v++) {
            hipGraphExec_t exec = v == 0 ? c.own : c.multi;
            const int per = v == 0 ? 1 : GRAPH_STEPS, n = steps / per;
            for (int r = 0; r < 10; r++) CHECK_HIP(hipGraphLaunch(exec, c.stream));
            CHECK_HIP(hipStreamSynchronize(c.stream));
            const double t0 = now_us();
            for (int r = 0; r < n; r++) CHECK_HIP(hipGraphLaunch(exec, c.stream));
            const double t1 = now_us();
            CHECK_HIP(hipStreamSynchronize(c.stream));
            const double t2 = now_us();
            printf(", \"stream_graph_of_%d\": {\"sustained_us_per_step\": %.2f, \"host_enqueue_us_per_step\": %.2f}",
                   per, (t2 - t0) / (n * per), (t1 - t0) / (n * per));
        }
        for (int s = 0; s < steps; s++) {
            (void)hipEventDestroy(t_begin[s]);
            (void)hipEventDestroy(t_end[s]);
        }
        free(t_begin);
        free(t_end);
        for (int i = 0; i < RING; i++) {
            (void)hipFree(ring_dev[i]);
            (void)hipHostFree(ring_host[i]);
            (void)hipEventDestroy(filled[i]);
            (void)hipEventDestroy(drained[i]);
        }
        (void)hipStreamDestroy(copy_stream);
    }
    printf("}\n");
    fflush(stdout);

    gs_step_graph_destroy(c.g0);
    gs_step_graph_destroy(c.g1);
    (void)hipGraphExecDestroy(c.own);
    (void)hipGraphExecDestroy(c.own_uploaded);
    (void)hipGraphExecDestroy(c.multi);
    for (int i = 0; i < M; i++) {
        (void)hipFree(c.par_dev[i]);
        (void)hipHostFree(c.par_host[i]);
    }
    (void)hipFree(c.table_dev);
    (void)hipFree(c.table_ahead_dev);
    (void)hipFree(tables_all_dev);
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

/* ---- many chunks at once --------------------------------------------------- */

static double median_of(double *v, int n)
{
    qsort(v, n, sizeof(double), cmp_double);
    return v[n / 2];
}

static int run_many(void)
{
    static const struct { int k, m, n_erased, erased[2]; size_t S; int n; } shapes[] = {
        {8, 2, 1, {3, 0}, (size_t)2 << 20, 64},
        {8, 2, 2, {3, 6}, (size_t)256 << 10, 256},
        {4, 1, 0, {0, 0}, (size_t)512 << 10, 64},
    };
    const int iters = 15, warm = 3;
    hipStream_t stream;
    CHECK_HIP(hipStreamCreateWithFlags(&stream, hipStreamNonBlocking));
    printf("[");
    for (size_t sh = 0; sh < sizeof shapes / sizeof shapes[0]; sh++) {
        const int k = shapes[sh].k, m = shapes[sh].m, n = shapes[sh].n, e = shapes[sh].n_erased;
        const size_t S = shapes[sh].S;
        gs_code *code = NULL;
        gs_batch *batch = NULL;
        gs_pool *pool = NULL;
        CHECK_GS(gs_make_code(k, m, GS_CAUCHY, &code));
        CHECK_GS(gs_batch_create(code, n, &batch));
        CHECK_GS(gs_pool_create(16, &pool));
        uint8_t *big = NULL;
        CHECK_HIP(hipMalloc((void **)&big, (size_t)n * (k + m) * S));
        if (fill_random(big, (size_t)n * (k + m) * S)) return 3;
        void **shards = (void **)malloc(sizeof(void *) * n * (k + m));
        const void **data = (const void **)malloc(sizeof(void *) * n * k);
        void **par = (void **)malloc(sizeof(void *) * n * m);
        size_t *sizes = (size_t *)malloc(sizeof(size_t) * n);
        for (int c = 0; c < n; c++) {
            for (int r = 0; r < k + m; r++) shards[c * (k + m) + r] = big + ((size_t)c * (k + m) + r) * S;
            for (int j = 0; j < k; j++) data[c * k + j] = shards[c * (k + m) + j];
            for (int i = 0; i < m; i++) par[c * m + i] = shards[c * (k + m) + k + i];
            sizes[c] = S;
        }
        double t[4][32];
        for (int form = 0; form < 4; form++) {
            /* form 3: one launch per chunk again, with the kernel form of small launches switched off */
            CHECK_GS(gs_set_size_forms(form != 3));
            for (int it = 0; it < iters + warm; it++) {
                CHECK_HIP(hipStreamSynchronize(stream));
                const double t0 = now_us();
                if (form == 0 || form == 3) {
                    for (int c = 0; c < n; c++)
                        CHECK_GS(e ? gs_reconstruct(code, shards + (size_t)c * (k + m), shapes[sh].erased, e, S, stream)
                                   : gs_encode(code, data + (size_t)c * k, par + (size_t)c * m, S, stream));
                } else if (form == 1) {
                    CHECK_GS(e ? gs_reconstruct_streams(code, pool, n, shards, shapes[sh].erased, e, sizes, stream)
                               : gs_encode_streams(code, pool, n, data, par, sizes, stream));
                } else {
                    CHECK_GS(e ? gs_reconstruct_batch(batch, n, shards, shapes[sh].erased, e, sizes, stream)
                               : gs_encode_batch(batch, n, data, par, sizes, stream));
                }
                CHECK_HIP(hipStreamSynchronize(stream));
                if (it >= warm) t[form][it - warm] = (now_us() - t0) * 1e-3;
            }
        }
        CHECK_GS(gs_set_size_forms(1));
        const double traffic = (double)(k + (e ? e : m)) * S * n;
        const double grouped = median_of(t[2], iters);
        printf("%s{\"op\": \"%s\", \"k\": %d, \"m\": %d, \"n_erased\": %d, \"chunks\": %d, \"shard_bytes\": %zu, "
               "\"one_launch_per_chunk_ms\": %.4f, \"stream_pool_16_ms\": %.4f, \"grouped_launch_ms\": %.4f, "
               "\"grouped_launch_traffic_GBps\": %.1f, \"one_launch_per_chunk_bulk_kernel_form_ms\": %.4f}",
               sh ? ", " : "", e ? "reconstruct" : "encode", k, m, e, n, S, median_of(t[0], iters), median_of(t[1], iters),
               grouped, traffic / grouped / 1e6, median_of(t[3], iters));
        gs_batch_destroy(batch);
        gs_pool_destroy(pool);
        gs_free_code(code);
        (void)hipFree(big);
        free(shards);
        free(data);
        free(par);
        free(sizes);
    }
    printf("]\n");
    fflush(stdout);
    (void)hipStreamDestroy(stream);
    return 0;
}

int main(int argc, char **argv)
{
    if (argc >= 2 && strcmp(argv[1], "decode") == 0) {
        const int steps = argc > 2 ? atoi(argv[2]) : 1000;
        const int layers = argc > 3 ? atoi(argv[3]) : 32;
        if (steps >= 8 && steps <= 100000 && layers >= 1 && layers <= 512) return run_decode(steps, layers);
    } else if (argc == 2 && strcmp(argv[1], "many") == 0) {
        return run_many();
    }
    fprintf(stderr, "usage: bench_native decode [steps 8..100000] [layers 1..512] | bench_native many\n");
    return 1;
}
