// Synchronisation of the checkpoint / restore pipelines, the stream pool and
// the grouped-launch descriptor ring, checked on the CPU.
//
// This program is linked with the library's own sources (host code only) and
// REPLACES the HIP runtime: every runtime call the library makes lands in the
// recorder below, which keeps, for every enqueued operation, a vector clock
// (one counter per stream, plus what the host has observed through its own
// waits).  Kernels do not run; copies are done with memcpy so that their
// ranges are checked by AddressSanitizer.  From the record the tests decide
// "A happens before B" exactly as the stream and event semantics define it,
// independent of timing, and assert the orderings the pipelines rely on:
//
//   checkpoint  copy of chunk c's parity      after  encode of chunk c
//               encode of chunk c + depth     after  copy of chunk c (slot reuse)
//   restore     reconstruct of chunk c        after  H2D of chunk c's parity
//               H2D of chunk c + depth        after  reconstruct of chunk c
//   paged       the same four relations for gs_checkpoint_paged / gs_restore_paged,
//               whose chunks are windows of page slots moved by strided copies
//   failure     a refused call enqueues nothing; after a runtime failure part of
//               the way, gs_pipe_sync still waits for everything that was enqueued
//   pool        every chunk's launch after what was enqueued on the caller's
//               stream before the call; what the caller enqueues afterwards
//               after every chunk
//   ring        a descriptor slot is rewritten only after the launch that
//               read it (four calls earlier) has been waited for
//
// Built and run by tests/test_host_sanitize.py (ASan + UBSan, no GPU).
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <vector>

#include "../include/ghostserve_ec.h"

namespace {

constexpr int kMaxStreams = 96;  // stream 0 = the null stream

enum OpKind { LAUNCH, COPY, HOSTWRITE };

struct Op {
    OpKind kind;
    int stream;                 // -1 for host writes
    int seq;                    // position among this stream's operations (1-based)
    int vc[kMaxStreams];        // what this operation is ordered after, per stream
    const void *dst, *src;      // copies
    size_t bytes;
    hipMemcpyKind dir;
    size_t shmem;               // launches: dynamic LDS asked for
    unsigned grid_x, grid_y;
};

struct Event { int vc[kMaxStreams]; bool recorded; };

int stream_vc[kMaxStreams][kMaxStreams];  // per stream: what its next operation is ordered after
int host_vc[kMaxStreams];                 // what the host has waited for
bool stream_live[kMaxStreams];
std::vector<Op> ops;
std::vector<Event *> events;
int fail_malloc_after = -1;               // >= 0: that many device allocations succeed, then they fail
int fail_copy_after = -1;                 // >= 0: that many async copies succeed, then they fail

int sid(hipStream_t s) { return static_cast<int>(reinterpret_cast<uintptr_t>(s)); }

void join(int *into, const int *from)
{
    for (int i = 0; i < kMaxStreams; ++i) into[i] = std::max(into[i], from[i]);
}

Op &enqueue(OpKind kind, hipStream_t stream)
{
    const int s = sid(stream);
    join(stream_vc[s], host_vc);  // enqueued after everything the host has already seen finish
    stream_vc[s][s] += 1;
    Op op{};
    op.kind = kind;
    op.stream = s;
    op.seq = stream_vc[s][s];
    std::memcpy(op.vc, stream_vc[s], sizeof op.vc);
    ops.push_back(op);
    return ops.back();
}

// a finished before b started, by stream order and event edges alone
bool before(const Op &a, const Op &b) { return b.vc[a.stream] >= a.seq && &a != &b; }

void reset_record()
{
    ops.clear();
}

}  // namespace

// ------------------------------------------------------------ the recorder, as the HIP runtime
extern "C" {

hipError_t hipMalloc(void **p, size_t n)
{
    if (fail_malloc_after == 0) { *p = nullptr; return hipErrorOutOfMemory; }
    if (fail_malloc_after > 0) --fail_malloc_after;
    *p = std::malloc(n ? n : 1);
    return *p ? hipSuccess : hipErrorOutOfMemory;
}
hipError_t hipFree(void *p) { std::free(p); return hipSuccess; }
hipError_t hipHostMalloc(void **p, size_t n, unsigned) { *p = std::malloc(n ? n : 1); return *p ? hipSuccess : hipErrorOutOfMemory; }
hipError_t hipHostFree(void *p) { std::free(p); return hipSuccess; }

hipError_t hipStreamCreateWithFlags(hipStream_t *s, unsigned)
{
    for (int i = 1; i < kMaxStreams; ++i)
        if (!stream_live[i]) {
            stream_live[i] = true;
            std::memset(stream_vc[i], 0, sizeof stream_vc[i]);
            *s = reinterpret_cast<hipStream_t>(static_cast<uintptr_t>(i));
            return hipSuccess;
        }
    return hipErrorOutOfMemory;
}
hipError_t hipStreamDestroy(hipStream_t s) { stream_live[sid(s)] = false; return hipSuccess; }
hipError_t hipStreamSynchronize(hipStream_t s) { join(host_vc, stream_vc[sid(s)]); return hipSuccess; }
hipError_t hipStreamWaitEvent(hipStream_t s, hipEvent_t e, unsigned)
{
    Event *ev = reinterpret_cast<Event *>(e);
    if (ev->recorded) join(stream_vc[sid(s)], ev->vc);
    return hipSuccess;
}

hipError_t hipEventCreateWithFlags(hipEvent_t *e, unsigned)
{
    Event *ev = new Event();
    events.push_back(ev);
    *e = reinterpret_cast<hipEvent_t>(ev);
    return hipSuccess;
}
hipError_t hipEventCreate(hipEvent_t *e) { return hipEventCreateWithFlags(e, 0); }
hipError_t hipEventDestroy(hipEvent_t e)
{
    Event *ev = reinterpret_cast<Event *>(e);
    events.erase(std::find(events.begin(), events.end(), ev));
    delete ev;
    return hipSuccess;
}
hipError_t hipEventRecord(hipEvent_t e, hipStream_t s)
{
    Event *ev = reinterpret_cast<Event *>(e);
    join(stream_vc[sid(s)], host_vc);
    std::memcpy(ev->vc, stream_vc[sid(s)], sizeof ev->vc);
    ev->recorded = true;
    return hipSuccess;
}
hipError_t hipEventSynchronize(hipEvent_t e)
{
    Event *ev = reinterpret_cast<Event *>(e);
    if (ev->recorded) join(host_vc, ev->vc);
    return hipSuccess;
}
hipError_t hipEventElapsedTime(float *ms, hipEvent_t, hipEvent_t) { *ms = 0.0f; return hipSuccess; }

hipError_t hipMemcpyAsync(void *dst, const void *src, size_t n, hipMemcpyKind kind, hipStream_t s)
{
    if (fail_copy_after == 0) return hipErrorUnknown;
    if (fail_copy_after > 0) --fail_copy_after;
    Op &op = enqueue(COPY, s);
    op.dst = dst;
    op.src = src;
    op.bytes = n;
    op.dir = kind;
    std::memcpy(dst, src, n);
    return hipSuccess;
}

hipError_t hipMemcpy2DAsync(void *dst, size_t dpitch, const void *src, size_t spitch, size_t width, size_t height,
                            hipMemcpyKind kind, hipStream_t s)
{
    Op &op = enqueue(COPY, s);
    op.dst = dst;
    op.src = src;
    op.bytes = width * height;
    op.dir = kind;
    for (size_t r = 0; r < height; ++r)
        std::memcpy(static_cast<uint8_t *>(dst) + r * dpitch, static_cast<const uint8_t *>(src) + r * spitch, width);
    return hipSuccess;
}

hipError_t hipGetLastError(void) { return hipSuccess; }

static dim3 cfg_grid, cfg_block;
static size_t cfg_shmem;
static hipStream_t cfg_stream;
hipError_t __hipPushCallConfiguration(dim3 grid, dim3 block, size_t shmem, hipStream_t stream)
{
    cfg_grid = grid; cfg_block = block; cfg_shmem = shmem; cfg_stream = stream;
    return hipSuccess;
}
hipError_t __hipPopCallConfiguration(dim3 *grid, dim3 *block, size_t *shmem, hipStream_t *stream)
{
    *grid = cfg_grid; *block = cfg_block; *shmem = cfg_shmem; *stream = cfg_stream;
    return hipSuccess;
}
hipError_t hipLaunchKernel(const void *, dim3 grid, dim3 block, void **, size_t shmem, hipStream_t s)
{
    if (grid.x == 0 || grid.y == 0 || grid.z == 0 || block.x != 256) return hipErrorInvalidConfiguration;
    Op &op = enqueue(LAUNCH, s);
    op.shmem = shmem;
    op.grid_x = grid.x;
    op.grid_y = grid.y;
    return hipSuccess;
}

void **__hipRegisterFatBinary(const void *) { static void *handle; return &handle; }
void __hipRegisterFunction(void **, const void *, char *, const char *, unsigned, void *, void *, void *, void *, int *) {}
void __hipUnregisterFatBinary(void **) {}

hipError_t hipStreamBeginCapture(hipStream_t, hipStreamCaptureMode) { return hipSuccess; }
hipError_t hipStreamEndCapture(hipStream_t, hipGraph_t *g) { *g = reinterpret_cast<hipGraph_t>(std::malloc(1)); return hipSuccess; }
hipError_t hipGraphInstantiate(hipGraphExec_t *x, hipGraph_t, hipGraphNode_t *, char *, size_t)
{
    *x = reinterpret_cast<hipGraphExec_t>(std::malloc(1));
    return hipSuccess;
}
hipError_t hipGraphLaunch(hipGraphExec_t, hipStream_t s) { enqueue(LAUNCH, s); return hipSuccess; }
hipError_t hipGraphExecDestroy(hipGraphExec_t x) { std::free(x); return hipSuccess; }
hipError_t hipGraphDestroy(hipGraph_t g) { std::free(g); return hipSuccess; }

}  // extern "C"

// ------------------------------------------------------------ the checks
#define EXPECT(cond) do { if (!(cond)) { std::printf("FAIL line %d: %s\n", __LINE__, #cond); return 1; } } while (0)

static std::vector<const Op *> launches_on(int stream)
{
    std::vector<const Op *> v;
    for (const Op &o : ops)
        if (o.kind == LAUNCH && o.stream == stream) v.push_back(&o);
    return v;
}

static int check_pipelines(int k, int m, int kind, size_t chunk, int depth, size_t S, const std::vector<int> &erased)
{
    gs_code *code = nullptr;
    if (kind == GS_RDP) EXPECT(gs_make_rdp_code(k, 64, &code) == GS_OK);
    else EXPECT(gs_make_code(k, m, kind, &code) == GS_OK);
    gs_pipe *pipe = nullptr;
    EXPECT(gs_pipe_create(code, chunk, depth, &pipe) == GS_OK);
    hipStream_t cs;
    EXPECT(hipStreamCreateWithFlags(&cs, 0) == hipSuccess);
    std::vector<void *> dev(k + m), host(m);
    for (auto &p : dev) p = std::malloc(S);
    for (auto &p : host) p = std::malloc(S);
    const size_t n = (S + chunk - 1) / chunk;

    for (int rep = 0; rep < 2; ++rep) {  // the second call starts with every slot in use
        reset_record();
        EXPECT(gs_pipe_set_timing(pipe, rep) == GS_OK);
        EXPECT(gs_checkpoint(pipe, dev.data(), S, host.data(), cs) == GS_OK);
        const std::vector<const Op *> enc = launches_on(sid(cs));
        EXPECT(!enc.empty() && enc.size() % n == 0);
        const size_t L = enc.size() / n;  // launches per chunk (wide codes take several)
        std::vector<std::vector<const Op *>> copies(n);
        for (const Op &o : ops)
            if (o.kind == COPY) {
                EXPECT(o.dir == hipMemcpyDeviceToHost);
                bool found = false;
                for (int i = 0; i < m && !found; ++i) {
                    const uint8_t *base = static_cast<const uint8_t *>(host[i]);
                    const uint8_t *d = static_cast<const uint8_t *>(o.dst);
                    if (d >= base && d < base + S) {
                        const size_t c = static_cast<size_t>(d - base) / chunk;
                        EXPECT(static_cast<size_t>(d - base) == c * chunk && o.bytes == std::min(chunk, S - c * chunk));
                        copies[c].push_back(&o);
                        found = true;
                    }
                }
                EXPECT(found);
            }
        for (size_t c = 0; c < n; ++c) {
            EXPECT(copies[c].size() == static_cast<size_t>(m));
            for (const Op *cp : copies[c]) {
                EXPECT(before(*enc[c * L + L - 1], *cp));                          // parity is copied after it is made
                if (c + depth < n) EXPECT(before(*cp, *enc[(c + depth) * L]));      // a slot is reused after it is drained
                if (c + 1 < n && depth > 1) EXPECT(!before(*cp, *enc[(c + 1) * L + L - 1]));  // the next encode does not wait for it
            }
        }
        EXPECT(gs_pipe_sync(pipe) == GS_OK);
    }

    // restore of `erased`: the parity shards among the k lowest-numbered survivors come back over PCIe
    size_t parity_read = 0;
    for (int r = 0, taken = 0; r < k + m && taken < k; ++r)
        if (std::find(erased.begin(), erased.end(), r) == erased.end()) {
            ++taken;
            if (r >= k) ++parity_read;
        }
    for (int rep = 0; rep < 2; ++rep) {
        reset_record();
        std::vector<void *> shards(dev);
        EXPECT(gs_restore(pipe, shards.data(), host.data(), erased.data(), static_cast<int>(erased.size()), S, cs) == GS_OK);
        const std::vector<const Op *> rec = launches_on(sid(cs));
        EXPECT(!rec.empty() && rec.size() % n == 0);
        const size_t L = rec.size() / n;
        std::vector<std::vector<const Op *>> h2d(n);
        for (const Op &o : ops)
            if (o.kind == COPY) {
                EXPECT(o.dir == hipMemcpyHostToDevice);
                bool found = false;
                for (int i = 0; i < m && !found; ++i) {
                    const uint8_t *base = static_cast<const uint8_t *>(host[i]);
                    const uint8_t *s = static_cast<const uint8_t *>(o.src);
                    if (s >= base && s < base + S) {
                        h2d[static_cast<size_t>(s - base) / chunk].push_back(&o);
                        found = true;
                    }
                }
                EXPECT(found);
            }
        for (size_t c = 0; c < n; ++c) {
            if (kind == GS_RDP) EXPECT(h2d[c].size() <= 2);
            else EXPECT(h2d[c].size() == parity_read);
            for (const Op *cp : h2d[c]) {
                EXPECT(before(*cp, *rec[c * L]));                            // parity is on the device before it is used
                if (c + depth < n) for (const Op *later : h2d[c + depth]) EXPECT(before(*rec[c * L + L - 1], *later));
                if (c + 1 < n && depth > 1) for (const Op *next : h2d[c + 1]) EXPECT(!before(*rec[c * L], *next));
            }
        }
        EXPECT(gs_pipe_sync(pipe) == GS_OK);
    }
    // a checkpoint straight after a restore: the first encodes wait for the last reconstructs' slots
    reset_record();
    EXPECT(gs_checkpoint(pipe, dev.data(), S, host.data(), cs) == GS_OK);
    EXPECT(launches_on(sid(cs)).size() % n == 0);

    gs_pipe_destroy(pipe);
    for (void *p : dev) std::free(p);
    for (void *p : host) std::free(p);
    EXPECT(hipStreamDestroy(cs) == hipSuccess);
    gs_free_code(code);
    return 0;
}

static int check_pool(int n_streams, int n_chunks)
{
    const int k = 4, m = 2;
    gs_code *code = nullptr;
    EXPECT(gs_make_code(k, m, GS_CAUCHY, &code) == GS_OK);
    gs_pool *pool = nullptr;
    EXPECT(gs_pool_create(n_streams, &pool) == GS_OK);
    hipStream_t cs;
    EXPECT(hipStreamCreateWithFlags(&cs, 0) == hipSuccess);
    std::vector<void *> ptrs(static_cast<size_t>(n_chunks) * (k + m));
    for (size_t i = 0; i < ptrs.size(); ++i) ptrs[i] = reinterpret_cast<void *>(0x100000000ull + 0x200000ull * i);
    std::vector<const void *> data;
    std::vector<void *> parity;
    for (int c = 0; c < n_chunks; ++c) {
        for (int j = 0; j < k; ++j) data.push_back(ptrs[static_cast<size_t>(c) * (k + m) + j]);
        for (int i = 0; i < m; ++i) parity.push_back(ptrs[static_cast<size_t>(c) * (k + m) + k + i]);
    }
    std::vector<size_t> bytes(n_chunks, 4096);
    if (n_chunks > 2) bytes[1] = 0;  // an empty chunk launches nothing
    for (int which = 0; which < 2; ++which) {
        reset_record();
        int64_t marker_src = 1, marker_dst = 0;
        EXPECT(hipMemcpyAsync(&marker_dst, &marker_src, 8, hipMemcpyHostToHost, cs) == hipSuccess);  // "before the call"
        if (which == 0) {
            EXPECT(gs_encode_streams(code, pool, n_chunks, data.data(), parity.data(), bytes.data(), cs) == GS_OK);
        } else {
            const int erased[2] = {1, 4};
            EXPECT(gs_reconstruct_streams(code, pool, n_chunks, ptrs.data(), erased, 2, bytes.data(), cs) == GS_OK);
        }
        EXPECT(hipMemcpyAsync(&marker_dst, &marker_src, 8, hipMemcpyHostToHost, cs) == hipSuccess);  // "after the call"
        const Op *first = nullptr, *last = nullptr;
        int launches = 0;
        for (const Op &o : ops)
            if (o.kind == COPY) (first ? last : first) = &o;
        EXPECT(first && last);
        for (const Op &o : ops)
            if (o.kind == LAUNCH) {
                ++launches;
                EXPECT(o.stream != sid(cs));
                EXPECT(before(*first, o) && before(o, *last));
            }
        EXPECT(launches == n_chunks - (n_chunks > 2 ? 1 : 0));
    }
    gs_pool_destroy(pool);
    EXPECT(hipStreamDestroy(cs) == hipSuccess);
    gs_free_code(code);
    return 0;
}

// Which launches ask for LDS they never use (to keep 2 or 3 workgroups on a CU instead of 8): bulk
// launches of the contiguous, Horner, grouped and RDP kernels at the default launch shape, by kernel
// variant; never the paged gather, never a small launch, never with the switch off.
static int check_occupancy_reservation()
{
    const size_t two = 65536, three = 53248, four = 40960;
    hipStream_t s = nullptr;
    EXPECT(hipStreamCreateWithFlags(&s, 0) == hipSuccess);
    std::vector<void *> ptr(24);
    for (size_t i = 0; i < ptr.size(); ++i) ptr[i] = reinterpret_cast<void *>(0x100000000ull + 0x800000000ull * i);
    auto lds_of = [&](gs_code *code, size_t bytes, const int *erased, int n_erased) -> long {
        reset_record();
        int k = 0, m = 0;
        if (gs_code_params(code, &k, &m) != GS_OK) return -1;
        const int rc = n_erased ? gs_reconstruct(code, ptr.data(), erased, n_erased, bytes, s)
                                : gs_encode(code, ptr.data(), ptr.data() + k, bytes, s);
        if (rc != GS_OK || ops.size() != 1 || ops[0].kind != LAUNCH) return -1;
        return static_cast<long>(ops[0].shmem);
    };
    const size_t big = 1ull << 30, small = 1ull << 20;
    const int e1[1] = {1}, e2[2] = {1, 3}, e3[3] = {0, 1, 2}, e4[4] = {0, 1, 2, 3}, e14[2] = {1, 6}, e02[2] = {0, 2};
    struct Case { int k, m, kind; const int *erased; int n_erased; size_t want; } cases[] = {
        {4, 2, GS_CAUCHY, nullptr, 0, four},  {4, 2, GS_CAUCHY, e2, 2, four},  {4, 2, GS_CAUCHY, e1, 1, three},   // the 8B workload
        {8, 2, GS_CAUCHY, nullptr, 0, three}, {8, 2, GS_CAUCHY, e2, 2, four},                                     // the 70B workload
        {8, 3, GS_CAUCHY, nullptr, 0, four},  {8, 3, GS_CAUCHY, e3, 3, four},  {16, 3, GS_CAUCHY, e3, 3, four},
        {4, 1, GS_CAUCHY, nullptr, 0, three}, {2, 1, GS_CAUCHY, nullptr, 0, four}, {1, 1, GS_CAUCHY, nullptr, 0, 0},
        {2, 2, GS_CAUCHY, nullptr, 0, four},
        {8, 4, GS_CAUCHY, nullptr, 0, 0},     {8, 4, GS_CAUCHY, e4, 4, 0},     {1, 4, GS_CAUCHY, nullptr, 0, three},   // four rows: left alone
        {8, 3, GS_POWER, nullptr, 0, three},  {2, 2, GS_POWER, nullptr, 0, three},                                 // Horner kernel
        {2, 2, GS_RDP, nullptr, 0, 0},        {4, 2, GS_RDP, nullptr, 0, three}, {6, 2, GS_RDP, e1, 1, three},
        {4, 2, GS_RDP, e2, 2, four},          {6, 2, GS_RDP, e02, 2, four},      {6, 2, GS_RDP, e14, 2, three},   // cells of many syndromes; of few
        {10, 2, GS_RDP, nullptr, 0, two},     {10, 2, GS_RDP, e2, 2, three},     {10, 2, GS_RDP, e1, 1, two},
        {16, 2, GS_RDP, e2, 2, two},
    };
    for (const Case &c : cases) {
        gs_code *code = nullptr;
        EXPECT(gs_make_code(c.k, c.m, c.kind, &code) == GS_OK);
        size_t unit = 1;
        if (c.kind == GS_RDP) {
            int p = 0;
            size_t cell = 0;
            EXPECT(gs_rdp_prime(code, &p) == GS_OK && gs_rdp_cell_bytes(code, &cell) == GS_OK);
            unit = cell * static_cast<size_t>(p - 1);
        }
        const size_t B = big / unit * unit, Sm = small < unit ? unit : small / unit * unit;
        EXPECT(lds_of(code, B, c.erased, c.n_erased) == static_cast<long>(c.want));
        EXPECT(lds_of(code, Sm, c.erased, c.n_erased) == 0);           // a small launch keeps every wavefront
        EXPECT(gs_set_occupancy_cap(0) == GS_OK);
        EXPECT(lds_of(code, B, c.erased, c.n_erased) == 0);
        EXPECT(gs_set_occupancy_cap(1) == GS_OK);
        EXPECT(gs_set_launch_shape(1, 0, -1, -1) == GS_OK);            // another vector count: no reservation
        EXPECT(lds_of(code, B, c.erased, c.n_erased) == 0 || c.kind == GS_RDP);
        EXPECT(gs_set_launch_shape(0, 0, -1, -1) == GS_OK);
        EXPECT(lds_of(code, B, c.erased, c.n_erased) == static_cast<long>(c.want));   // the shape knobs left the switch on
        // without the kernel forms by size a rebuild of three shards of a wide code is three lookup rows again
        EXPECT(gs_set_size_forms(0) == GS_OK);
        EXPECT(lds_of(code, B, c.erased, c.n_erased) == static_cast<long>(c.k == 16 && c.n_erased == 3 ? 0 : c.want));
        EXPECT(gs_set_size_forms(1) == GS_OK);
        gs_free_code(code);
    }
    // where the reservation starts: 6144 workgroups of 8 KiB per stream for two and more rows, 12288 for one row
    {
        gs_code *two_rows = nullptr, *one_row = nullptr;
        EXPECT(gs_make_code(8, 2, GS_CAUCHY, &two_rows) == GS_OK && gs_make_code(4, 1, GS_CAUCHY, &one_row) == GS_OK);
        EXPECT(lds_of(two_rows, 6144ull * 8192, nullptr, 0) == static_cast<long>(three));
        EXPECT(lds_of(two_rows, 6144ull * 8192, e2, 2) == static_cast<long>(four));
        EXPECT(lds_of(two_rows, 6112ull * 8192, nullptr, 0) == 0);
        EXPECT(lds_of(one_row, 12288ull * 8192, nullptr, 0) == static_cast<long>(three));
        EXPECT(lds_of(one_row, 12256ull * 8192, nullptr, 0) == 0);
        EXPECT(lds_of(two_rows, 12256ull * 8192, e1, 1) == 0);   // one lost shard: a one-row launch
        gs_free_code(two_rows);
        gs_free_code(one_row);
        // the Horner kernel from 6144 workgroups, RDP from 96 MiB per disk (workgroups x (p - 1) >= 49152)
        gs_code *power = nullptr, *rdp = nullptr;
        EXPECT(gs_make_code(8, 3, GS_POWER, &power) == GS_OK && gs_make_code(8, 2, GS_RDP, &rdp) == GS_OK);
        EXPECT(lds_of(power, 6144ull * 8192, nullptr, 0) == static_cast<long>(three));
        EXPECT(lds_of(power, 6112ull * 8192, nullptr, 0) == 0);
        size_t cell = 0;
        EXPECT(gs_rdp_cell_bytes(rdp, &cell) == GS_OK && cell == 32768);
        EXPECT(lds_of(rdp, 308 * 10 * cell, nullptr, 0) == static_cast<long>(two));   // p = 11: 4928 x 10
        EXPECT(lds_of(rdp, 306 * 10 * cell, nullptr, 0) == 0);                                            // 4896 x 10
        gs_free_code(power);
        gs_free_code(rdp);
    }
    // the paged gather keeps full occupancy
    struct Paged { int k, m; int pages_per_shard; size_t want; } paged[] = {
        {4, 2, 4096, 0}, {8, 3, 4096, 0}, {8, 2, 4096, 0}, {16, 1, 4096, 0}, {8, 2, 16, 0},
    };
    for (const Paged &c : paged) {
        gs_code *code = nullptr;
        EXPECT(gs_make_code(c.k, c.m, GS_CAUCHY, &code) == GS_OK);
        reset_record();
        EXPECT(gs_encode_paged(code, reinterpret_cast<const void *const *>(ptr[0]), 64, 32768, 1 << 20,
                               reinterpret_cast<const int32_t *>(ptr[1]), c.pages_per_shard, ptr.data() + 4, s) == GS_OK);
        EXPECT(ops.size() == 1 && ops[0].kind == LAUNCH && ops[0].shmem == c.want);
        // a rebuild into pages never reserves
        const int lost[1] = {1};
        reset_record();
        EXPECT(gs_reconstruct_paged(code, reinterpret_cast<const void *const *>(ptr[0]), 64, 32768, 1 << 20,
                                    reinterpret_cast<const int32_t *>(ptr[1]), c.pages_per_shard, ptr.data() + 4, lost, 1, s) == GS_OK);
        EXPECT(ops.size() == 1 && ops[0].kind == LAUNCH && ops[0].shmem == 0);
        gs_free_code(code);
    }
    EXPECT(hipStreamDestroy(s) == hipSuccess);
    return 0;
}

static int check_ring()
{
    const int k = 8, m = 2, n_chunks = 5;
    gs_code *code = nullptr;
    EXPECT(gs_make_code(k, m, GS_CAUCHY, &code) == GS_OK);
    gs_batch *batch = nullptr;
    EXPECT(gs_batch_create(code, n_chunks, &batch) == GS_OK);
    hipStream_t st[3];
    for (hipStream_t &s : st) EXPECT(hipStreamCreateWithFlags(&s, 0) == hipSuccess);
    std::vector<const void *> data(static_cast<size_t>(n_chunks) * k);
    std::vector<void *> parity(static_cast<size_t>(n_chunks) * m), shards(static_cast<size_t>(n_chunks) * (k + m));
    for (size_t i = 0; i < data.size(); ++i) data[i] = reinterpret_cast<void *>(0x100000000ull + 0x200000ull * i);
    for (size_t i = 0; i < parity.size(); ++i) parity[i] = reinterpret_cast<void *>(0x900000000ull + 0x200000ull * i);
    for (size_t i = 0; i < shards.size(); ++i) shards[i] = reinterpret_cast<void *>(0x100000000ull + 0x200000ull * i);
    const std::vector<size_t> bytes = {4096, 0, 100, 1 << 20, 17};
    reset_record();
    const int calls = 11;
    for (int c = 0; c < calls; ++c) {
        hipStream_t cs = st[c % 3];  // slot reuse (every 4th call) then falls on a different stream
        if (c % 4 == 2) {
            const int erased[2] = {0, 9};
            EXPECT(gs_reconstruct_batch(batch, n_chunks, shards.data(), erased, 2, bytes.data(), cs) == GS_OK);
        } else {
            EXPECT(gs_encode_batch(batch, n_chunks, data.data(), parity.data(), bytes.data(), cs) == GS_OK);
        }
    }
    // one descriptor upload and one launch per call; the upload into a slot is ordered after the
    // launch that last read that slot, which across streams only the host's wait can establish
    std::vector<const Op *> uploads, launches;
    for (const Op &o : ops) (o.kind == COPY ? uploads : launches).push_back(&o);
    EXPECT(uploads.size() == static_cast<size_t>(calls) && launches.size() == static_cast<size_t>(calls));
    std::map<const void *, const Op *> last_reader;
    int slots = 0;
    for (int c = 0; c < calls; ++c) {
        EXPECT(before(*uploads[c], *launches[c]));
        auto it = last_reader.find(uploads[c]->dst);
        if (it == last_reader.end()) ++slots;
        else EXPECT(before(*it->second, *uploads[c]));
        last_reader[uploads[c]->dst] = launches[c];
    }
    EXPECT(slots == 4);
    EXPECT(gs_encode_batch(batch, n_chunks + 1, data.data(), parity.data(), bytes.data(), st[0]) == GS_EINVAL);
    gs_batch_destroy(batch);
    for (hipStream_t s : st) EXPECT(hipStreamDestroy(s) == hipSuccess);
    gs_free_code(code);
    return 0;
}

// The grouped launch with an RDP code: the same ring discipline, and every chunk
// is checked (whole stripes, no output on an input) before anything is enqueued.
static int check_rdp_ring()
{
    const int k = 4, n_chunks = 3;
    gs_code *code = nullptr;
    EXPECT(gs_make_rdp_code(k, 64, &code) == GS_OK);  // p = 5: stripes of 256 bytes
    gs_batch *batch = nullptr;
    EXPECT(gs_batch_create(code, n_chunks, &batch) == GS_OK);
    hipStream_t s = nullptr;
    EXPECT(hipStreamCreateWithFlags(&s, 0) == hipSuccess);
    std::vector<const void *> data(static_cast<size_t>(n_chunks) * k);
    std::vector<void *> parity(static_cast<size_t>(n_chunks) * 2), shards(static_cast<size_t>(n_chunks) * (k + 2));
    for (size_t i = 0; i < data.size(); ++i) data[i] = reinterpret_cast<void *>(0x100000000ull + 0x200000ull * i);
    for (size_t i = 0; i < parity.size(); ++i) parity[i] = reinterpret_cast<void *>(0x900000000ull + 0x200000ull * i);
    for (size_t i = 0; i < shards.size(); ++i) shards[i] = reinterpret_cast<void *>(0x100000000ull + 0x200000ull * i);
    std::vector<size_t> bytes = {256 * 40, 0, 256};
    reset_record();
    for (int c = 0; c < 6; ++c) {
        if (c & 1) {
            const int erased[2] = {1, 4};
            EXPECT(gs_reconstruct_batch(batch, n_chunks, shards.data(), erased, 2, bytes.data(), s) == GS_OK);
        } else {
            EXPECT(gs_encode_batch(batch, n_chunks, data.data(), parity.data(), bytes.data(), s) == GS_OK);
        }
    }
    size_t uploads = 0, launches = 0;
    for (const Op &o : ops) (o.kind == COPY ? uploads : launches) += 1;
    EXPECT(uploads == 6 && launches == 6);
    reset_record();
    bytes[2] = 256 + 64;  // a cell too many
    EXPECT(gs_encode_batch(batch, n_chunks, data.data(), parity.data(), bytes.data(), s) == GS_EINVAL);
    bytes[2] = 256;
    void *keep = parity[0];
    parity[0] = const_cast<void *>(data[1]);  // chunk 0 writes its row parity over its own data
    EXPECT(gs_encode_batch(batch, n_chunks, data.data(), parity.data(), bytes.data(), s) == GS_EINVAL);
    parity[0] = keep;
    const int three[3] = {0, 1, 2};
    EXPECT(gs_reconstruct_batch(batch, n_chunks, shards.data(), three, 3, bytes.data(), s) != GS_OK);
    EXPECT(ops.empty());
    bytes = {0, 0, 0};
    EXPECT(gs_encode_batch(batch, n_chunks, data.data(), parity.data(), bytes.data(), s) == GS_OK && ops.empty());
    gs_batch_destroy(batch);
    EXPECT(hipStreamDestroy(s) == hipSuccess);
    gs_free_code(code);
    return 0;
}

// device allocations that fail part of the way through object creation: nothing leaks (ASan's leak
// check at exit), nothing is handed back
static int check_allocation_failures()
{
    gs_code *code = nullptr;
    EXPECT(gs_make_code(4, 2, GS_CAUCHY, &code) == GS_OK);
    for (int ok = 0; ok < 2; ++ok) {
        fail_malloc_after = ok;
        gs_pipe *pipe = reinterpret_cast<gs_pipe *>(1);
        gs_batch *batch = reinterpret_cast<gs_batch *>(1);
        const int rp = gs_pipe_create(code, 4096, 3, &pipe);
        fail_malloc_after = ok;
        const int rb = gs_batch_create(code, 16, &batch);
        fail_malloc_after = -1;
        if (ok == 0) {
            EXPECT(rp == GS_ENOMEM && pipe == nullptr);
            EXPECT(rb == GS_ENOMEM && batch == nullptr);
        } else {
            EXPECT(rp == GS_OK && pipe != nullptr && rb == GS_OK && batch != nullptr);
            gs_pipe_destroy(pipe);
            gs_batch_destroy(batch);
        }
    }
    gs_free_code(code);
    return 0;
}

// the captured per-step checkpoint: one launch and m copies are recorded at creation, the private
// capture stream is gone afterwards, and a failing capture hands nothing back
static int check_step_graph()
{
    const int k = 4, m = 2, n_planes = 3, pps = 5;
    const size_t page = 2048, out_bytes = static_cast<size_t>(n_planes) * pps * page;
    gs_code *code = nullptr;
    EXPECT(gs_make_code(k, m, GS_CAUCHY, &code) == GS_OK);
    std::vector<void *> par(m), host(m);
    for (auto &p : par) p = std::malloc(out_bytes);
    for (auto &p : host) p = std::malloc(out_bytes);
    for (auto &p : par) std::memset(p, 0x11, out_bytes);
    void *planes = reinterpret_cast<void *>(0x100000), *table = reinterpret_cast<void *>(0x200000);
    reset_record();
    gs_step_graph *g = nullptr;
    EXPECT(gs_step_graph_create(code, static_cast<const void *const *>(planes), n_planes, page, 64,
                                static_cast<const int32_t *>(table), pps, par.data(), host.data(), &g) == GS_OK && g != nullptr);
    int launches = 0, copies = 0;
    for (const Op &o : ops) (o.kind == LAUNCH ? launches : copies) += 1;
    EXPECT(launches == 1 && copies == m);
    for (int i = 1; i < kMaxStreams; ++i) EXPECT(!stream_live[i]);
    EXPECT(gs_step_graph_launch(g, nullptr) == GS_OK);
    gs_step_graph_destroy(g);
    g = reinterpret_cast<gs_step_graph *>(1);
    EXPECT(gs_step_graph_create(code, static_cast<const void *const *>(planes), n_planes, 24, 64,
                                static_cast<const int32_t *>(table), pps, par.data(), host.data(), &g) == GS_EINVAL && g == nullptr);
    for (int i = 1; i < kMaxStreams; ++i) EXPECT(!stream_live[i]);
    for (void *p : par) std::free(p);
    for (void *p : host) std::free(p);
    gs_free_code(code);
    return 0;
}

// Checkpoint / restore over a paged pool: chunks are windows of `spc` page slots of every plane;
// a chunk's parity moves as one strided copy per parity shard, inside the dense layout
// [plane][pages_per_shard][page].
static int check_paged_pipelines(int depth)
{
    const int k = 4, m = 2, n_planes = 3, pps = 11, spc = 4;
    const size_t page = 256, row = static_cast<size_t>(pps) * page, S = n_planes * row;
    const size_t chunk = static_cast<size_t>(n_planes) * page * spc + 32;  // the 32 extra bytes hold no whole slot
    const size_t n = (pps + spc - 1) / spc;
    gs_code *code = nullptr;
    EXPECT(gs_make_code(k, m, GS_CAUCHY, &code) == GS_OK);
    gs_pipe *pipe = nullptr;
    EXPECT(gs_pipe_create(code, chunk, depth, &pipe) == GS_OK);
    hipStream_t cs;
    EXPECT(hipStreamCreateWithFlags(&cs, 0) == hipSuccess);
    std::vector<void *> host(m), dev_par(m);
    for (auto &p : host) p = std::malloc(S);
    for (auto &p : dev_par) p = std::malloc(S);
    for (auto &p : host) std::memset(p, 0x22, S);
    const void *const *planes = reinterpret_cast<const void *const *>(0x100000);
    const int32_t *table = reinterpret_cast<const int32_t *>(0x200000);

    for (int rep = 0; rep < 2; ++rep) {
        reset_record();
        EXPECT(gs_checkpoint_paged(pipe, planes, n_planes, page, 64, table, pps, host.data(), cs) == GS_OK);
        const std::vector<const Op *> enc = launches_on(sid(cs));
        EXPECT(enc.size() == n);
        std::vector<std::vector<const Op *>> copies(n);
        for (const Op &o : ops)
            if (o.kind == COPY) {
                EXPECT(o.dir == hipMemcpyDeviceToHost);
                bool found = false;
                for (int i = 0; i < m && !found; ++i) {
                    const uint8_t *base = static_cast<const uint8_t *>(host[i]);
                    const uint8_t *d = static_cast<const uint8_t *>(o.dst);
                    if (d >= base && d < base + S) {
                        const size_t c = static_cast<size_t>(d - base) / (spc * page);
                        const size_t slots = std::min<size_t>(spc, pps - c * spc);
                        EXPECT(static_cast<size_t>(d - base) == c * spc * page && o.bytes == n_planes * slots * page);
                        copies[c].push_back(&o);
                        found = true;
                    }
                }
                EXPECT(found);
            }
        for (size_t c = 0; c < n; ++c) {
            EXPECT(copies[c].size() == static_cast<size_t>(m));
            for (const Op *cp : copies[c]) {
                EXPECT(before(*enc[c], *cp));
                if (c + depth < n) EXPECT(before(*cp, *enc[c + depth]));
                if (c + 1 < n) EXPECT(!before(*cp, *enc[c + 1]));
            }
        }
        EXPECT(gs_pipe_sync(pipe) == GS_OK);
    }
    // data shard 1 and parity shard 0 lost: parity 1 comes back from the host, parity 0 is rebuilt
    // into the caller's dense device buffer
    const int erased[2] = {1, 4};
    for (int rep = 0; rep < 2; ++rep) {
        reset_record();
        EXPECT(gs_restore_paged(pipe, planes, n_planes, page, 64, table, pps, host.data(), dev_par.data(), erased, 2, cs) == GS_OK);
        const std::vector<const Op *> rec = launches_on(sid(cs));
        EXPECT(rec.size() == n);
        std::vector<const Op *> h2d;
        for (const Op &o : ops)
            if (o.kind == COPY) {
                EXPECT(o.dir == hipMemcpyHostToDevice);
                const uint8_t *base = static_cast<const uint8_t *>(host[1]);
                const uint8_t *sp = static_cast<const uint8_t *>(o.src);
                EXPECT(sp >= base && sp < base + S && static_cast<size_t>(sp - base) == h2d.size() * spc * page);
                h2d.push_back(&o);
            }
        EXPECT(h2d.size() == n);
        for (size_t c = 0; c < n; ++c) {
            EXPECT(before(*h2d[c], *rec[c]));
            if (c + depth < n) EXPECT(before(*rec[c], *h2d[c + depth]));
            if (c + 1 < n) EXPECT(!before(*rec[c], *h2d[c + 1]));
        }
        EXPECT(gs_pipe_sync(pipe) == GS_OK);
    }
    // refusals: nothing is enqueued
    reset_record();
    EXPECT(gs_restore_paged(pipe, planes, n_planes, page, 64, table, pps, host.data(), nullptr, erased, 2, cs) == GS_EINVAL);
    const int three[3] = {0, 1, 2};
    EXPECT(gs_restore_paged(pipe, planes, n_planes, page, 64, table, pps, host.data(), dev_par.data(), three, 3, cs) == GS_ETOOMANY);
    EXPECT(gs_checkpoint_paged(pipe, planes, n_planes, 8 * page, 64, table, pps, host.data(), cs) == GS_EINVAL);  // no whole slot fits a chunk
    EXPECT(gs_checkpoint_paged(pipe, planes, n_planes, page + 8, 64, table, pps, host.data(), cs) == GS_EINVAL);
    EXPECT(gs_checkpoint_paged(pipe, planes, n_planes, page, 64, table, 0, host.data(), cs) == GS_OK);            // empty
    EXPECT(ops.empty());
    gs_pipe_destroy(pipe);
    for (void *p : host) std::free(p);
    for (void *p : dev_par) std::free(p);
    EXPECT(hipStreamDestroy(cs) == hipSuccess);
    gs_free_code(code);
    return 0;
}

// A call that is refused enqueues nothing; a runtime failure part of the way leaves a pipe whose
// gs_pipe_sync waits for everything that did get enqueued.
static int check_pipeline_failures()
{
    gs_code *rdp = nullptr;
    EXPECT(gs_make_rdp_code(4, 64, &rdp) == GS_OK);  // p = 5: stripes of 256 bytes
    gs_pipe *pipe = nullptr;
    EXPECT(gs_pipe_create(rdp, 1024, 2, &pipe) == GS_OK);
    hipStream_t cs;
    EXPECT(hipStreamCreateWithFlags(&cs, 0) == hipSuccess);
    const size_t S = 5 * 1024;
    std::vector<void *> dev(6), host(2);
    for (auto &p : dev) p = std::malloc(S);
    for (auto &p : host) p = std::malloc(S);
    reset_record();
    // three whole chunks and a last one that is not a whole number of stripes: refused up front
    EXPECT(gs_checkpoint(pipe, dev.data(), 3 * 1024 + 128, host.data(), cs) == GS_EINVAL);
    EXPECT(ops.empty());
    EXPECT(gs_pipe_done_event(pipe) == nullptr && gs_pipe_sync(pipe) == GS_OK);
    const int erased[2] = {0, 5};
    EXPECT(gs_restore(pipe, dev.data(), host.data(), erased, 2, 3 * 1024 + 128, cs) == GS_EINVAL);
    EXPECT(ops.empty());

    // the fourth copy fails: two chunks are complete, the third has its kernel and one copy
    for (int which = 0; which < 2; ++which) {
        reset_record();
        std::memset(host_vc, 0, sizeof host_vc);
        fail_copy_after = which == 0 ? 5 : 2;
        const int rc = which == 0 ? gs_checkpoint(pipe, dev.data(), S, host.data(), cs)
                                  : gs_restore(pipe, dev.data(), host.data(), erased, 2, S, cs);
        fail_copy_after = -1;
        EXPECT(rc == GS_EHIP);
        EXPECT(!ops.empty());
        EXPECT(gs_pipe_done_event(pipe) != nullptr);
        EXPECT(gs_pipe_sync(pipe) == GS_OK);
        for (const Op &o : ops) EXPECT(host_vc[o.stream] >= o.seq);  // the host has waited for every one of them
    }
    gs_pipe_destroy(pipe);
    for (void *p : dev) std::free(p);
    for (void *p : host) std::free(p);
    EXPECT(hipStreamDestroy(cs) == hipSuccess);
    gs_free_code(rdp);
    return 0;
}

int main()
{
    if (check_pipelines(4, 2, GS_CAUCHY, 4096, 2, 10 * 4096 + 100, {1, 3})) return 1;
    if (check_pipelines(8, 3, GS_CAUCHY, 1024, 4, 23 * 1024, {0, 9, 5})) return 1;
    if (check_pipelines(4, 1, GS_CAUCHY, 2048, 3, 2048, {2})) return 1;          // a single chunk
    if (check_pipelines(40, 6, GS_VANDERMONDE, 512, 2, 5 * 512 + 16, {39, 41})) return 1;  // several launches per chunk
    if (check_pipelines(4, 2, GS_RDP, 1024, 2, 7 * 1024, {0, 5})) return 1;       // p = 5: stripes of 256 bytes
    if (check_pipelines(8, 3, GS_POWER, 4096, 2, 3 * 4096 + 1, {8})) return 1;    // Horner encode, lost parity
    if (check_paged_pipelines(2) || check_paged_pipelines(3)) return 1;
    if (check_pipeline_failures()) return 1;
    if (check_pool(4, 11) || check_pool(16, 3) || check_pool(1, 5)) return 1;
    if (check_occupancy_reservation()) return 1;
    if (check_ring()) return 1;
    if (check_rdp_ring()) return 1;
    if (check_step_graph()) return 1;
    if (check_allocation_failures()) return 1;
    for (int i = 1; i < kMaxStreams; ++i) EXPECT(!stream_live[i]);  // every stream was destroyed
    EXPECT(events.empty());                                          // and every event
    std::printf("OK\n");
    return 0;
}
