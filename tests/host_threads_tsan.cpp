// Thread safety of the library's host side, checked with ThreadSanitizer and
// no GPU.  The header promises: a gs_code is immutable and may be shared
// between threads; pipes, batches and pools belong to one thread at a time;
// the launch knobs are atomics; the last HIP error is per thread; the
// allocation-free grouped encode looks its device array up once per device
// under a lock.  Here several threads use one set of codes at the same time,
// each with objects of its own, while one of them keeps changing the knobs.
// The HIP runtime is replaced by stubs that are themselves thread-safe and
// touch only memory the test owns, so every report would be the library's.
#include <hip/hip_runtime_api.h>

#include <atomic>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <thread>
#include <vector>

#include "../include/ghostserve_ec.h"

// ------------------------------------------------------------ a thread-safe stand-in for the runtime
extern "C" {

static std::atomic<uintptr_t> next_stream{1};
static unsigned char fake_symbol[GS_STATIC_MAX_CHUNKS * 256];

hipError_t hipMalloc(void **p, size_t n) { *p = std::malloc(n ? n : 1); return *p ? hipSuccess : hipErrorOutOfMemory; }
hipError_t hipFree(void *p) { std::free(p); return hipSuccess; }
hipError_t hipHostMalloc(void **p, size_t n, unsigned) { return hipMalloc(p, n); }
hipError_t hipHostFree(void *p) { std::free(p); return hipSuccess; }
hipError_t hipStreamCreateWithFlags(hipStream_t *s, unsigned)
{
    *s = reinterpret_cast<hipStream_t>(next_stream.fetch_add(1));
    return hipSuccess;
}
hipError_t hipStreamDestroy(hipStream_t) { return hipSuccess; }
hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
hipError_t hipStreamWaitEvent(hipStream_t, hipEvent_t, unsigned) { return hipSuccess; }
hipError_t hipEventCreateWithFlags(hipEvent_t *e, unsigned)
{
    *e = reinterpret_cast<hipEvent_t>(std::malloc(1));
    return *e ? hipSuccess : hipErrorOutOfMemory;
}
hipError_t hipEventCreate(hipEvent_t *e) { return hipEventCreateWithFlags(e, 0); }
hipError_t hipEventDestroy(hipEvent_t e) { std::free(e); return hipSuccess; }
hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
hipError_t hipEventElapsedTime(float *ms, hipEvent_t, hipEvent_t) { *ms = 0.0f; return hipSuccess; }
// every buffer the test hands to the library is real host memory, so copies are carried out: a
// copy into memory another thread owns would be reported
hipError_t hipMemcpyAsync(void *dst, const void *src, size_t n, hipMemcpyKind, hipStream_t)
{
    std::memcpy(dst, src, n);
    return hipSuccess;
}
hipError_t hipMemcpy2DAsync(void *dst, size_t dpitch, const void *src, size_t spitch, size_t width, size_t height,
                            hipMemcpyKind, hipStream_t)
{
    for (size_t r = 0; r < height; ++r)
        std::memcpy(static_cast<uint8_t *>(dst) + r * dpitch, static_cast<const uint8_t *>(src) + r * spitch, width);
    return hipSuccess;
}
hipError_t hipGetLastError(void) { return hipSuccess; }
hipError_t hipGetDevice(int *d) { *d = 0; return hipSuccess; }
hipError_t hipGetSymbolAddress(void **p, const void *) { *p = fake_symbol; return hipSuccess; }

static thread_local dim3 cfg_grid, cfg_block;
static thread_local size_t cfg_shmem;
static thread_local hipStream_t cfg_stream;
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
static std::atomic<long> launches{0};
hipError_t hipLaunchKernel(const void *, dim3 grid, dim3 block, void **, size_t, hipStream_t)
{
    if (grid.x == 0 || grid.y == 0 || grid.z == 0 || block.x == 0) return hipErrorInvalidConfiguration;
    launches.fetch_add(1, std::memory_order_relaxed);
    return hipSuccess;
}
void **__hipRegisterFatBinary(const void *) { static void *handle; return &handle; }
void __hipRegisterFunction(void **, const void *, char *, const char *, unsigned, void *, void *, void *, void *, int *) {}
void __hipRegisterVar(void **, void *, char *, const char *, int, size_t, int, int) {}
void __hipUnregisterFatBinary(void **) {}
hipError_t hipStreamBeginCapture(hipStream_t, hipStreamCaptureMode) { return hipSuccess; }
hipError_t hipStreamEndCapture(hipStream_t, hipGraph_t *g) { *g = reinterpret_cast<hipGraph_t>(std::malloc(1)); return hipSuccess; }
hipError_t hipGraphInstantiate(hipGraphExec_t *x, hipGraph_t, hipGraphNode_t *, char *, size_t)
{
    *x = reinterpret_cast<hipGraphExec_t>(std::malloc(1));
    return hipSuccess;
}
hipError_t hipGraphLaunch(hipGraphExec_t, hipStream_t) { launches.fetch_add(1, std::memory_order_relaxed); return hipSuccess; }
hipError_t hipGraphExecDestroy(hipGraphExec_t x) { std::free(x); return hipSuccess; }
hipError_t hipGraphDestroy(hipGraph_t g) { std::free(g); return hipSuccess; }

}  // extern "C"

// ------------------------------------------------------------ the test
static std::atomic<int> failures{0};
#define EXPECT(cond)                                                              \
    do {                                                                          \
        if (!(cond)) {                                                            \
            std::fprintf(stderr, "FAIL line %d: %s\n", __LINE__, #cond);          \
            failures.fetch_add(1);                                                \
            return;                                                               \
        }                                                                         \
    } while (0)

namespace {

constexpr int K = 8, M = 3;
constexpr size_t S = 24 * 1024;   // whole stripes of the RDP code below (p = 7: 6 cells of 1 KiB) and of 4 KiB chunks

struct Shared {
    gs_code *cauchy = nullptr, *power = nullptr, *rdp = nullptr;
    std::vector<uint8_t> R_expected;   // decode matrix of {1, 6, 9}, found before the threads start
    int surv_expected[K];
};

// aligned host memory standing in for device and pinned buffers of one thread
struct Buffers {
    std::vector<void *> all;
    void *get(size_t n)
    {
        void *p = nullptr;
        if (posix_memalign(&p, 256, n ? n : 256) != 0) std::abort();
        std::memset(p, 0x5A, n);
        all.push_back(p);
        return p;
    }
    ~Buffers() { for (void *p : all) std::free(p); }
};

void worker(const Shared &sh, int id, int rounds)
{
    Buffers mem;
    void *shards[K + M], *host_parity[M];
    for (void *&p : shards) p = mem.get(S);
    for (void *&p : host_parity) p = mem.get(S);
    hipStream_t stream = nullptr;
    EXPECT(hipStreamCreateWithFlags(&stream, 0) == hipSuccess);
    gs_pipe *pipe = nullptr, *rdp_pipe = nullptr;
    gs_batch *batch = nullptr, *rdp_batch = nullptr;
    gs_pool *pool = nullptr;
    EXPECT(gs_pipe_create(sh.cauchy, 4096, 2, &pipe) == GS_OK);
    EXPECT(gs_pipe_create(sh.rdp, 6 * 1024, 2, &rdp_pipe) == GS_OK);
    EXPECT(gs_batch_create(sh.cauchy, 8, &batch) == GS_OK);
    EXPECT(gs_batch_create(sh.rdp, 8, &rdp_batch) == GS_OK);
    EXPECT(gs_pool_create(3, &pool) == GS_OK);

    // four chunks of a quarter shard each, for the grouped and per-stream forms
    const int n_chunks = 4;
    const size_t per = S / n_chunks;
    std::vector<const void *> cdata(n_chunks * K);
    std::vector<void *> cpar(n_chunks * M), cshards(n_chunks * (K + M)), rshards(n_chunks * (6 + 2)), rpar(n_chunks * 2);
    std::vector<const void *> rdata(n_chunks * 6);
    std::vector<size_t> sizes(n_chunks, per);
    for (int c = 0; c < n_chunks; ++c) {
        for (int j = 0; j < K + M; ++j) {
            void *p = static_cast<uint8_t *>(shards[j]) + c * per;
            cshards[c * (K + M) + j] = p;
            if (j < K) cdata[c * K + j] = p;
            else cpar[c * M + (j - K)] = p;
            if (j < 6) rdata[c * 6 + j] = p;
            if (j < 8) rshards[c * 8 + j] = p;
            if (j >= 6 && j < 8) rpar[c * 2 + (j - 6)] = p;
        }
    }

    for (int r = 0; r < rounds; ++r) {
        // the shared codes, read by every thread at once
        uint8_t R[M * K];
        int surv[K];
        const int erased[3] = {1, 6, 9};
        EXPECT(gs_decode_matrix(sh.cauchy, erased, 3, R, surv) == GS_OK);
        EXPECT(std::memcmp(R, sh.R_expected.data(), sizeof R) == 0);
        EXPECT(std::memcmp(surv, sh.surv_expected, sizeof surv) == 0);
        int read[18], n_read = 0;
        uint32_t masks[2 * 16];
        const int miss[2] = {r % 6, 6 + (r & 1)};
        EXPECT(gs_rdp_plan(sh.rdp, miss, 2, read, &n_read, masks) == GS_OK && n_read == 6);
        uint32_t words[5];
        EXPECT(gs_coef_words((r * 7 + id) & 255, words) == GS_OK);

        EXPECT(gs_encode(sh.cauchy, shards, shards + K, S, stream) == GS_OK);
        EXPECT(gs_reconstruct(sh.cauchy, shards, erased, 3, S, stream) == GS_OK);
        EXPECT(gs_encode(sh.power, shards, shards + K, S, stream) == GS_OK);   // 8+2: parity = the first two of three
        EXPECT(gs_encode(sh.rdp, shards, shards + 6, S, stream) == GS_OK);
        EXPECT(gs_reconstruct(sh.rdp, shards, miss, 2, S, stream) == GS_OK);

        // objects of this thread only
        EXPECT(gs_checkpoint(pipe, shards, S, host_parity, stream) == GS_OK);
        EXPECT(gs_restore(pipe, shards, host_parity, erased, 3, S, stream) == GS_OK);
        EXPECT(gs_pipe_sync(pipe) == GS_OK);
        EXPECT(gs_checkpoint(rdp_pipe, shards, S, host_parity, stream) == GS_OK);
        EXPECT(gs_pipe_sync(rdp_pipe) == GS_OK);
        EXPECT(gs_encode_batch(batch, n_chunks, cdata.data(), cpar.data(), sizes.data(), stream) == GS_OK);
        EXPECT(gs_reconstruct_batch(batch, n_chunks, cshards.data(), erased, 3, sizes.data(), stream) == GS_OK);
        EXPECT(gs_encode_batch(rdp_batch, n_chunks, rdata.data(), rpar.data(), sizes.data(), stream) == GS_OK);
        EXPECT(gs_reconstruct_batch(rdp_batch, n_chunks, rshards.data(), miss, 2, sizes.data(), stream) == GS_OK);
        EXPECT(gs_encode_streams(sh.cauchy, pool, n_chunks, cdata.data(), cpar.data(), sizes.data(), stream) == GS_OK);
        // the allocation-free form: every thread's descriptors go to the one array of the device, which
        // the header says callers must not do at the same time on a GPU; on the host side only the
        // cached address is shared
        EXPECT(gs_encode_batch_static(sh.cauchy, n_chunks, cdata.data(), cpar.data(), sizes.data(), stream) == GS_OK);

        // errors are per thread
        EXPECT(gs_encode(sh.cauchy, shards, shards + K, S, stream) == GS_OK);
        EXPECT(gs_reconstruct(sh.cauchy, shards, erased, 4, S, stream) != GS_OK);
        (void)gs_last_hip_error();
        EXPECT(gs_strerror(GS_EINVAL) != nullptr);

        // one thread keeps turning the process-wide knobs while the others launch
        if (id == 0) {
            EXPECT(gs_set_launch_shape(1 + (r & 1), 1 + (r % 3), r & 1, r % 7) == GS_OK);
            EXPECT(gs_set_power_horner(r & 1) == GS_OK);
            EXPECT(gs_set_size_forms((r >> 1) % 3) == GS_OK);
        }
    }
    gs_pool_destroy(pool);
    gs_batch_destroy(rdp_batch);
    gs_batch_destroy(batch);
    gs_pipe_destroy(rdp_pipe);
    gs_pipe_destroy(pipe);
    (void)hipStreamDestroy(stream);
}

}  // namespace

int main()
{
    Shared sh;
    if (gs_make_code(K, M, GS_CAUCHY, &sh.cauchy) != GS_OK || gs_make_code(K, 2, GS_POWER, &sh.power) != GS_OK ||
        gs_make_rdp_code(6, 1024, &sh.rdp) != GS_OK) {
        std::fprintf(stderr, "FAIL: codes\n");
        return 1;
    }
    sh.R_expected.resize(M * K);
    const int erased[3] = {1, 6, 9};
    if (gs_decode_matrix(sh.cauchy, erased, 3, sh.R_expected.data(), sh.surv_expected) != GS_OK) return 1;

    // codes made and freed while other threads work: construction shares only the constant field tables
    std::vector<std::thread> threads;
    for (int id = 0; id < 6; ++id) threads.emplace_back(worker, std::cref(sh), id, 40);
    threads.emplace_back([] {
        for (int i = 0; i < 200; ++i) {
            gs_code *c = nullptr;
            if (gs_make_code(2 + i % 30, 1 + i % 4, i & 1 ? GS_CAUCHY : GS_VANDERMONDE, &c) != GS_OK) failures.fetch_add(1);
            gs_free_code(c);
        }
    });
    for (std::thread &t : threads) t.join();
    gs_set_launch_shape(0, 0, -1, -1);
    gs_set_power_horner(1);
    gs_set_size_forms(1);
    gs_free_code(sh.cauchy);
    gs_free_code(sh.power);
    gs_free_code(sh.rdp);
    if (failures.load() != 0 || launches.load() == 0) {
        std::fprintf(stderr, "FAIL: %d failures, %ld launches\n", failures.load(), launches.load());
        return 1;
    }
    std::printf("OK\n");
    return 0;
}
