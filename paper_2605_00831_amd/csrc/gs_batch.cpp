// Many chunks at once: a grouped launch over a device-side descriptor array
// (gs_batch), and the one-stream-per-chunk form the paper describes (gs_pool).
#include "../../include/ghostserve_ec.h"

#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <new>
#include <vector>

#include "gs_internal.h"

using namespace gs;

namespace {
constexpr int kRing = 4;  // descriptor slots in flight per gs_batch
}

// Descriptor slots are reused round-robin; a slot's event is recorded after
// the kernel that reads it, and the host waits on it only when the ring wraps
// while that kernel is still running.
struct gs_batch {
    const gs_code *code = nullptr;
    int max_chunks = 0;
    size_t slot_bytes = 0;
    uint8_t *dev = nullptr;     // kRing * slot_bytes
    uint8_t *host = nullptr;    // pinned mirror
    hipEvent_t done[kRing] = {};
    bool used[kRing] = {};
    unsigned next = 0;
};

struct gs_pool {
    std::vector<hipStream_t> streams;
    hipEvent_t fork = nullptr;
    std::vector<hipEvent_t> join;
};

#define GS_TRY(expr)                                 \
    do {                                             \
        const hipError_t e_ = (expr);                \
        if (e_ != hipSuccess) return hip_status(e_); \
    } while (0)

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Enqueue one grouped launch: rows x k matrix C over n chunks; in/out are
// chunk-major pointer arrays with strides in_stride / out_stride entries.
static int run_batch(gs_batch *b, int rows, const uint8_t *C, int n, const void *const *in, int in_stride,
                     void *const *out, int out_stride, const size_t *bytes, hipStream_t stream)
{
    const int k = b->code->k;
    const LaunchShape shape = current_shape();
    size_t max_bytes = 0;
    for (int c = 0; c < n; ++c) max_bytes = std::max(max_bytes, bytes[c]);
    if (max_bytes == 0) return GS_OK;
    if (max_bytes >= (1ull << 34)) return GS_EINVAL;  // 16 GiB per stream and chunk: one tile per workgroup
    const unsigned slot = b->next % kRing;
    if (b->used[slot]) GS_TRY(hipEventSynchronize(b->done[slot]));
    uint8_t *hslot = b->host + static_cast<size_t>(slot) * b->slot_bytes;
    uint8_t *dslot = b->dev + static_cast<size_t>(slot) * b->slot_bytes;
    int order[kLaunchMaxM];
    batch_row_order(rows, k, C, k, order);  // the same matrix for every chunk: planned once
    for (int c = 0; c < n; ++c)
        write_batch_desc(hslot, c, rows, k, order, in + static_cast<size_t>(c) * in_stride,
                         out + static_cast<size_t>(c) * out_stride, bytes[c], shape);
    GS_TRY(hipMemcpyAsync(dslot, hslot, static_cast<size_t>(n) * batch_desc_bytes(), hipMemcpyHostToDevice, stream));
    GS_TRY(launch_apply_batch(rows, k, C, k, dslot, n, max_bytes, shape, stream));
    GS_TRY(hipEventRecord(b->done[slot], stream));
    b->used[slot] = true;
    ++b->next;
    return GS_OK;
}

// The RDP form of run_batch: one plan for all chunks; shards is chunk-major with k+2 entries per chunk
// (data, row parity, diagonal parity), every chunk whole stripes.
static int run_rdp_batch(gs_batch *b, const RdpPlan &plan, int n, const void *const *shards, const size_t *bytes,
                         hipStream_t stream)
{
    const gs_code *code = b->code;
    const int width = code->k + 2;
    const size_t stripe = code->rdp_cell * static_cast<size_t>(plan.p - 1);
    const LaunchShape shape = current_shape();
    size_t max_bytes = 0;
    for (int c = 0; c < n; ++c) {
        // whole stripes, and what one launch covers: 16 GiB per stripe row (p = 3: chunks below 32 GiB)
        if (bytes[c] % stripe != 0 || bytes[c] / (plan.p - 1) >= (16ull << 30)) return GS_EINVAL;
        max_bytes = std::max(max_bytes, bytes[c]);
    }
    if (max_bytes == 0) return GS_OK;
    // pointers of every chunk that has bytes: the shards the plan reads and the ones it writes
    for (int c = 0; c < n; ++c) {
        if (bytes[c] == 0) continue;
        const void *const *row = shards + static_cast<size_t>(c) * width;
        const void *in[kRdpMaxDisks];
        void *out[2];
        int n_in = 0, n_out = 0;
        for (int j = 0; j <= plan.p; ++j) {
            const int sh = plan.shard_of_disk[j];
            if (sh < 0) continue;
            if (row[sh] == nullptr || !aligned16(row[sh])) return GS_EINVAL;
            in[n_in++] = row[sh];
        }
        for (int sh : plan.outputs) {
            if (row[sh] == nullptr || !aligned16(row[sh])) return GS_EINVAL;
            out[n_out++] = const_cast<void *>(row[sh]);
        }
        if (outputs_overlap(in, n_in, out, n_out, bytes[c])) return GS_EINVAL;
    }
    const unsigned slot = b->next % kRing;
    if (b->used[slot]) GS_TRY(hipEventSynchronize(b->done[slot]));
    uint8_t *hslot = b->host + static_cast<size_t>(slot) * b->slot_bytes;
    uint8_t *dslot = b->dev + static_cast<size_t>(slot) * b->slot_bytes;
    for (int c = 0; c < n; ++c)
        if (!write_rdp_batch_desc(hslot, c, plan, shards + static_cast<size_t>(c) * width, bytes[c], code->rdp_cell, shape))
            return GS_EINVAL;
    GS_TRY(hipMemcpyAsync(dslot, hslot, static_cast<size_t>(n) * batch_desc_bytes(), hipMemcpyHostToDevice, stream));
    GS_TRY(launch_rdp_batch(plan, dslot, n, max_bytes, code->rdp_cell, shape, stream));
    GS_TRY(hipEventRecord(b->done[slot], stream));
    b->used[slot] = true;
    ++b->next;
    return GS_OK;
}

// chunk c runs on pool stream c mod n; the pool streams start after everything
// already enqueued on `stream`, and `stream` continues after all of them
template <typename PerChunk>
static int fan_out(gs_pool *p, int n_chunks, hipStream_t stream, PerChunk per_chunk)
{
    const int ns = static_cast<int>(p->streams.size());
    const int active = std::min(ns, n_chunks);
    GS_TRY(hipEventRecord(p->fork, stream));
    for (int s = 0; s < active; ++s) GS_TRY(hipStreamWaitEvent(p->streams[s], p->fork, 0));
    int rc = GS_OK;
    for (int c = 0; c < n_chunks && rc == GS_OK; ++c) rc = per_chunk(c, p->streams[c % ns]);
    // join also after a failed chunk, so `stream` still follows what was enqueued
    for (int s = 0; s < active; ++s) {
        GS_TRY(hipEventRecord(p->join[s], p->streams[s]));
        GS_TRY(hipStreamWaitEvent(stream, p->join[s], 0));
    }
    return rc;
}

extern "C" {

void gs_batch_destroy(gs_batch *b)
{
    if (b == nullptr) return;
    for (int s = 0; s < kRing; ++s) {
        if (b->used[s]) (void)hipEventSynchronize(b->done[s]);
        if (b->done[s]) (void)hipEventDestroy(b->done[s]);
    }
    if (b->dev) (void)hipFree(b->dev);
    if (b->host) (void)hipHostFree(b->host);
    delete b;
}

int gs_batch_create(const gs_code *code, int max_chunks, gs_batch **out)
try {
    if (out == nullptr) return GS_EINVAL;
    *out = nullptr;
    if (code == nullptr || max_chunks < 1 || max_chunks > 65535) return GS_EINVAL;
    if (code->k > kLaunchMaxK || code->m > kLaunchMaxM) return GS_EINVAL;
    gs_batch *b = new (std::nothrow) gs_batch;
    if (b == nullptr) return GS_ENOMEM;
    b->code = code;
    b->max_chunks = max_chunks;
    b->slot_bytes = static_cast<size_t>(max_chunks) * batch_desc_bytes();
    int rc = GS_OK;
    auto step = [&](hipError_t e) { if (rc == GS_OK && e != hipSuccess) rc = hip_status(e); };
    step(hipMalloc(reinterpret_cast<void **>(&b->dev), kRing * b->slot_bytes));
    step(hipHostMalloc(reinterpret_cast<void **>(&b->host), kRing * b->slot_bytes, hipHostMallocDefault));
    for (int s = 0; s < kRing && rc == GS_OK; ++s) step(hipEventCreateWithFlags(&b->done[s], hipEventDisableTiming));
    if (rc != GS_OK) {
        gs_batch_destroy(b);
        return rc;
    }
    *out = b;
    return GS_OK;
}
catch (...) {
    return caught();
}

int gs_encode_batch(gs_batch *b, int n_chunks, const void *const *data, void *const *parity,
                    const size_t *shard_bytes, void *stream)
try {
    if (b == nullptr || n_chunks < 0 || n_chunks > b->max_chunks) return GS_EINVAL;
    if (n_chunks == 0) return GS_OK;
    if (data == nullptr || parity == nullptr || shard_bytes == nullptr) return GS_EINVAL;
    const int k = b->code->k, m = b->code->m;
    if (b->code->is_rdp()) {
        // one stripe view per chunk: k data shards, then the two parity shards
        std::vector<const void *> shards(static_cast<size_t>(n_chunks) * (k + 2));
        for (int c = 0; c < n_chunks; ++c) {
            for (int j = 0; j < k; ++j) shards[static_cast<size_t>(c) * (k + 2) + j] = data[c * k + j];
            for (int i = 0; i < 2; ++i) shards[static_cast<size_t>(c) * (k + 2) + k + i] = parity[c * 2 + i];
        }
        return run_rdp_batch(b, b->code->rdp_encode, n_chunks, shards.data(), shard_bytes, static_cast<hipStream_t>(stream));
    }
    for (int c = 0; c < n_chunks; ++c) {
        if (shard_bytes[c] == 0) continue;
        for (int j = 0; j < k; ++j)
            if (data[c * k + j] == nullptr || !aligned16(data[c * k + j])) return GS_EINVAL;
        for (int i = 0; i < m; ++i)
            if (parity[c * m + i] == nullptr || !aligned16(parity[c * m + i])) return GS_EINVAL;
        if (outputs_overlap(data + static_cast<size_t>(c) * k, k, parity + static_cast<size_t>(c) * m, m, shard_bytes[c]))
            return GS_EINVAL;
    }
    return run_batch(b, m, b->code->P.data(), n_chunks, data, k, parity, m, shard_bytes,
                     static_cast<hipStream_t>(stream));
}
catch (...) {
    return caught();
}

int gs_reconstruct_batch(gs_batch *b, int n_chunks, void *const *shards, const int *erased, int n_erased,
                         const size_t *shard_bytes, void *stream)
try {
    if (b == nullptr || n_chunks < 0 || n_chunks > b->max_chunks) return GS_EINVAL;
    if (b->code->is_rdp()) {
        std::vector<uint8_t> lost;
        const int rcr = check_erasures(b->code, erased, n_erased, lost);
        if (rcr != GS_OK) return rcr;
        if (n_chunks == 0 || n_erased == 0) return GS_OK;
        if (shards == nullptr || shard_bytes == nullptr) return GS_EINVAL;
        RdpPlan plan;
        if (!rdp_plan(b->code->k, erased, n_erased, plan)) return GS_ESINGULAR;
        return run_rdp_batch(b, plan, n_chunks, shards, shard_bytes, static_cast<hipStream_t>(stream));
    }
    std::vector<uint8_t> R;
    std::vector<int> surv;
    const int rc = decode_matrix(b->code, erased, n_erased, R, surv);
    if (rc != GS_OK) return rc;
    if (n_chunks == 0 || n_erased == 0) return GS_OK;
    if (shards == nullptr || shard_bytes == nullptr) return GS_EINVAL;
    const int k = b->code->k, n = k + b->code->m;
    std::vector<const void *> in(static_cast<size_t>(n_chunks) * k);
    std::vector<void *> out(static_cast<size_t>(n_chunks) * n_erased);
    for (int c = 0; c < n_chunks; ++c) {
        for (int j = 0; j < k; ++j) {
            const void *p = shards[static_cast<size_t>(c) * n + surv[j]];
            if (shard_bytes[c] != 0 && (p == nullptr || !aligned16(p))) return GS_EINVAL;
            in[static_cast<size_t>(c) * k + j] = p;
        }
        for (int x = 0; x < n_erased; ++x) {
            void *p = shards[static_cast<size_t>(c) * n + erased[x]];
            if (shard_bytes[c] != 0 && (p == nullptr || !aligned16(p))) return GS_EINVAL;
            out[static_cast<size_t>(c) * n_erased + x] = p;
        }
        if (shard_bytes[c] != 0 && outputs_overlap(&in[static_cast<size_t>(c) * k], k, &out[static_cast<size_t>(c) * n_erased],
                                                   n_erased, shard_bytes[c]))
            return GS_EINVAL;
    }
    return run_batch(b, n_erased, R.data(), n_chunks, in.data(), k, out.data(), n_erased, shard_bytes,
                     static_cast<hipStream_t>(stream));
}
catch (...) {
    return caught();
}

// ---- one stream per chunk (Section 5, "CUDA Streams"; continuous batching) ----

void gs_pool_destroy(gs_pool *p)
{
    if (p == nullptr) return;
    for (hipStream_t s : p->streams) if (s) { (void)hipStreamSynchronize(s); (void)hipStreamDestroy(s); }
    for (hipEvent_t e : p->join) if (e) (void)hipEventDestroy(e);
    if (p->fork) (void)hipEventDestroy(p->fork);
    delete p;
}

int gs_pool_create(int n_streams, gs_pool **out)
try {
    if (out == nullptr) return GS_EINVAL;
    *out = nullptr;
    if (n_streams < 1 || n_streams > 64) return GS_EINVAL;
    gs_pool *p = new (std::nothrow) gs_pool;
    if (p == nullptr) return GS_ENOMEM;
    try {
        p->streams.assign(n_streams, nullptr);
        p->join.assign(n_streams, nullptr);
    } catch (...) {
        delete p;
        throw;
    }
    int rc = GS_OK;
    auto step = [&](hipError_t e) { if (rc == GS_OK && e != hipSuccess) rc = hip_status(e); };
    for (int s = 0; s < n_streams && rc == GS_OK; ++s) {
        step(hipStreamCreateWithFlags(&p->streams[s], hipStreamNonBlocking));  // default priority
        step(hipEventCreateWithFlags(&p->join[s], hipEventDisableTiming));
    }
    step(hipEventCreateWithFlags(&p->fork, hipEventDisableTiming));
    if (rc != GS_OK) {
        gs_pool_destroy(p);
        return rc;
    }
    *out = p;
    return GS_OK;
}
catch (...) {
    return caught();
}

int gs_encode_streams(const gs_code *code, gs_pool *pool, int n_chunks, const void *const *data,
                      void *const *parity, const size_t *shard_bytes, void *stream)
try {
    if (code == nullptr || pool == nullptr || n_chunks < 0) return GS_EINVAL;
    if (n_chunks == 0) return GS_OK;
    if (data == nullptr || parity == nullptr || shard_bytes == nullptr) return GS_EINVAL;
    const int k = code->k, m = code->m;
    // every chunk is checked before the first one is enqueued
    for (int c = 0; c < n_chunks; ++c) {
        const int rc = check_encode_args(code, data + static_cast<size_t>(c) * k, parity + static_cast<size_t>(c) * m,
                                         shard_bytes[c]);
        if (rc != GS_OK) return rc;
    }
    return fan_out(pool, n_chunks, static_cast<hipStream_t>(stream), [&](int c, hipStream_t s) {
        return gs_encode(code, data + static_cast<size_t>(c) * k, parity + static_cast<size_t>(c) * m,
                         shard_bytes[c], s);
    });
}
catch (...) {
    return caught();
}

int gs_reconstruct_streams(const gs_code *code, gs_pool *pool, int n_chunks, void *const *shards,
                           const int *erased, int n_erased, const size_t *shard_bytes, void *stream)
try {
    if (code == nullptr || pool == nullptr || n_chunks < 0) return GS_EINVAL;
    std::vector<int> read;
    std::vector<uint8_t> R;  // found once for all chunks (not RDP)
    const int rc = code->is_rdp() ? shards_read(code, erased, n_erased, read)
                                  : decode_matrix(code, erased, n_erased, R, read);
    if (rc != GS_OK) return rc;
    if (n_chunks == 0 || n_erased == 0) return GS_OK;
    if (shards == nullptr || shard_bytes == nullptr) return GS_EINVAL;
    const int n = code->k + code->m;
    for (int c = 0; c < n_chunks; ++c) {
        const int rcc = check_rebuild_args(code, shards + static_cast<size_t>(c) * n, read, erased, n_erased, shard_bytes[c]);
        if (rcc != GS_OK) return rcc;
    }
    return fan_out(pool, n_chunks, static_cast<hipStream_t>(stream), [&](int c, hipStream_t s) {
        void *const *stripe = shards + static_cast<size_t>(c) * n;
        if (code->is_rdp()) return gs_reconstruct(code, stripe, erased, n_erased, shard_bytes[c], s);
        return apply_rebuild(code, R, read, stripe, erased, n_erased, shard_bytes[c], s);
    });
}
catch (...) {
    return caught();
}

}  // extern "C"
