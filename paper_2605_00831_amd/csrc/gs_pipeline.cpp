// Checkpoint / restore pipelines (encode overlapped with parity D2H; parity
// H2D overlapped with reconstruct) and the captured per-step checkpoint.
#include "../../include/ghostserve_ec.h"

#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <new>
#include <vector>

#include "gs_internal.h"

using namespace gs;

// Staging slot s holds m buffers of chunk_bytes.  Two events per slot:
//   filled[s]   the slot's producer has finished (encode kernel, or H2D copy)
//   drained[s]  the slot's consumer has finished (D2H copy, or reconstruct kernel)
// A producer waits on drained[s] before reusing slot s.
struct gs_pipe {
    const gs_code *code = nullptr;
    size_t chunk_bytes = 0;
    int depth = 0;
    uint8_t *staging = nullptr;  // depth * m * chunk_bytes
    std::vector<hipEvent_t> filled, drained;
    std::vector<char> used;
    hipStream_t copy_stream = nullptr;
    hipEvent_t done = nullptr;
    bool any = false;
    // optional per-chunk timing of the last gs_checkpoint / gs_restore call
    bool timing = false;
    hipEvent_t t_origin = nullptr;
    std::vector<hipEvent_t> t_kernel_begin, t_kernel_end, t_copy_end;
    size_t timed_chunks = 0;

    uint8_t *slot_buf(int slot, int row) const
    {
        return staging + (static_cast<size_t>(slot) * code->m + row) * chunk_bytes;
    }
};

struct gs_step_graph {
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
};

// timing events for chunks [0, n), created on first use and kept
static hipError_t grow_timing(gs_pipe *p, size_t n)
{
    if (p->t_origin == nullptr) {
        const hipError_t e = hipEventCreate(&p->t_origin);
        if (e != hipSuccess) return e;
    }
    for (std::vector<hipEvent_t> *v : {&p->t_kernel_begin, &p->t_kernel_end, &p->t_copy_end}) {
        while (v->size() < n) {
            hipEvent_t ev = nullptr;
            const hipError_t e = hipEventCreate(&ev);
            if (e != hipSuccess) return e;
            v->push_back(ev);
        }
    }
    return hipSuccess;
}

#define GS_TRY(expr)                                 \
    do {                                             \
        const hipError_t e_ = (expr);                \
        if (e_ != hipSuccess) return hip_status(e_); \
    } while (0)

extern "C" {

void gs_pipe_destroy(gs_pipe *p)
{
    if (p == nullptr) return;
    if (p->copy_stream) (void)hipStreamSynchronize(p->copy_stream);
    for (hipEvent_t e : p->filled) if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : p->drained) if (e) (void)hipEventDestroy(e);
    if (p->done) (void)hipEventDestroy(p->done);
    if (p->t_origin) (void)hipEventDestroy(p->t_origin);
    for (std::vector<hipEvent_t> *v : {&p->t_kernel_begin, &p->t_kernel_end, &p->t_copy_end})
        for (hipEvent_t e : *v) (void)hipEventDestroy(e);
    if (p->copy_stream) (void)hipStreamDestroy(p->copy_stream);
    if (p->staging) (void)hipFree(p->staging);
    delete p;
}

int gs_pipe_create(const gs_code *code, size_t chunk_bytes, int depth, gs_pipe **out)
try {
    if (out == nullptr) return GS_EINVAL;
    *out = nullptr;
    if (code == nullptr || chunk_bytes == 0 || chunk_bytes % 16 != 0 || depth < 2 || depth > 64) return GS_EINVAL;
    // RDP chunks must hold whole stripes
    if (code->is_rdp() && chunk_bytes % (code->rdp_cell * (code->rdp_encode.p - 1)) != 0) return GS_EINVAL;
    gs_pipe *p = new (std::nothrow) gs_pipe;
    if (p == nullptr) return GS_ENOMEM;
    p->code = code;
    p->chunk_bytes = chunk_bytes;
    p->depth = depth;
    try {
        p->filled.assign(depth, nullptr);
        p->drained.assign(depth, nullptr);
        p->used.assign(depth, 0);
    } catch (...) {
        delete p;
        throw;
    }
    int rc = GS_OK;
    auto step = [&](hipError_t e) { if (rc == GS_OK && e != hipSuccess) rc = hip_status(e); };
    step(hipMalloc(reinterpret_cast<void **>(&p->staging), static_cast<size_t>(depth) * code->m * chunk_bytes));
    // default priority on purpose: streams of mixed priority are not used
    step(hipStreamCreateWithFlags(&p->copy_stream, hipStreamNonBlocking));
    for (int s = 0; s < depth && rc == GS_OK; ++s) {
        step(hipEventCreateWithFlags(&p->filled[s], hipEventDisableTiming));
        step(hipEventCreateWithFlags(&p->drained[s], hipEventDisableTiming));
    }
    step(hipEventCreateWithFlags(&p->done, hipEventDisableTiming));
    if (rc != GS_OK) {
        gs_pipe_destroy(p);
        return rc;
    }
    *out = p;
    return GS_OK;
}
catch (...) {
    return caught();
}

int gs_checkpoint(gs_pipe *p, const void *const *data, size_t shard_bytes, void *const *host_parity,
                  void *compute_stream)
try {
    if (p == nullptr || data == nullptr || host_parity == nullptr) return GS_EINVAL;
    const int k = p->code->k, m = p->code->m;
    for (int j = 0; j < k; ++j)
        if (data[j] == nullptr || (reinterpret_cast<uintptr_t>(data[j]) & 15u)) return GS_EINVAL;
    for (int i = 0; i < m; ++i)
        if (host_parity[i] == nullptr) return GS_EINVAL;
    if (shard_bytes == 0) return GS_OK;
    hipStream_t cs = static_cast<hipStream_t>(compute_stream);
    std::vector<const void *> in(k);
    std::vector<void *> out(m);
    const size_t nchunks = (shard_bytes + p->chunk_bytes - 1) / p->chunk_bytes;
    p->timed_chunks = 0;
    if (p->timing) {
        GS_TRY(grow_timing(p, nchunks));
        GS_TRY(hipEventRecord(p->t_origin, cs));
    }
    for (size_t c = 0; c < nchunks; ++c) {
        const int slot = static_cast<int>(c % p->depth);
        const size_t off = c * p->chunk_bytes;
        const size_t len = std::min(p->chunk_bytes, shard_bytes - off);
        if (p->used[slot]) GS_TRY(hipStreamWaitEvent(cs, p->drained[slot], 0));
        for (int j = 0; j < k; ++j) in[j] = static_cast<const uint8_t *>(data[j]) + off;
        for (int i = 0; i < m; ++i) out[i] = p->slot_buf(slot, i);
        if (p->timing) GS_TRY(hipEventRecord(p->t_kernel_begin[c], cs));
        const int rc = gs_encode(p->code, in.data(), out.data(), len, cs);
        if (rc != GS_OK) return rc;
        if (p->timing) GS_TRY(hipEventRecord(p->t_kernel_end[c], cs));
        GS_TRY(hipEventRecord(p->filled[slot], cs));
        GS_TRY(hipStreamWaitEvent(p->copy_stream, p->filled[slot], 0));
        for (int i = 0; i < m; ++i)
            GS_TRY(hipMemcpyAsync(static_cast<uint8_t *>(host_parity[i]) + off, p->slot_buf(slot, i), len,
                                  hipMemcpyDeviceToHost, p->copy_stream));
        if (p->timing) GS_TRY(hipEventRecord(p->t_copy_end[c], p->copy_stream));
        GS_TRY(hipEventRecord(p->drained[slot], p->copy_stream));
        p->used[slot] = 1;
    }
    if (p->timing) p->timed_chunks = nchunks;
    GS_TRY(hipEventRecord(p->done, p->copy_stream));
    p->any = true;
    return GS_OK;
}
catch (...) {
    return caught();
}

int gs_restore(gs_pipe *p, void *const *shards, void *const *host_parity, const int *erased,
               int n_erased, size_t shard_bytes, void *compute_stream)
try {
    if (p == nullptr || shards == nullptr || host_parity == nullptr) return GS_EINVAL;
    const int k = p->code->k, m = p->code->m;
    std::vector<int> read;  // shard ids the rebuild reads
    std::vector<uint8_t> R;  // rebuild matrix, found once for all chunks (not RDP)
    const int rc0 = p->code->is_rdp() ? shards_read(p->code, erased, n_erased, read)
                                      : decode_matrix(p->code, erased, n_erased, R, read);
    if (rc0 != GS_OK) return rc0;
    if (n_erased == 0 || shard_bytes == 0) return GS_OK;
    if (p->code->is_rdp() && shard_bytes % (p->code->rdp_cell * (p->code->rdp_encode.p - 1)) != 0) return GS_EINVAL;
    for (int s : read) {
        if (s < k) {
            if (shards[s] == nullptr || (reinterpret_cast<uintptr_t>(shards[s]) & 15u)) return GS_EINVAL;
        } else if (host_parity[s - k] == nullptr) {
            return GS_EINVAL;
        }
    }
    for (int x = 0; x < n_erased; ++x)
        if (shards[erased[x]] == nullptr || (reinterpret_cast<uintptr_t>(shards[erased[x]]) & 15u)) return GS_EINVAL;
    hipStream_t cs = static_cast<hipStream_t>(compute_stream);
    std::vector<void *> view(k + m);  // the stripe as the rebuild of one chunk sees it
    const size_t nchunks = (shard_bytes + p->chunk_bytes - 1) / p->chunk_bytes;
    p->timed_chunks = 0;
    if (p->timing) {
        GS_TRY(grow_timing(p, nchunks));
        GS_TRY(hipEventRecord(p->t_origin, cs));
    }
    for (size_t c = 0; c < nchunks; ++c) {
        const int slot = static_cast<int>(c % p->depth);
        const size_t off = c * p->chunk_bytes;
        const size_t len = std::min(p->chunk_bytes, shard_bytes - off);
        if (p->used[slot]) GS_TRY(hipStreamWaitEvent(p->copy_stream, p->drained[slot], 0));
        for (int r = 0; r < k + m; ++r) view[r] = nullptr;
        for (int s : read) {
            if (s < k) {
                view[s] = static_cast<uint8_t *>(shards[s]) + off;
            } else {
                uint8_t *stage = p->slot_buf(slot, s - k);
                GS_TRY(hipMemcpyAsync(stage, static_cast<const uint8_t *>(host_parity[s - k]) + off, len,
                                      hipMemcpyHostToDevice, p->copy_stream));
                view[s] = stage;
            }
        }
        for (int x = 0; x < n_erased; ++x) view[erased[x]] = static_cast<uint8_t *>(shards[erased[x]]) + off;
        if (p->timing) GS_TRY(hipEventRecord(p->t_copy_end[c], p->copy_stream));
        GS_TRY(hipEventRecord(p->filled[slot], p->copy_stream));
        GS_TRY(hipStreamWaitEvent(cs, p->filled[slot], 0));
        if (p->timing) GS_TRY(hipEventRecord(p->t_kernel_begin[c], cs));
        const int rc = p->code->is_rdp() ? gs_reconstruct(p->code, view.data(), erased, n_erased, len, cs)
                                         : apply_rebuild(p->code, R, read, view.data(), erased, n_erased, len, cs);
        if (rc != GS_OK) return rc;
        if (p->timing) GS_TRY(hipEventRecord(p->t_kernel_end[c], cs));
        GS_TRY(hipEventRecord(p->drained[slot], cs));
        p->used[slot] = 1;
    }
    if (p->timing) p->timed_chunks = nchunks;
    GS_TRY(hipEventRecord(p->done, cs));
    p->any = true;
    return GS_OK;
}
catch (...) {
    return caught();
}

int gs_pipe_sync(gs_pipe *p)
{
    if (p == nullptr) return GS_EINVAL;
    if (!p->any) return GS_OK;
    GS_TRY(hipEventSynchronize(p->done));
    return GS_OK;
}

int gs_pipe_set_timing(gs_pipe *p, int enable)
{
    if (p == nullptr) return GS_EINVAL;
    p->timing = enable != 0;
    if (!p->timing) p->timed_chunks = 0;
    return GS_OK;
}

int gs_pipe_chunk_times(gs_pipe *p, int max_chunks, float *kernel_begin_ms, float *kernel_end_ms,
                        float *copy_end_ms, int *n_chunks_out)
{
    if (p == nullptr || n_chunks_out == nullptr || max_chunks < 0) return GS_EINVAL;
    *n_chunks_out = static_cast<int>(p->timed_chunks);
    if (p->timed_chunks == 0) return GS_OK;
    GS_TRY(hipEventSynchronize(p->done));
    const size_t n = std::min(p->timed_chunks, static_cast<size_t>(max_chunks));
    for (size_t c = 0; c < n; ++c) {
        if (kernel_begin_ms) GS_TRY(hipEventElapsedTime(&kernel_begin_ms[c], p->t_origin, p->t_kernel_begin[c]));
        if (kernel_end_ms) GS_TRY(hipEventElapsedTime(&kernel_end_ms[c], p->t_origin, p->t_kernel_end[c]));
        if (copy_end_ms) GS_TRY(hipEventElapsedTime(&copy_end_ms[c], p->t_origin, p->t_copy_end[c]));
    }
    return GS_OK;
}

void *gs_pipe_done_event(gs_pipe *p) { return (p && p->any) ? static_cast<void *>(p->done) : nullptr; }

void gs_step_graph_destroy(gs_step_graph *g)
{
    if (g == nullptr) return;
    if (g->exec) (void)hipGraphExecDestroy(g->exec);
    if (g->graph) (void)hipGraphDestroy(g->graph);
    delete g;
}

int gs_step_graph_create(const gs_code *code, const void *const *plane_base, int n_planes,
                         size_t page_bytes, int64_t pages_per_plane, const int32_t *table,
                         int pages_per_shard, void *const *parity, void *const *host_parity,
                         gs_step_graph **out)
try {
    if (out == nullptr) return GS_EINVAL;
    *out = nullptr;
    if (code == nullptr || n_planes < 1 || pages_per_shard < 1 || code->is_rdp()) return GS_EINVAL;
    gs_step_graph *g = new (std::nothrow) gs_step_graph;
    if (g == nullptr) return GS_ENOMEM;
    hipStream_t s = nullptr;
    hipError_t e = hipStreamCreateWithFlags(&s, hipStreamNonBlocking);
    if (e != hipSuccess) {
        delete g;
        return hip_status(e);
    }
    int rc = GS_OK;
    e = hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal);
    if (e != hipSuccess) rc = hip_status(e);
    if (rc == GS_OK) {
        rc = gs_encode_paged(code, plane_base, n_planes, page_bytes, pages_per_plane, table,
                             pages_per_shard, parity, s);
        if (rc == GS_OK && host_parity != nullptr) {
            const size_t bytes = static_cast<size_t>(n_planes) * pages_per_shard * page_bytes;
            for (int i = 0; i < code->m && rc == GS_OK; ++i) {
                if (host_parity[i] == nullptr) { rc = GS_EINVAL; break; }
                e = hipMemcpyAsync(host_parity[i], parity[i], bytes, hipMemcpyDeviceToHost, s);
                if (e != hipSuccess) rc = hip_status(e);
            }
        }
        // always close the capture, also on failure
        e = hipStreamEndCapture(s, &g->graph);
        if (rc == GS_OK && e != hipSuccess) rc = hip_status(e);
    }
    if (rc == GS_OK) {
        e = hipGraphInstantiate(&g->exec, g->graph, nullptr, nullptr, 0);
        if (e != hipSuccess) rc = hip_status(e);
    }
    (void)hipStreamDestroy(s);
    if (rc != GS_OK) {
        gs_step_graph_destroy(g);
        return rc;
    }
    *out = g;
    return GS_OK;
}
catch (...) {
    return caught();
}

int gs_step_graph_launch(gs_step_graph *g, void *stream)
{
    if (g == nullptr || g->exec == nullptr) return GS_EINVAL;
    GS_TRY(hipGraphLaunch(g->exec, static_cast<hipStream_t>(stream)));
    return GS_OK;
}

}  // extern "C"
