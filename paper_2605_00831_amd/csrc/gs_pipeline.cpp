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

// Copy `rows` pieces of `width` bytes, `spitch` / `dpitch` bytes apart: one
// plain copy when the pieces are back to back on both sides, else one strided
// copy (the parity of a window of page slots inside the dense parity layout).
static hipError_t copy_rows(void *dst, size_t dpitch, const void *src, size_t spitch, size_t width, size_t rows,
                            hipMemcpyKind kind, hipStream_t stream)
{
    if (rows == 1 || (dpitch == width && spitch == width))
        return hipMemcpyAsync(dst, src, width * rows, kind, stream);
    return hipMemcpy2DAsync(dst, dpitch, src, spitch, width, rows, kind, stream);
}

// What differs between the contiguous and the paged pipelines: how chunk c is
// encoded into / rebuilt from a staging slot, and how a parity row of chunk c
// moves between staging and pinned host memory.
struct ChunkOps {
    size_t n_chunks;
    // kernel(s) of chunk c on stream cs, parity rows in / out of staging slot `slot`
    virtual int compute(size_t c, int slot, hipStream_t cs) = 0;
    // copy of parity row i of chunk c between the slot and host memory
    virtual hipError_t copy(size_t c, int slot, int row, hipStream_t copy_stream) = 0;
    virtual ~ChunkOps() {}
};

// Checkpoint: per chunk, compute on the compute stream into a staging slot,
// then copy the slot's m rows to host memory on the copy stream.  Whatever
// happens, `done` is recorded after the last operation that was enqueued, so
// gs_pipe_sync() covers it.
static int run_checkpoint(gs_pipe *p, ChunkOps &ops, hipStream_t cs)
{
    const int m = p->code->m;
    p->timed_chunks = 0;
    int rc = GS_OK;
    auto step = [&](hipError_t e) {
        if (rc == GS_OK && e != hipSuccess) rc = hip_status(e);
        return rc == GS_OK;
    };
    if (p->timing && step(grow_timing(p, ops.n_chunks))) step(hipEventRecord(p->t_origin, cs));
    size_t c = 0;
    for (; c < ops.n_chunks && rc == GS_OK; ++c) {
        const int slot = static_cast<int>(c % p->depth);
        if (p->used[slot] && !step(hipStreamWaitEvent(cs, p->drained[slot], 0))) break;
        if (p->timing && !step(hipEventRecord(p->t_kernel_begin[c], cs))) break;
        rc = ops.compute(c, slot, cs);
        if (rc != GS_OK) break;
        if (p->timing && !step(hipEventRecord(p->t_kernel_end[c], cs))) break;
        if (!step(hipEventRecord(p->filled[slot], cs))) break;
        if (!step(hipStreamWaitEvent(p->copy_stream, p->filled[slot], 0))) break;
        for (int i = 0; i < m && rc == GS_OK; ++i) step(ops.copy(c, slot, i, p->copy_stream));
        if (rc != GS_OK) break;
        if (p->timing && !step(hipEventRecord(p->t_copy_end[c], p->copy_stream))) break;
        if (!step(hipEventRecord(p->drained[slot], p->copy_stream))) break;
        p->used[slot] = 1;
    }
    if (rc == GS_OK && p->timing) p->timed_chunks = ops.n_chunks;
    // after a failure the copy stream may not have been told to wait for the last kernel: order
    // `done` after both streams
    if (rc != GS_OK && hipEventRecord(p->done, cs) == hipSuccess) (void)hipStreamWaitEvent(p->copy_stream, p->done, 0);
    if (hipEventRecord(p->done, p->copy_stream) == hipSuccess) p->any = true;
    return rc;
}

// Restore: per chunk, bring the parity rows in `rows_in` from host memory into a
// staging slot on the copy stream, then compute on the compute stream.
static int run_restore(gs_pipe *p, ChunkOps &ops, const std::vector<int> &rows_in, hipStream_t cs)
{
    p->timed_chunks = 0;
    int rc = GS_OK;
    auto step = [&](hipError_t e) {
        if (rc == GS_OK && e != hipSuccess) rc = hip_status(e);
        return rc == GS_OK;
    };
    if (p->timing && step(grow_timing(p, ops.n_chunks))) step(hipEventRecord(p->t_origin, cs));
    for (size_t c = 0; c < ops.n_chunks && rc == GS_OK; ++c) {
        const int slot = static_cast<int>(c % p->depth);
        if (p->used[slot] && !step(hipStreamWaitEvent(p->copy_stream, p->drained[slot], 0))) break;
        for (size_t x = 0; x < rows_in.size() && rc == GS_OK; ++x) step(ops.copy(c, slot, rows_in[x], p->copy_stream));
        if (rc != GS_OK) break;
        if (p->timing && !step(hipEventRecord(p->t_copy_end[c], p->copy_stream))) break;
        if (!step(hipEventRecord(p->filled[slot], p->copy_stream))) break;
        if (!step(hipStreamWaitEvent(cs, p->filled[slot], 0))) break;
        if (p->timing && !step(hipEventRecord(p->t_kernel_begin[c], cs))) break;
        rc = ops.compute(c, slot, cs);
        if (rc != GS_OK) break;
        if (p->timing && !step(hipEventRecord(p->t_kernel_end[c], cs))) break;
        if (!step(hipEventRecord(p->drained[slot], cs))) break;
        p->used[slot] = 1;
    }
    if (rc == GS_OK && p->timing) p->timed_chunks = ops.n_chunks;
    // copies that were enqueued but whose kernel never followed must still be waited for
    if (rc != GS_OK && hipEventRecord(p->done, p->copy_stream) == hipSuccess) (void)hipStreamWaitEvent(cs, p->done, 0);
    if (hipEventRecord(p->done, cs) == hipSuccess) p->any = true;
    return rc;
}

static bool misaligned(const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15u) != 0; }

int gs_checkpoint(gs_pipe *p, const void *const *data, size_t shard_bytes, void *const *host_parity,
                  void *compute_stream)
try {
    if (p == nullptr || data == nullptr || host_parity == nullptr) return GS_EINVAL;
    const int k = p->code->k, m = p->code->m;
    for (int j = 0; j < k; ++j)
        if (data[j] == nullptr || misaligned(data[j])) return GS_EINVAL;
    for (int i = 0; i < m; ++i)
        if (host_parity[i] == nullptr) return GS_EINVAL;
    if (shard_bytes == 0) return GS_OK;
    // RDP shards hold whole stripes; refused here, before anything is enqueued
    if (p->code->is_rdp() && shard_bytes % (p->code->rdp_cell * (p->code->rdp_encode.p - 1)) != 0) return GS_EINVAL;
    struct Ops : ChunkOps {
        gs_pipe *p;
        const void *const *data;
        void *const *host;
        size_t S;
        std::vector<const void *> in;
        std::vector<void *> out;
        size_t len(size_t c) const { return std::min(p->chunk_bytes, S - c * p->chunk_bytes); }
        int compute(size_t c, int slot, hipStream_t cs) override
        {
            for (size_t j = 0; j < in.size(); ++j) in[j] = static_cast<const uint8_t *>(data[j]) + c * p->chunk_bytes;
            for (size_t i = 0; i < out.size(); ++i) out[i] = p->slot_buf(slot, static_cast<int>(i));
            return gs_encode(p->code, in.data(), out.data(), len(c), cs);
        }
        hipError_t copy(size_t c, int slot, int i, hipStream_t s) override
        {
            return hipMemcpyAsync(static_cast<uint8_t *>(host[i]) + c * p->chunk_bytes, p->slot_buf(slot, i), len(c),
                                  hipMemcpyDeviceToHost, s);
        }
    } ops;
    ops.p = p;
    ops.data = data;
    ops.host = host_parity;
    ops.S = shard_bytes;
    ops.in.resize(k);
    ops.out.resize(m);
    ops.n_chunks = (shard_bytes + p->chunk_bytes - 1) / p->chunk_bytes;
    return run_checkpoint(p, ops, static_cast<hipStream_t>(compute_stream));
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
    std::vector<int> rows_in;
    std::vector<const void *> in_dev;
    std::vector<void *> out_dev;
    for (int s : read) {
        if (s < k) {
            if (shards[s] == nullptr || misaligned(shards[s])) return GS_EINVAL;
            in_dev.push_back(shards[s]);
        } else {
            if (host_parity[s - k] == nullptr) return GS_EINVAL;
            rows_in.push_back(s - k);
        }
    }
    for (int x = 0; x < n_erased; ++x) {
        if (shards[erased[x]] == nullptr || misaligned(shards[erased[x]])) return GS_EINVAL;
        out_dev.push_back(shards[erased[x]]);
    }
    if (outputs_overlap(in_dev.data(), static_cast<int>(in_dev.size()), out_dev.data(), n_erased, shard_bytes))
        return GS_EINVAL;
    struct Ops : ChunkOps {
        gs_pipe *p;
        void *const *shards, *const *host;
        const int *erased;
        int n_erased;
        size_t S;
        const std::vector<int> *read;
        const std::vector<uint8_t> *R;
        std::vector<void *> view;  // the stripe as the rebuild of one chunk sees it
        size_t len(size_t c) const { return std::min(p->chunk_bytes, S - c * p->chunk_bytes); }
        int compute(size_t c, int slot, hipStream_t cs) override
        {
            const int k = p->code->k;
            const size_t off = c * p->chunk_bytes;
            std::fill(view.begin(), view.end(), nullptr);
            for (int s : *read) view[s] = s < k ? static_cast<uint8_t *>(shards[s]) + off : p->slot_buf(slot, s - k);
            for (int x = 0; x < n_erased; ++x) view[erased[x]] = static_cast<uint8_t *>(shards[erased[x]]) + off;
            return p->code->is_rdp() ? gs_reconstruct(p->code, view.data(), erased, n_erased, len(c), cs)
                                     : apply_rebuild(p->code, *R, *read, view.data(), erased, n_erased, len(c), cs);
        }
        hipError_t copy(size_t c, int slot, int i, hipStream_t s) override
        {
            return hipMemcpyAsync(p->slot_buf(slot, i), static_cast<const uint8_t *>(host[i]) + c * p->chunk_bytes, len(c),
                                  hipMemcpyHostToDevice, s);
        }
    } ops;
    ops.p = p;
    ops.shards = shards;
    ops.host = host_parity;
    ops.erased = erased;
    ops.n_erased = n_erased;
    ops.S = shard_bytes;
    ops.read = &read;
    ops.R = &R;
    ops.view.assign(k + m, nullptr);
    ops.n_chunks = (shard_bytes + p->chunk_bytes - 1) / p->chunk_bytes;
    return run_restore(p, ops, rows_in, static_cast<hipStream_t>(compute_stream));
}
catch (...) {
    return caught();
}

// ---- the same two pipelines over a paged KV pool ------------------------------
// A chunk is a window of `slots_per_chunk` page slots of every plane; its parity
// is produced into (or consumed from) a staging slot laid out [plane][slot][page]
// and lives in host memory inside the dense layout of gs_encode_paged,
// [plane][pages_per_shard][page], which a strided copy reaches.

struct PagedChunks {
    const void *const *plane_base;
    int n_planes;
    size_t page_bytes;
    int64_t pages_per_plane;
    const int32_t *table;
    int pps;               // pages per shard (table row length)
    int spc;               // page slots per chunk
    int slots(size_t c) const { return std::min(spc, pps - static_cast<int>(c) * spc); }
    gs::PagedView view(size_t c) const
    {
        return gs::PagedView{plane_base, n_planes, page_bytes, pages_per_plane, table + c * static_cast<size_t>(spc), pps, slots(c)};
    }
};

// chunk geometry of a paged pipeline call; GS_OK with spc == 0 means nothing to do
static int paged_chunks(const gs_pipe *p, const void *const *plane_base, int n_planes, size_t page_bytes,
                        int64_t pages_per_plane, const int32_t *table, int pages_per_shard, PagedChunks &g)
{
    bool empty;
    const int rc = check_paged_geometry(plane_base, n_planes, page_bytes, pages_per_plane, table, pages_per_shard, &empty);
    g = PagedChunks{plane_base, n_planes, page_bytes, pages_per_plane, table, pages_per_shard, 0};
    if (rc != GS_OK || empty) return rc;
    // a staging buffer holds whole page slots of every plane -- whole stripes of them for RDP
    const size_t slot_row = static_cast<size_t>(n_planes) * page_bytes;
    size_t spc = std::min<size_t>(p->chunk_bytes / slot_row, static_cast<size_t>(pages_per_shard));
    if (p->code->is_rdp()) {
        const int rc2 = check_rdp_paged(p->code, page_bytes, pages_per_shard);
        if (rc2 != GS_OK) return rc2;
        const size_t rows = static_cast<size_t>(p->code->rdp_encode.p - 1);
        spc = spc / rows * rows;
    }
    if (spc == 0) return GS_EINVAL;
    g.spc = static_cast<int>(spc);
    return GS_OK;
}

int gs_checkpoint_paged(gs_pipe *p, const void *const *plane_base, int n_planes, size_t page_bytes,
                        int64_t pages_per_plane, const int32_t *table, int pages_per_shard,
                        void *const *host_parity, void *compute_stream)
try {
    if (p == nullptr || host_parity == nullptr) return GS_EINVAL;
    PagedChunks g;
    const int rc = paged_chunks(p, plane_base, n_planes, page_bytes, pages_per_plane, table, pages_per_shard, g);
    if (rc != GS_OK) return rc;
    for (int i = 0; i < p->code->m; ++i)
        if (host_parity[i] == nullptr) return GS_EINVAL;
    if (g.spc == 0) return GS_OK;
    struct Ops : ChunkOps {
        gs_pipe *p;
        PagedChunks g;
        void *const *host;
        std::vector<gs::PagedStream> out;
        int compute(size_t c, int slot, hipStream_t cs) override
        {
            for (size_t i = 0; i < out.size(); ++i) out[i] = gs::PagedStream{-1, p->slot_buf(slot, static_cast<int>(i))};
            return encode_paged_view(p->code, g.view(c), out.data(), cs);
        }
        hipError_t copy(size_t c, int slot, int i, hipStream_t s) override
        {
            const size_t width = static_cast<size_t>(g.slots(c)) * g.page_bytes;
            return copy_rows(static_cast<uint8_t *>(host[i]) + c * static_cast<size_t>(g.spc) * g.page_bytes,
                             static_cast<size_t>(g.pps) * g.page_bytes, p->slot_buf(slot, i), width, width,
                             static_cast<size_t>(g.n_planes), hipMemcpyDeviceToHost, s);
        }
    } ops;
    ops.p = p;
    ops.g = g;
    ops.host = host_parity;
    ops.out.resize(p->code->m);
    ops.n_chunks = (static_cast<size_t>(pages_per_shard) + g.spc - 1) / g.spc;
    return run_checkpoint(p, ops, static_cast<hipStream_t>(compute_stream));
}
catch (...) {
    return caught();
}

int gs_restore_paged(gs_pipe *p, const void *const *plane_base, int n_planes, size_t page_bytes,
                     int64_t pages_per_plane, const int32_t *table, int pages_per_shard,
                     void *const *host_parity, void *const *parity_out, const int *erased, int n_erased,
                     void *compute_stream)
try {
    if (p == nullptr || host_parity == nullptr) return GS_EINVAL;
    PagedChunks g;
    const int rc = paged_chunks(p, plane_base, n_planes, page_bytes, pages_per_plane, table, pages_per_shard, g);
    if (rc != GS_OK) return rc;
    const int k = p->code->k, m = p->code->m;
    std::vector<uint8_t> R;
    std::vector<int> surv;  // the shards the rebuild reads
    const int rc1 = p->code->is_rdp() ? shards_read(p->code, erased, n_erased, surv)
                                      : decode_matrix(p->code, erased, n_erased, R, surv);
    if (rc1 != GS_OK) return rc1;
    if (n_erased == 0 || g.spc == 0) return GS_OK;
    std::vector<int> rows_in;
    for (int s : surv)
        if (s >= k) {
            if (host_parity[s - k] == nullptr) return GS_EINVAL;
            rows_in.push_back(s - k);
        }
    for (int x = 0; x < n_erased; ++x)
        if (erased[x] >= k && (parity_out == nullptr || parity_out[erased[x] - k] == nullptr || misaligned(parity_out[erased[x] - k])))
            return GS_EINVAL;
    struct Ops : ChunkOps {
        gs_pipe *p;
        PagedChunks g;
        void *const *host, *const *parity_out;
        const int *erased;
        int n_erased;
        const std::vector<uint8_t> *R;
        const std::vector<int> *surv;
        std::vector<gs::PagedStream> pin, pout;
        int compute(size_t c, int slot, hipStream_t cs) override
        {
            const int k = p->code->k;
            // surviving parity comes from the staging slot; a lost parity shard goes straight into the
            // caller's dense device buffer, at this chunk's slots
            for (int i = 0; i < p->code->m; ++i) {
                pin[i] = gs::PagedStream{-1, p->slot_buf(slot, i)};
                pout[i] = gs::PagedStream{-1, nullptr};
            }
            for (int x = 0; x < n_erased; ++x)
                if (erased[x] >= k)
                    pout[erased[x] - k] = gs::PagedStream{-1, static_cast<uint8_t *>(parity_out[erased[x] - k]) +
                                                                  c * static_cast<size_t>(g.spc) * g.page_bytes,
                                                          static_cast<size_t>(g.pps) * g.page_bytes};
            return rebuild_paged_view(p->code, *R, *surv, g.view(c), pin.data(), pout.data(), erased, n_erased, cs);
        }
        hipError_t copy(size_t c, int slot, int i, hipStream_t s) override
        {
            const size_t width = static_cast<size_t>(g.slots(c)) * g.page_bytes;
            return copy_rows(p->slot_buf(slot, i), width,
                             static_cast<const uint8_t *>(host[i]) + c * static_cast<size_t>(g.spc) * g.page_bytes,
                             static_cast<size_t>(g.pps) * g.page_bytes, width, static_cast<size_t>(g.n_planes),
                             hipMemcpyHostToDevice, s);
        }
    } ops;
    ops.p = p;
    ops.g = g;
    ops.host = host_parity;
    ops.parity_out = parity_out;
    ops.erased = erased;
    ops.n_erased = n_erased;
    ops.R = &R;
    ops.surv = &surv;
    ops.pin.resize(m);
    ops.pout.resize(m);
    ops.n_chunks = (static_cast<size_t>(pages_per_shard) + g.spc - 1) / g.spc;
    return run_restore(p, ops, rows_in, static_cast<hipStream_t>(compute_stream));
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
