// Grouped encode for callers that cannot allocate device memory (code under
// graph capture, tight serving loops, harnesses that forbid hipMalloc).
//
// gs_encode_batch keeps its chunk descriptors in a device buffer that a
// gs_batch object allocates.  Here the descriptors live in a fixed array in
// the library's own device image instead, and they reach it through the
// arguments of a small fill kernel, so the entry point calls no allocation
// routine and no copy: everything it enqueues is a kernel launch.
#include <hip/hip_runtime.h>

#include <mutex>

#include "../../include/ghostserve_ec.h"
#include "gs_internal.h"
#include "gs_launch.h"

using namespace gs;

namespace {

// Descriptor array of the allocation-free grouped encode: one per device (every
// device that loads the library holds its own copy until the process ends).
// In host code this name is only a handle for hipGetSymbolAddress; the address
// the kernels use is the one that call returns for the current device.
static __device__ __align__(256) unsigned char scratch[GS_STATIC_MAX_CHUNKS * kBatchDescBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];  // device address of `scratch`, per device, found on first use

hipError_t scratch_of_current_device(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (p == nullptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

// Chunks travel to the device as kernel arguments: per chunk k input
// pointers, `rows` output pointers (already in the launch's row order) and
// one word holding the stream length (low 56 bits) and the chunk's interleave
// shift (high 8 bits).
constexpr int kFillWords = 384;
constexpr int kFillThreads = 64;  // one thread per chunk of a fill launch

struct FillArgs {
    uint64_t words[kFillWords];
    BatchDesc *descs;  // where this launch's first descriptor goes
    uint32_t count, k, rows;
};

__global__ __launch_bounds__(kFillThreads) void fill_descs_kernel(const FillArgs a)
{
    const uint32_t c = threadIdx.x;
    if (c >= a.count) return;
    const uint64_t *w = a.words + static_cast<size_t>(c) * (a.k + a.rows + 1);
    BatchDesc d;
    for (uint32_t j = 0; j < static_cast<uint32_t>(kLaunchMaxK); ++j)
        d.in[j] = j < a.k ? reinterpret_cast<const uint8_t *>(w[j]) : nullptr;
    for (uint32_t r = 0; r < static_cast<uint32_t>(kLaunchMaxM); ++r)
        d.out[r] = r < a.rows ? reinterpret_cast<uint8_t *>(w[a.k + r]) : nullptr;
    const uint64_t len = w[a.k + a.rows] & ((1ull << 56) - 1);
    d.nvec = len / 16;
    d.tail = static_cast<uint32_t>(len % 16);
    d.nx_shift = static_cast<uint32_t>(w[a.k + a.rows] >> 56);
    a.descs[c] = d;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

extern "C" int gs_encode_batch_static(const gs_code *code, int n_chunks, const void *const *data, void *const *parity,
                                      const size_t *shard_bytes, void *stream_)
try {
    if (code == nullptr || n_chunks < 0) return GS_EINVAL;
    if (code->is_rdp() || code->k > kLaunchMaxK || code->m > kLaunchMaxM) return GS_EINVAL;
    if (n_chunks > GS_STATIC_MAX_CHUNKS) return GS_ELIMIT;
    if (n_chunks == 0) return GS_OK;
    if (data == nullptr || parity == nullptr || shard_bytes == nullptr) return GS_EINVAL;
    const int k = code->k, m = code->m;
    size_t max_bytes = 0;
    for (int c = 0; c < n_chunks; ++c) {
        if (shard_bytes[c] == 0) continue;
        if (shard_bytes[c] >= (1ull << 34)) return GS_ELIMIT;  // 16 GiB per stream and chunk: one tile per workgroup
        for (int j = 0; j < k; ++j)
            if (data[c * k + j] == nullptr || !aligned16(data[c * k + j])) return GS_EINVAL;
        for (int i = 0; i < m; ++i)
            if (parity[c * m + i] == nullptr || !aligned16(parity[c * m + i])) return GS_EINVAL;
        if (outputs_overlap(data + static_cast<size_t>(c) * k, k, parity + static_cast<size_t>(c) * m, m, shard_bytes[c]))
            return GS_EINVAL;
        if (shard_bytes[c] > max_bytes) max_bytes = shard_bytes[c];
    }
    if (max_bytes == 0) return GS_OK;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    void *base = nullptr;
    hipError_t e = scratch_of_current_device(&base);
    if (e != hipSuccess) return hip_status(e);
    BatchDesc *descs = static_cast<BatchDesc *>(base);

    const LaunchShape shape = current_shape();
    int order[kLaunchMaxM];
    batch_row_order(m, k, code->P.data(), k, order);
    const int per_chunk = k + m + 1;
    // what the argument block holds, and no more than the fill kernel has threads (narrow codes)
    const int per_launch = kFillWords / per_chunk < kFillThreads ? kFillWords / per_chunk : kFillThreads;
    FillArgs a;
    a.k = static_cast<uint32_t>(k);
    a.rows = static_cast<uint32_t>(m);
    for (int c0 = 0; c0 < n_chunks; c0 += per_launch) {
        const int n = n_chunks - c0 < per_launch ? n_chunks - c0 : per_launch;
        for (int c = 0; c < n; ++c) {
            uint64_t *w = a.words + static_cast<size_t>(c) * per_chunk;
            const size_t bytes = shard_bytes[c0 + c];
            for (int j = 0; j < k; ++j) w[j] = reinterpret_cast<uintptr_t>(data[static_cast<size_t>(c0 + c) * k + j]);
            for (int r = 0; r < m; ++r) w[k + r] = reinterpret_cast<uintptr_t>(parity[static_cast<size_t>(c0 + c) * m + order[r]]);
            w[k + m] = static_cast<uint64_t>(bytes) | (static_cast<uint64_t>(batch_interleave_shift(m, bytes, shape)) << 56);
        }
        a.descs = descs + c0;
        a.count = static_cast<uint32_t>(n);
        hipLaunchKernelGGL(fill_descs_kernel, dim3(1), dim3(kFillThreads), 0, stream, a);
        e = hipGetLastError();
        if (e != hipSuccess) return hip_status(e);
    }
    return hip_status(launch_apply_batch(m, k, code->P.data(), k, descs, n_chunks, max_bytes, shape, stream));
}
catch (...) {
    return caught();
}
