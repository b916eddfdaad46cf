// HIP kernel for gfx950: masked XOR of blocks, the one operation both RDP
// encoding and RDP reconstruction reduce to.
//
// A shard is a sequence of stripes; a stripe is p-1 cells ("rows") of
// cell_bytes each.  Every output cell is the XOR of a set of input cells of
// the same stripe, taken at the same offset inside the cell; the sets arrive
// as one 32-bit mask per input row (bit o = this row is part of output o).  A
// lane handles one vector offset of one stripe: it reads that vector from
// every row of every input shard and XORs it into the accumulators the mask
// names.  With cells that are a multiple of the piece interleave period the
// rows of a stripe sit next to each other in memory (one TLB page, one
// residue class of pieces per XCD), unlike whole-shard rows.  The masks are
// wavefront-uniform, so the selection is a scalar bit test and branch around
// four XORs.  Offsets are dealt to workgroups in the same interleaved 1 KiB
// pieces as the GF(2^8) kernels (a given XCD keeps to one residue class of
// pieces), which is what the HBM rate depends on.
#include <hip/hip_runtime.h>

#include "gs_launch.h"
#include "gs_rdp.h"

namespace gs {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct XorArgs {
    const uint8_t *in[kRdpMaxInputs];
    uint8_t *out[2];
    uint32_t mask[kRdpMaxInputs * kRdpMaxRows];
    uint64_t nvb;       // vectors per row summed over all stripes: shard_bytes / (p-1) / vector bytes
    uint32_t n_in;      // shards read
    uint32_t nx_shift;  // log2 of the piece interleave modulus
    uint32_t cell_shift;  // log2 of the vectors per cell
};

// W = dwords per lane and vector (4 = 16 bytes, 2 = 8 bytes).  The number of
// accumulators is E*(p-1); for the large primes 16-byte vectors would need more
// registers than a wavefront may hold at a useful occupancy, so those use W = 2.
template <int W> struct VecOf;
template <> struct VecOf<4> { typedef uint32_t type __attribute__((ext_vector_type(4))); };
template <> struct VecOf<2> { typedef uint32_t type __attribute__((ext_vector_type(2))); };

template <int P, int E, int W, bool FULL>
__device__ __forceinline__ void xor_tile(const XorArgs &a, uint64_t v)
{
    typedef typename VecOf<W>::type vec;
    constexpr int kRows = P - 1, kOut = E * kRows;
    const bool ok = FULL || v < a.nvb;
    const uint64_t vv = ok ? v : 0;  // always a valid address; the value is dropped
    // row r of this lane's stripe, at this lane's offset inside the cell
    const uint64_t cell_mask = (1ull << a.cell_shift) - 1;
    const uint64_t row0 = (((vv >> a.cell_shift) * kRows) << a.cell_shift) + (vv & cell_mask);
    const uint64_t row_step = 1ull << a.cell_shift;
    vec acc[kOut];
#pragma unroll
    for (int o = 0; o < kOut; ++o) acc[o] = vec(0);

    // Loads of several shards are issued together (about 16 per lane in flight)
    // before their masks are applied: with one shard at a time a lane has only
    // p-1 small loads outstanding, too few to cover HBM latency.
    constexpr int kShards = P <= 5 ? 4 : (P <= 11 ? 2 : 1);
    auto apply = [&](const vec(&x)[kRows], uint32_t s) {
#pragma unroll
        for (int row = 0; row < kRows; ++row) {
            const uint32_t m = a.mask[s * kRows + row];
#pragma unroll
            for (int o = 0; o < kOut; ++o)
                if (m >> o & 1u) acc[o] ^= x[row];
        }
    };
    uint32_t s = 0;
    for (; s + kShards <= a.n_in; s += kShards) {
        vec x[kShards][kRows];
#pragma unroll
        for (int b = 0; b < kShards; ++b) {
            const vec *base = reinterpret_cast<const vec *>(a.in[s + b]) + row0;
#pragma unroll
            for (int row = 0; row < kRows; ++row) x[b][row] = __builtin_nontemporal_load(base + row * row_step);
        }
#pragma unroll
        for (int b = 0; b < kShards; ++b) apply(x[b], s + b);
    }
    for (; s < a.n_in; ++s) {
        const vec *base = reinterpret_cast<const vec *>(a.in[s]) + row0;
        vec x[kRows];
#pragma unroll
        for (int row = 0; row < kRows; ++row) x[row] = __builtin_nontemporal_load(base + row * row_step);
        apply(x, s);
    }
    if (ok) {
#pragma unroll
        for (int o = 0; o < kOut; ++o) {
            vec *dst = reinterpret_cast<vec *>(a.out[o / kRows]) + row0 + (o % kRows) * row_step;
            __builtin_nontemporal_store(acc[o], dst);
        }
    }
}

template <int P, int E, int W>
__global__ __launch_bounds__(kThreads) void rdp_xor_kernel(const XorArgs a)
{
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63u;
    constexpr uint32_t kPieces = kThreads / 64;  // one piece per wavefront
    const uint64_t t = blockIdx.x;
    const uint64_t g = t >> a.nx_shift, r = t & ((1ull << a.nx_shift) - 1);
    if (((g * kPieces) << a.nx_shift) * 64 >= a.nvb) return;
    const uint64_t v = ((((g * kPieces + wave) << a.nx_shift) + r) << 6) + lane;
    if ((((g + 1) * kPieces) << a.nx_shift) * 64 <= a.nvb) xor_tile<P, E, W, true>(a, v);
    else xor_tile<P, E, W, false>(a, v);
}

template <int P, int W>
static hipError_t launch_p(const XorArgs &a, int n_out, dim3 grid, hipStream_t stream)
{
    if (n_out == 1) hipLaunchKernelGGL((rdp_xor_kernel<P, 1, W>), grid, dim3(kThreads), 0, stream, a);
    else hipLaunchKernelGGL((rdp_xor_kernel<P, 2, W>), grid, dim3(kThreads), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_rdp_xor(const RdpPlan &plan, const void *const *shards, size_t shard_bytes,
                          size_t cell_bytes, const LaunchShape &shape, hipStream_t stream)
{
    const int rows = plan.p - 1;
    if (cell_bytes < 16 || (cell_bytes & (cell_bytes - 1)) != 0) return hipErrorInvalidValue;
    const int n_in = static_cast<int>(plan.inputs.size()), n_out = static_cast<int>(plan.outputs.size());
    if (n_in < 1 || n_in > kRdpMaxInputs || n_out < 1 || n_out > 2 || plan.p > kRdpMaxPrime) return hipErrorInvalidValue;
    if (shard_bytes == 0 || shard_bytes % (cell_bytes * rows) != 0) return hipErrorInvalidValue;
    XorArgs a;
    for (int s = 0; s < kRdpMaxInputs; ++s) a.in[s] = s < n_in ? static_cast<const uint8_t *>(shards[plan.inputs[s]]) : nullptr;
    for (int x = 0; x < 2; ++x)
        a.out[x] = x < n_out ? static_cast<uint8_t *>(const_cast<void *>(shards[plan.outputs[x]])) : nullptr;
    for (size_t i = 0; i < sizeof(a.mask) / sizeof(a.mask[0]); ++i) a.mask[i] = i < plan.mask.size() ? plan.mask[i] : 0u;
    // 8-byte vectors measured as fast or faster than 16-byte ones for every prime
    // (fewer registers per accumulator); 16-byte vectors stay selectable for sweeps
    const int w = shape.unroll == 4 ? 4 : 2;  // dwords per lane
    a.nvb = shard_bytes / rows / (4u * w);
    a.cell_shift = 0;
    while ((static_cast<size_t>(4u * w) << a.cell_shift) < cell_bytes) ++a.cell_shift;
    a.n_in = static_cast<uint32_t>(n_in);
    uint32_t nx_shift = shape.interleave_shift >= 0 && shape.interleave_shift <= 10
                            ? static_cast<uint32_t>(shape.interleave_shift) : 5u;
    const uint64_t tile = kThreads;  // vectors per workgroup
    while (nx_shift > 0 && (tile << nx_shift) > a.nvb) --nx_shift;
    const uint64_t super = tile << nx_shift;
    const uint64_t tiles = ((a.nvb + super - 1) / super) << nx_shift;
    if (tiles >= (1ull << 23)) return hipErrorInvalidValue;  // launch limit on workgroups per dimension
    a.nx_shift = nx_shift;
    const dim3 grid(static_cast<uint32_t>(tiles ? tiles : 1));
#define GS_RDP_CASE(P_) \
    case P_: return w == 2 ? launch_p<P_, 2>(a, n_out, grid, stream) : launch_p<P_, 4>(a, n_out, grid, stream);
    switch (plan.p) {
        GS_RDP_CASE(3) GS_RDP_CASE(5) GS_RDP_CASE(7) GS_RDP_CASE(11) GS_RDP_CASE(13) GS_RDP_CASE(17)
        default: return hipErrorInvalidValue;
    }
#undef GS_RDP_CASE
}

}  // namespace gs
