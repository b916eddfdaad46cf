// HIP kernel for gfx950: masked XOR of blocks, the one operation both RDP
// encoding and RDP reconstruction reduce to.
//
// A shard of S bytes is p-1 blocks ("rows") of B = S/(p-1) bytes.  Every
// output block is the XOR of a set of input blocks taken at the same offset
// inside the block; the sets arrive as one 32-bit mask per input block (bit o
// = this block is part of output o).  A lane handles one 16-byte vector offset
// v inside the block: it reads that vector from every row of every input
// shard and XORs it into the accumulators the mask names.  The masks are
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
    uint64_t nvb;       // 16-byte vectors per block
    uint32_t n_in;      // shards read
    uint32_t nx_shift;  // log2 of the piece interleave modulus
};

template <int P, int E, bool FULL>
__device__ __forceinline__ void xor_tile(const XorArgs &a, uint64_t v)
{
    constexpr int kRows = P - 1, kOut = E * kRows;
    const bool ok = FULL || v < a.nvb;
    const uint64_t vv = ok ? v : 0;  // always a valid address; the value is dropped
    u32x4 acc[kOut];
#pragma unroll
    for (int o = 0; o < kOut; ++o) acc[o] = u32x4{0, 0, 0, 0};

    for (uint32_t s = 0; s < a.n_in; ++s) {
        const u32x4 *base = reinterpret_cast<const u32x4 *>(a.in[s]) + vv;
        u32x4 x[kRows];
#pragma unroll
        for (int row = 0; row < kRows; ++row) x[row] = __builtin_nontemporal_load(base + row * a.nvb);
#pragma unroll
        for (int row = 0; row < kRows; ++row) {
            const uint32_t m = a.mask[s * kRows + row];
#pragma unroll
            for (int o = 0; o < kOut; ++o)
                if (m >> o & 1u) acc[o] ^= x[row];
        }
    }
    if (ok) {
#pragma unroll
        for (int o = 0; o < kOut; ++o) {
            u32x4 *dst = reinterpret_cast<u32x4 *>(a.out[o / kRows]) + (o % kRows) * a.nvb + v;
            __builtin_nontemporal_store(acc[o], dst);
        }
    }
}

template <int P, int E>
__global__ __launch_bounds__(kThreads) void rdp_xor_kernel(const XorArgs a)
{
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63u;
    constexpr uint32_t kPieces = kThreads / 64;  // one piece per wavefront
    const uint64_t t = blockIdx.x;
    const uint64_t g = t >> a.nx_shift, r = t & ((1ull << a.nx_shift) - 1);
    if (((g * kPieces) << a.nx_shift) * 64 >= a.nvb) return;
    const uint64_t v = ((((g * kPieces + wave) << a.nx_shift) + r) << 6) + lane;
    if ((((g + 1) * kPieces) << a.nx_shift) * 64 <= a.nvb) xor_tile<P, E, true>(a, v);
    else xor_tile<P, E, false>(a, v);
}

template <int P>
static hipError_t launch_p(const XorArgs &a, int n_out, dim3 grid, hipStream_t stream)
{
    if (n_out == 1) hipLaunchKernelGGL((rdp_xor_kernel<P, 1>), grid, dim3(kThreads), 0, stream, a);
    else hipLaunchKernelGGL((rdp_xor_kernel<P, 2>), grid, dim3(kThreads), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_rdp_xor(const RdpPlan &plan, const void *const *shards, size_t shard_bytes,
                          const LaunchShape &shape, hipStream_t stream)
{
    const int rows = plan.p - 1;
    const int n_in = static_cast<int>(plan.inputs.size()), n_out = static_cast<int>(plan.outputs.size());
    if (n_in < 1 || n_in > kRdpMaxInputs || n_out < 1 || n_out > 2 || plan.p > kRdpMaxPrime) return hipErrorInvalidValue;
    if (shard_bytes == 0 || shard_bytes % (16u * rows) != 0) return hipErrorInvalidValue;
    XorArgs a;
    for (int s = 0; s < kRdpMaxInputs; ++s) a.in[s] = s < n_in ? static_cast<const uint8_t *>(shards[plan.inputs[s]]) : nullptr;
    for (int x = 0; x < 2; ++x)
        a.out[x] = x < n_out ? static_cast<uint8_t *>(const_cast<void *>(shards[plan.outputs[x]])) : nullptr;
    for (size_t i = 0; i < sizeof(a.mask) / sizeof(a.mask[0]); ++i) a.mask[i] = i < plan.mask.size() ? plan.mask[i] : 0u;
    a.nvb = shard_bytes / rows / 16;
    a.n_in = static_cast<uint32_t>(n_in);
    uint32_t nx_shift = shape.interleave_shift >= 0 && shape.interleave_shift <= 10
                            ? static_cast<uint32_t>(shape.interleave_shift) : 5u;
    const uint64_t tile = kThreads;  // vectors per workgroup
    while (nx_shift > 0 && (tile << nx_shift) > a.nvb) --nx_shift;
    const uint64_t super = tile << nx_shift;
    const uint64_t tiles = ((a.nvb + super - 1) / super) << nx_shift;
    if (tiles >= (1ull << 22)) return hipErrorInvalidValue;  // 2^22 workgroups of 4 KiB per block row
    a.nx_shift = nx_shift;
    const dim3 grid(static_cast<uint32_t>(tiles ? tiles : 1));
    switch (plan.p) {
        case 3: return launch_p<3>(a, n_out, grid, stream);
        case 5: return launch_p<5>(a, n_out, grid, stream);
        case 7: return launch_p<7>(a, n_out, grid, stream);
        case 11: return launch_p<11>(a, n_out, grid, stream);
        case 13: return launch_p<13>(a, n_out, grid, stream);
        case 17: return launch_p<17>(a, n_out, grid, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace gs
