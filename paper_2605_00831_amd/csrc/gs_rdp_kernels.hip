// HIP kernel for gfx950: RDP (row-diagonal parity) encode and rebuild.
//
// A shard is a sequence of stripes; a stripe is p-1 cells ("rows") of
// cell_bytes per shard.  A lane handles one vector offset of one stripe in
// two steps:
//   1. syndromes: it reads that vector from every row of every shard that is
//      present and accumulates SR[i] (row i over disks 0..p-1) and SD[d]
//      (diagonal d over disks 0..p-1, plus diagonal-parity cell d).  Which
//      accumulator a cell goes to depends only on (row, disk), so this step
//      is straight-line code: no masks, no branches except "disk absent".
//   2. outputs: every missing cell is the XOR of a set of syndromes, given as
//      a 32-bit mask per output row (wavefront-uniform: scalar bit test and
//      branch around the XOR).  Encoding is the case "both parity shards
//      missing".
// The diagonal walk of the published reconstruction is thereby replaced by a
// host-solved linear map from syndromes to cells; the device never needs a
// dynamic register index.  Offsets are dealt to workgroups in the same
// interleaved pieces as the GF(2^8) kernels; with cells that are a multiple of
// the interleave period the rows of a stripe sit next to each other in memory
// (one TLB page, one residue class of pieces per XCD).
#include <hip/hip_runtime.h>

#include "gs_launch.h"
#include "gs_rdp.h"

namespace gs {

struct RdpArgs {
    const uint8_t *disk[kRdpMaxDisks];  // stripe disks 0..p, nullptr = not read
    uint8_t *out[2];
    uint32_t syndrome_mask[2 * kRdpMaxRows];
    uint64_t nvb;            // vectors per row summed over all stripes
    uint32_t nx_shift;       // log2 of the piece interleave modulus
    uint32_t cell_shift;     // log2 of the vectors per cell
    uint32_t needs_diagonals;
};

// W = dwords per lane and vector (4 = 16 bytes, 2 = 8 bytes): 2(p-1) syndromes
// live in registers, so the large primes want the narrower vector.
template <int W> struct VecOf;
template <> struct VecOf<4> { typedef uint32_t type __attribute__((ext_vector_type(4))); };
template <> struct VecOf<2> { typedef uint32_t type __attribute__((ext_vector_type(2))); };

template <int P, int E, int W, bool FULL>
__device__ __forceinline__ void rdp_tile(const RdpArgs &a, uint64_t v)
{
    typedef typename VecOf<W>::type vec;
    constexpr int kRows = P - 1;
    const bool ok = FULL || v < a.nvb;
    const uint64_t vv = ok ? v : 0;  // always a valid address; the value is dropped
    // row r of this lane's stripe, at this lane's offset inside the cell
    const uint64_t cell_mask = (1ull << a.cell_shift) - 1;
    const uint64_t row0 = (((vv >> a.cell_shift) * kRows) << a.cell_shift) + (vv & cell_mask);
    const uint64_t row_step = 1ull << a.cell_shift;
    const bool diagonals = a.needs_diagonals != 0;

    vec sr[kRows], sd[kRows];
#pragma unroll
    for (int i = 0; i < kRows; ++i) {
        sr[i] = vec(0);
        sd[i] = vec(0);
    }
#pragma unroll
    for (int j = 0; j < P; ++j) {  // data disks and the row-parity disk
        const uint8_t *disk = a.disk[j];
        if (disk == nullptr) continue;
        const vec *base = reinterpret_cast<const vec *>(disk) + row0;
        vec x[kRows];
#pragma unroll
        for (int row = 0; row < kRows; ++row) x[row] = __builtin_nontemporal_load(base + row * row_step);
#pragma unroll
        for (int row = 0; row < kRows; ++row) sr[row] ^= x[row];
        if (diagonals) {
#pragma unroll
            for (int row = 0; row < kRows; ++row) {
                constexpr int kNone = P - 1;  // the diagonal that is not stored
                const int d = (row + j) % P;
                if (d != kNone) sd[d] ^= x[row];
            }
        }
    }
    if (diagonals && a.disk[P] != nullptr) {
        const vec *base = reinterpret_cast<const vec *>(a.disk[P]) + row0;
#pragma unroll
        for (int d = 0; d < kRows; ++d) sd[d] ^= __builtin_nontemporal_load(base + d * row_step);
    }

    if (!ok) return;
#pragma unroll
    for (int o = 0; o < E * kRows; ++o) {
        const uint32_t m = a.syndrome_mask[o];
        vec acc = vec(0);
#pragma unroll
        for (int i = 0; i < kRows; ++i)
            if (m >> i & 1u) acc ^= sr[i];
        if (diagonals) {
#pragma unroll
            for (int d = 0; d < kRows; ++d)
                if (m >> (kRows + d) & 1u) acc ^= sd[d];
        }
        vec *dst = reinterpret_cast<vec *>(a.out[o / kRows]) + row0 + (o % kRows) * row_step;
        __builtin_nontemporal_store(acc, dst);
    }
}

template <int P, int E, int W>
__global__ __launch_bounds__(kThreads) void rdp_kernel(const RdpArgs a)
{
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63u;
    constexpr uint32_t kPieces = kThreads / 64;  // one piece per wavefront
    const uint64_t t = blockIdx.x;
    const uint64_t g = t >> a.nx_shift, r = t & ((1ull << a.nx_shift) - 1);
    if (((g * kPieces) << a.nx_shift) * 64 >= a.nvb) return;
    const uint64_t v = ((((g * kPieces + wave) << a.nx_shift) + r) << 6) + lane;
    if ((((g + 1) * kPieces) << a.nx_shift) * 64 <= a.nvb) rdp_tile<P, E, W, true>(a, v);
    else rdp_tile<P, E, W, false>(a, v);
}

template <int P, int W>
static hipError_t launch_p(const RdpArgs &a, int n_out, dim3 grid, hipStream_t stream)
{
    if (n_out == 1) hipLaunchKernelGGL((rdp_kernel<P, 1, W>), grid, dim3(kThreads), 0, stream, a);
    else hipLaunchKernelGGL((rdp_kernel<P, 2, W>), grid, dim3(kThreads), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_rdp(const RdpPlan &plan, const void *const *shards, size_t shard_bytes,
                      size_t cell_bytes, const LaunchShape &shape, hipStream_t stream)
{
    const int rows = plan.p - 1;
    const int n_out = static_cast<int>(plan.outputs.size());
    if (n_out < 1 || n_out > 2 || plan.p > kRdpMaxPrime) return hipErrorInvalidValue;
    if (cell_bytes < 16 || (cell_bytes & (cell_bytes - 1)) != 0) return hipErrorInvalidValue;
    if (shard_bytes == 0 || shard_bytes % (cell_bytes * rows) != 0) return hipErrorInvalidValue;
    RdpArgs a;
    for (int j = 0; j < kRdpMaxDisks; ++j)
        a.disk[j] = (j <= plan.p && plan.shard_of_disk[j] >= 0) ? static_cast<const uint8_t *>(shards[plan.shard_of_disk[j]]) : nullptr;
    for (int x = 0; x < 2; ++x)
        a.out[x] = x < n_out ? static_cast<uint8_t *>(const_cast<void *>(shards[plan.outputs[x]])) : nullptr;
    for (int i = 0; i < 2 * kRdpMaxRows; ++i)
        a.syndrome_mask[i] = i < static_cast<int>(plan.syndrome_mask.size()) ? plan.syndrome_mask[i] : 0u;
    a.needs_diagonals = plan.needs_diagonals ? 1u : 0u;
    // 8-byte vectors measured as fast or faster than 16-byte ones for every prime
    // (fewer registers per syndrome); 16-byte vectors stay selectable for sweeps
    const int w = shape.unroll == 4 ? 4 : 2;  // dwords per lane
    a.nvb = shard_bytes / rows / (4u * w);
    a.cell_shift = 0;
    while ((static_cast<size_t>(4u * w) << a.cell_shift) < cell_bytes) ++a.cell_shift;
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
