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
    // tiles beyond one grid row continue in the next (gridDim.x is a multiple of the interleave modulus)
    const uint64_t t = static_cast<uint64_t>(blockIdx.y) * gridDim.x + blockIdx.x;
    const uint64_t g = t >> a.nx_shift, r = t & ((1ull << a.nx_shift) - 1);
    if (((g * kPieces) << a.nx_shift) * 64 >= a.nvb) return;
    const uint64_t v = ((((g * kPieces + wave) << a.nx_shift) + r) << 6) + lane;
    if ((((g + 1) * kPieces) << a.nx_shift) * 64 <= a.nvb) rdp_tile<P, E, W, true>(a, v);
    else rdp_tile<P, E, W, false>(a, v);
}

// ---- many chunks in one launch --------------------------------------------------
// blockIdx.y is the chunk; its shard pointers and length come from a descriptor
// in device memory (scalar loads), the plan is the same for every chunk.
struct RdpBatchArgs {
    const RdpBatchDesc *descs;
    uint32_t syndrome_mask[2 * kRdpMaxRows];
    uint32_t cell_shift;
    uint32_t needs_diagonals;
};

typedef const RdpBatchDesc __attribute__((address_space(4))) *ConstRdpDesc;

template <int P, int E, int W>
__global__ __launch_bounds__(kThreads) void rdp_batch_kernel(const RdpBatchArgs b)
{
    ConstRdpDesc d = (ConstRdpDesc)b.descs + blockIdx.y;
    RdpArgs a;
#pragma unroll
    for (int j = 0; j < kRdpMaxDisks; ++j) a.disk[j] = j <= P ? d->disk[j] : nullptr;
    a.out[0] = d->out[0];
    a.out[1] = d->out[1];
#pragma unroll
    for (int i = 0; i < 2 * kRdpMaxRows; ++i) a.syndrome_mask[i] = b.syndrome_mask[i];
    a.nvb = d->nvb;
    a.nx_shift = d->nx_shift;
    a.cell_shift = b.cell_shift;
    a.needs_diagonals = b.needs_diagonals;
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63u;
    constexpr uint32_t kPieces = kThreads / 64;
    const uint64_t t = blockIdx.x;
    const uint64_t g = t >> a.nx_shift, r = t & ((1ull << a.nx_shift) - 1);
    if (((g * kPieces) << a.nx_shift) * 64 >= a.nvb) return;
    const uint64_t v = ((((g * kPieces + wave) << a.nx_shift) + r) << 6) + lane;
    if ((((g + 1) * kPieces) << a.nx_shift) * 64 <= a.nvb) rdp_tile<P, E, W, true>(a, v);
    else rdp_tile<P, E, W, false>(a, v);
}

// LDS reservation of a bulk RDP launch (8-byte vectors; measured for every prime on 1 and 2 GiB shards):
// a wavefront of p = 3 has two loads per disk in flight and needs full occupancy; p = 5 and 7 gain
// 2 to 5 points of HBM peak with three workgroups per CU, p >= 11 with two.  Rebuilds of two data
// shards, whose cells are XORs of many syndromes, want one workgroup more for their arithmetic: four
// at p = 5 and 7 (+1.5 to +2 points over three), three at p = 11 and 13 (at p = 17 the registers allow
// no more than three anyway).  Such plans are told by the share of syndromes in a cell.
static size_t rdp_reservation(const LaunchShape &shape, const RdpPlan &plan, int w, uint64_t workgroups)
{
    const int p = plan.p;
    if (!shape.occupancy_cap || w != 2 || p < 5) return 0;
    // a workgroup moves 2 KiB of each of a disk's p - 1 rows; the reservation pays from 96 MiB per disk
    // on (p = 17: from 256 MiB), below that it costs up to 5 points
    if (workgroups * static_cast<uint64_t>(p - 1) < (p < 17 ? kRdpCapMinRowPieces : 8 * kRdpCapMinRowPieces / 3)) return 0;
    size_t bits = 0;
    for (uint32_t m : plan.syndrome_mask) bits += static_cast<size_t>(__builtin_popcount(m));
    const size_t cells = plan.syndrome_mask.size();
    if (p < 11) return lds_for_workgroups_per_cu(10 * bits > 7 * static_cast<size_t>(p - 1) * cells ? 4 : 3);
    const bool dense = bits > 4 * cells;
    return lds_for_workgroups_per_cu(dense && p < 17 ? 3 : 2);
}

static uint32_t rdp_interleave_shift(uint64_t nvb, const LaunchShape &shape, uint64_t *tiles)
{
    uint32_t nx_shift = shape.interleave_shift >= 0 && shape.interleave_shift <= 10
                            ? static_cast<uint32_t>(shape.interleave_shift) : 5u;
    const uint64_t tile = kThreads;  // vectors per workgroup
    while (nx_shift > 0 && (tile << nx_shift) > nvb) --nx_shift;
    const uint64_t super = tile << nx_shift;
    if (tiles) *tiles = ((nvb + super - 1) / super) << nx_shift;
    return nx_shift;
}

constexpr int kRdpBatchW = 2;  // 8-byte vectors

bool write_rdp_batch_desc(void *slot, int idx, const RdpPlan &plan, const void *const *shards, size_t shard_bytes,
                          size_t cell_bytes, const LaunchShape &shape)
{
    const int rows = plan.p - 1;
    if (shard_bytes % (cell_bytes * rows) != 0) return false;
    RdpBatchDesc &d = static_cast<RdpBatchDesc *>(slot)[idx];
    for (int j = 0; j < kRdpMaxDisks; ++j)
        d.disk[j] = (j <= plan.p && plan.shard_of_disk[j] >= 0 && shard_bytes != 0)
                        ? static_cast<const uint8_t *>(shards[plan.shard_of_disk[j]]) : nullptr;
    for (int x = 0; x < 2; ++x)
        d.out[x] = x < static_cast<int>(plan.outputs.size()) ? static_cast<uint8_t *>(const_cast<void *>(shards[plan.outputs[x]])) : nullptr;
    d.nvb = shard_bytes / rows / (4u * kRdpBatchW);
    d.nx_shift = rdp_interleave_shift(d.nvb ? d.nvb : 1, shape, nullptr);
    d.pad = 0;
    return true;
}

template <int P>
static hipError_t launch_batch_p(const RdpBatchArgs &a, int n_out, dim3 grid, size_t lds, hipStream_t stream)
{
    if (n_out == 1) hipLaunchKernelGGL((rdp_batch_kernel<P, 1, kRdpBatchW>), grid, dim3(kThreads), lds, stream, a);
    else hipLaunchKernelGGL((rdp_batch_kernel<P, 2, kRdpBatchW>), grid, dim3(kThreads), lds, stream, a);
    return hipGetLastError();
}

hipError_t launch_rdp_batch(const RdpPlan &plan, const void *descs_dev, int n_chunks, size_t max_bytes,
                            size_t cell_bytes, const LaunchShape &shape, hipStream_t stream)
{
    const int rows = plan.p - 1;
    const int n_out = static_cast<int>(plan.outputs.size());
    if (n_out < 1 || n_out > 2 || plan.p > kRdpMaxPrime || n_chunks < 1 || n_chunks > 65535) return hipErrorInvalidValue;
    if (cell_bytes < 16 || (cell_bytes & (cell_bytes - 1)) != 0) return hipErrorInvalidValue;
    if (max_bytes == 0) return hipSuccess;
    RdpBatchArgs a;
    a.descs = static_cast<const RdpBatchDesc *>(descs_dev);
    for (int i = 0; i < 2 * kRdpMaxRows; ++i)
        a.syndrome_mask[i] = i < static_cast<int>(plan.syndrome_mask.size()) ? plan.syndrome_mask[i] : 0u;
    a.needs_diagonals = plan.needs_diagonals ? 1u : 0u;
    a.cell_shift = 0;
    while ((static_cast<size_t>(4u * kRdpBatchW) << a.cell_shift) < cell_bytes) ++a.cell_shift;
    uint64_t tiles = 0;
    rdp_interleave_shift(max_bytes / rows / (4u * kRdpBatchW), shape, &tiles);
    if (tiles >= (1ull << 23)) return hipErrorInvalidValue;
    const dim3 grid(static_cast<uint32_t>(tiles ? tiles : 1), static_cast<uint32_t>(n_chunks));
    // chunks differ in length: never fewer than three workgroups per CU
    size_t lds = rdp_reservation(shape, plan, kRdpBatchW, tiles * static_cast<uint64_t>(n_chunks));
    if (lds > lds_for_workgroups_per_cu(3)) lds = lds_for_workgroups_per_cu(3);
#define GS_RDP_BATCH_CASE(P_) case P_: return launch_batch_p<P_>(a, n_out, grid, lds, stream);
    switch (plan.p) {
        GS_RDP_BATCH_CASE(3) GS_RDP_BATCH_CASE(5) GS_RDP_BATCH_CASE(7) GS_RDP_BATCH_CASE(11) GS_RDP_BATCH_CASE(13)
        GS_RDP_BATCH_CASE(17)
        default: return hipErrorInvalidValue;
    }
#undef GS_RDP_BATCH_CASE
}

// ---- the same two steps over a paged pool ---------------------------------------
// A cell is one page, a stripe p-1 consecutive page slots of a plane; data
// disks are rows of the block table, parity disks dense buffers laid out
// [plane][slot][page] (on either side: a lost data shard is rebuilt into the
// pages of its table row).  Pages are at least 1 KiB, so the 64 lanes of a
// piece share one cell: stripe, slot and page id are wavefront-uniform and the
// table entries come through scalar loads.  A page id outside the plane reads
// as zeros and is not written.
struct RdpPagedArgs {
    const uint8_t *const *plane_base;   // device array [n_planes]
    const int32_t *table;               // device; row stride table_stride, first slot of the window
    const uint8_t *dense[kRdpMaxDisks]; // stripe disks 0..p that are dense buffers (else nullptr)
    int32_t row[kRdpMaxDisks];          // table row of a paged disk, -1 otherwise
    uint32_t stride[kRdpMaxDisks];      // dense: vectors from plane to plane
    uint8_t *out_dense[2];
    int32_t out_row[2];
    uint32_t out_stride[2];
    uint32_t syndrome_mask[2 * kRdpMaxRows];
    uint64_t pages_per_plane;
    uint64_t nvb;            // vectors per row summed over the stripes of one plane (multiple of 64)
    uint32_t table_stride;
    uint32_t nx_shift;
    uint32_t cell_shift;     // log2 of the vectors per cell (= per page)
    uint32_t needs_diagonals;
};

typedef const int32_t __attribute__((address_space(4))) *ConstTableRdp;

template <int P, int E, int W>
__global__ __launch_bounds__(kThreads) void rdp_paged_kernel(const RdpPagedArgs a)
{
    typedef typename VecOf<W>::type vec;
    constexpr int kRows = P - 1;
    constexpr uint32_t kPieces = kThreads / 64;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63u;
    const uint32_t plane = blockIdx.y;
    const uint64_t t = blockIdx.x;
    const uint64_t g = t >> a.nx_shift, r = t & ((1ull << a.nx_shift) - 1);
    const uint64_t piece = (((g * kPieces + wave) << a.nx_shift) + r) << 6;  // first vector of this wavefront's piece
    if (piece >= a.nvb) return;  // nvb is a multiple of 64: a piece is inside the plane or outside as a whole
    const uint64_t vpc = 1ull << a.cell_shift;
    const uint64_t stripe = piece >> a.cell_shift;
    const uint64_t off = (piece & (vpc - 1)) + lane;  // this lane's vector inside its cell
    const uint8_t *pbase = a.plane_base[plane];
    const bool diagonals = a.needs_diagonals != 0;

    // page of table row `trow` at `slot`, or -1
    auto page_of = [&](int32_t trow, uint64_t slot) -> int64_t {
        const int64_t page = ((ConstTableRdp)a.table)[static_cast<uint64_t>(trow) * a.table_stride + slot];
        return static_cast<uint64_t>(page) < a.pages_per_plane ? page : -1;
    };

    vec sr[kRows], sd[kRows];
#pragma unroll
    for (int i = 0; i < kRows; ++i) {
        sr[i] = vec(0);
        sd[i] = vec(0);
    }
#pragma unroll
    for (int j = 0; j <= P; ++j) {
        const int32_t trow = a.row[j];
        const uint8_t *dense = a.dense[j];
        if (trow < 0 && dense == nullptr) continue;   // disk absent (imaginary, missing, or not needed)
        if (j == P && !diagonals) continue;
        // one branch per disk, then all of its table entries, then all of its loads: the p-1
        // loads of a disk are in flight together
        vec x[kRows];
        if (trow >= 0) {
            int64_t page[kRows];
#pragma unroll
            for (int row = 0; row < kRows; ++row) page[row] = page_of(trow, stripe * kRows + row);
#pragma unroll
            for (int row = 0; row < kRows; ++row) {
                const vec *src = reinterpret_cast<const vec *>(pbase) + (page[row] < 0 ? 0 : static_cast<uint64_t>(page[row])) * vpc + off;
                x[row] = __builtin_nontemporal_load(src);
            }
#pragma unroll
            for (int row = 0; row < kRows; ++row)
                if (page[row] < 0) x[row] = vec(0);
        } else {
            const vec *src = reinterpret_cast<const vec *>(dense) + static_cast<uint64_t>(plane) * a.stride[j] + (stripe * kRows) * vpc + off;
#pragma unroll
            for (int row = 0; row < kRows; ++row) x[row] = __builtin_nontemporal_load(src + row * vpc);
        }
        if (j < P) {
#pragma unroll
            for (int row = 0; row < kRows; ++row) sr[row] ^= x[row];
            if (diagonals) {
#pragma unroll
                for (int row = 0; row < kRows; ++row) {
                    constexpr int kNone = P - 1;
                    const int d = (row + j) % P;
                    if (d != kNone) sd[d] ^= x[row];
                }
            }
        } else {
#pragma unroll
            for (int d = 0; d < kRows; ++d) sd[d] ^= x[d];
        }
    }

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
        const int x = o / kRows;
        const uint64_t slot = stripe * kRows + (o % kRows);
        const int32_t trow = a.out_row[x];
        if (trow >= 0) {
            const int64_t page = page_of(trow, slot);
            if (page < 0) continue;
            vec *dst = reinterpret_cast<vec *>(const_cast<uint8_t *>(pbase)) + static_cast<uint64_t>(page) * vpc + off;
            __builtin_nontemporal_store(acc, dst);
        } else {
            vec *dst = reinterpret_cast<vec *>(a.out_dense[x]) + static_cast<uint64_t>(plane) * a.out_stride[x] + slot * vpc + off;
            __builtin_nontemporal_store(acc, dst);
        }
    }
}

template <int P, int W>
static hipError_t launch_paged_p(const RdpPagedArgs &a, int n_out, dim3 grid, hipStream_t stream)
{
    if (n_out == 1) hipLaunchKernelGGL((rdp_paged_kernel<P, 1, W>), grid, dim3(kThreads), 0, stream, a);
    else hipLaunchKernelGGL((rdp_paged_kernel<P, 2, W>), grid, dim3(kThreads), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_rdp_paged(const RdpPlan &plan, const void *const *plane_base_dev, int n_planes, size_t page_bytes,
                            int64_t pages_per_plane, const int32_t *table_dev, int table_stride, int n_slots,
                            const PagedStream *shards, const LaunchShape &shape, hipStream_t stream)
{
    const int rows = plan.p - 1;
    const int n_out = static_cast<int>(plan.outputs.size());
    if (n_out < 1 || n_out > 2 || plan.p > kRdpMaxPrime) return hipErrorInvalidValue;
    if (page_bytes < 1024 || (page_bytes & (page_bytes - 1)) != 0) return hipErrorInvalidValue;
    if (n_planes < 1 || n_planes > 65535 || n_slots < 1 || n_slots % rows != 0 || table_stride < n_slots ||
        pages_per_plane < 1)
        return hipErrorInvalidValue;
    (void)shape;
    constexpr int w = 2;  // 8-byte vectors, as in the contiguous kernel
    const uint64_t vec_bytes = 4u * w;
    RdpPagedArgs a;
    const uint64_t packed = static_cast<uint64_t>(n_slots) * page_bytes / vec_bytes;  // dense: vectors per plane
    auto stride_of = [&](const PagedStream &s, uint32_t &out) {
        const uint64_t v = s.plane_stride_bytes == 0 ? packed : s.plane_stride_bytes / vec_bytes;
        if ((s.plane_stride_bytes % vec_bytes) != 0 || v < packed || v >= (1ull << 32)) return false;
        out = static_cast<uint32_t>(v);
        return true;
    };
    for (int j = 0; j < kRdpMaxDisks; ++j) {
        a.dense[j] = nullptr;
        a.row[j] = -1;
        a.stride[j] = 0;
        if (j > plan.p || plan.shard_of_disk[j] < 0) continue;
        const PagedStream &s = shards[plan.shard_of_disk[j]];
        if (s.table_row >= 0) {
            a.row[j] = s.table_row;
        } else {
            if (s.dense == nullptr || !stride_of(s, a.stride[j])) return hipErrorInvalidValue;
            a.dense[j] = static_cast<const uint8_t *>(s.dense);
        }
    }
    for (int x = 0; x < 2; ++x) {
        a.out_dense[x] = nullptr;
        a.out_row[x] = -1;
        a.out_stride[x] = 0;
        if (x >= n_out) continue;
        const PagedStream &s = shards[plan.outputs[x]];
        if (s.table_row >= 0) {
            a.out_row[x] = s.table_row;
        } else {
            if (s.dense == nullptr || !stride_of(s, a.out_stride[x])) return hipErrorInvalidValue;
            a.out_dense[x] = static_cast<uint8_t *>(const_cast<void *>(s.dense));
        }
    }
    for (int i = 0; i < 2 * kRdpMaxRows; ++i)
        a.syndrome_mask[i] = i < static_cast<int>(plan.syndrome_mask.size()) ? plan.syndrome_mask[i] : 0u;
    a.needs_diagonals = plan.needs_diagonals ? 1u : 0u;
    a.plane_base = reinterpret_cast<const uint8_t *const *>(plane_base_dev);
    a.table = table_dev;
    a.table_stride = static_cast<uint32_t>(table_stride);
    a.pages_per_plane = static_cast<uint64_t>(pages_per_plane < (1ll << 31) ? pages_per_plane : (1ll << 31));
    a.cell_shift = 0;
    while ((vec_bytes << a.cell_shift) < page_bytes) ++a.cell_shift;
    a.nvb = static_cast<uint64_t>(n_slots / rows) << a.cell_shift;
    uint32_t nx_shift = 5u;
    const uint64_t tile = kThreads;
    while (nx_shift > 0 && (tile << nx_shift) > a.nvb) --nx_shift;
    const uint64_t super = tile << nx_shift;
    const uint64_t tiles = ((a.nvb + super - 1) / super) << nx_shift;
    if (tiles >= (1ull << 23)) return hipErrorInvalidValue;
    a.nx_shift = nx_shift;
    const dim3 grid(static_cast<uint32_t>(tiles ? tiles : 1), static_cast<uint32_t>(n_planes));
#define GS_RDP_PAGED_CASE(P_) case P_: return launch_paged_p<P_, w>(a, n_out, grid, stream);
    switch (plan.p) {
        GS_RDP_PAGED_CASE(3) GS_RDP_PAGED_CASE(5) GS_RDP_PAGED_CASE(7) GS_RDP_PAGED_CASE(11) GS_RDP_PAGED_CASE(13)
        GS_RDP_PAGED_CASE(17)
        default: return hipErrorInvalidValue;
    }
#undef GS_RDP_PAGED_CASE
}

template <int P, int W>
static hipError_t launch_p(const RdpArgs &a, int n_out, dim3 grid, size_t lds, hipStream_t stream)
{
    if (n_out == 1) hipLaunchKernelGGL((rdp_kernel<P, 1, W>), grid, dim3(kThreads), lds, stream, a);
    else hipLaunchKernelGGL((rdp_kernel<P, 2, W>), grid, dim3(kThreads), lds, stream, a);
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
    // a grid row holds at most 2^22 workgroups (a power of two, so a multiple of the interleave modulus);
    // longer shards take further rows
    constexpr uint64_t kRowTiles = 1ull << 22;
    const uint64_t grid_rows = (tiles + kRowTiles - 1) / kRowTiles;
    if (grid_rows > 65535) return hipErrorInvalidValue;
    a.nx_shift = nx_shift;
    const dim3 grid(static_cast<uint32_t>(tiles <= kRowTiles ? (tiles ? tiles : 1) : kRowTiles),
                    static_cast<uint32_t>(grid_rows ? grid_rows : 1));
    const size_t lds = rdp_reservation(shape, plan, w, tiles);
#define GS_RDP_CASE(P_) \
    case P_: return w == 2 ? launch_p<P_, 2>(a, n_out, grid, lds, stream) : launch_p<P_, 4>(a, n_out, grid, lds, stream);
    switch (plan.p) {
        GS_RDP_CASE(3) GS_RDP_CASE(5) GS_RDP_CASE(7) GS_RDP_CASE(11) GS_RDP_CASE(13) GS_RDP_CASE(17)
        default: return hipErrorInvalidValue;
    }
#undef GS_RDP_CASE
}

}  // namespace gs
