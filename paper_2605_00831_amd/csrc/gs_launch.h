// Internal interface between the C ABI layer and the HIP kernels.
#pragma once
#include <hip/hip_runtime_api.h>
#include <cstddef>
#include <cstdint>

namespace gs {

constexpr int kLaunchMaxK = 16;  // input streams per launch
constexpr int kLaunchMaxM = 4;   // output rows per launch
constexpr int kThreads = 256;    // lanes per workgroup (4 wavefronts of 64)

struct LaunchShape {
    int unroll;        // 16-byte vectors per lane per stream per tile: 1, 2 or 4; 0 = per kernel family
    int tiles_per_wg;  // consecutive tiles per workgroup
    int nontemporal;   // streaming cache policy on loads and stores
    int interleave_shift;  // log2 of the XCD interleave modulus of the contiguous kernel (0 = off)
    int occupancy_cap;     // bulk launches reserve LDS so that fewer workgroups share a CU (see lds_for_workgroups_per_cu)
    int size_forms;        // 1: small launches and rebuilds of 3-4 shards run kernel forms of their own; 0 / 2: see gs_set_size_forms
};

// Resident workgroups per CU are limited by handing every workgroup a slice of
// the CU's 160 KiB of LDS that it never touches.  The streaming kernels move
// more bytes per second with 2 to 4 workgroups (8 to 16 wavefronts) on a CU
// than with the 8 their registers allow: fewer pieces of fewer streams are open
// at once in the memory system.  Which count is best depends on the arithmetic
// a wavefront does per load, so each launcher picks it per kernel variant;
// launches too small to fill the chip several times over are left alone.
// 0 = no reservation.
constexpr size_t lds_for_workgroups_per_cu(int n) { return n == 2 ? 65536 : n == 3 ? 53248 : n == 4 ? 40960 : 0; }
// Launches below these sizes keep the default occupancy (measured crossovers; a workgroup of the
// GF(2^8) kernels moves 8 KiB of every stream, one of the RDP kernels 2 KiB of each of a disk's p - 1 rows):
constexpr uint64_t kCapMinWorkgroupsRows = 6144;     // table kernels of two and more rows, Horner kernel: 48 MiB shards
constexpr uint64_t kCapMinWorkgroupsOneRow = 12288;  // table kernels of one row: 96 MiB shards
constexpr uint64_t kRdpCapMinRowPieces = 49152;      // RDP, workgroups x (p - 1): 96 MiB disks

// The other end: a launch of at most this many workgroups (half of what the
// chip holds at once: 256 CUs x 8) is over when its slowest wavefront is, and
// a wavefront's time is its memory round trips one after the other.  Such
// launches (grouped ones: half as many workgroups over all chunks) run
// kernel forms that issue the loads of four streams together
// (measured from a host thread, launch to idle: 8+2 on 4 MiB shards 26.1 ->
// 23.7 us, 16+2 on 2 MiB shards 30.8 -> 27.0 us; from 2048 workgroups on one
// stream at a time is the faster form again).
constexpr uint32_t kSmallWorkgroups = 1024;

// One launch: out[r] (r < rows <= 4) = XOR_j coef[r*coef_stride + j] (x) in[j], j < k <= 16,
// over `bytes` bytes; with accumulate the previous contents of out[r] are XORed in.
hipError_t launch_apply(int rows, int k, const uint8_t *coef, int coef_stride,
                        const void *const *in, void *const *out, size_t bytes,
                        bool accumulate, const LaunchShape &shape, hipStream_t stream);

// Encode of the power code (coef must be P[r][j] = 2^(r*j), 2 <= rows <= 3,
// k <= kLaunchMaxK) by Horner's rule instead of table lookups; same bytes out.
hipError_t launch_horner(int rows, int k, const uint8_t *coef, int coef_stride, const void *const *in,
                         void *const *out, size_t bytes, const LaunchShape &shape, hipStream_t stream);

// A stream of the paged variant: the pages named by row `table_row` of the
// block table (table_row >= 0), or a dense device buffer laid out
// [plane][slot][page bytes] like the parity buffers (table_row < 0).
struct PagedStream {
    int table_row;
    const void *dense;
    size_t plane_stride_bytes = 0;  // dense only: bytes from one plane's part to the next (0 = packed)
};

// One launch of the paged variant: k input streams, `rows` output streams,
// over n_slots page slots per plane.  table_dev points at the first slot's
// entry of table row 0; rows are table_stride entries apart (>= n_slots), so
// a launch can cover a window of the slots of a larger table.
hipError_t launch_apply_paged(int rows, int k, const uint8_t *coef, int coef_stride,
                              const void *const *plane_base_dev, int n_planes,
                              size_t page_bytes, int64_t pages_per_plane,
                              const int32_t *table_dev, int table_stride, int n_slots,
                              const PagedStream *in, const PagedStream *out, bool accumulate,
                              const LaunchShape &shape, hipStream_t stream);

// one chunk of a batched launch, as the kernel reads it from device memory
struct BatchDesc {
    const uint8_t *in[kLaunchMaxK];
    uint8_t *out[kLaunchMaxM];   // in the launch's row order (batch_row_order)
    uint64_t nvec;               // whole 16-byte vectors per stream
    uint32_t tail;               // trailing bytes after the last whole vector (0..15)
    uint32_t nx_shift;           // log2 of this chunk's piece interleave modulus
};
constexpr size_t kBatchDescBytes = 8 * (kLaunchMaxK + kLaunchMaxM) + 16;

// Batched form: n_chunks independent stream sets in one launch (blockIdx.y =
// chunk).  Descriptors are written on the host with write_batch_desc() into a
// buffer of n * batch_desc_bytes() bytes, copied to the device by the caller,
// and passed as descs_dev.  max_bytes is the largest chunk's stream length.
size_t batch_desc_bytes();
// order[kLaunchMaxM]: which matrix row each output position of the launch takes
// (an all-ones row moves to position 0); the same for every chunk of a call
void batch_row_order(int rows, int k, const uint8_t *coef, int coef_stride, int *order);
// log2 of the piece interleave modulus the kernel uses for a stream of `bytes`
uint32_t batch_interleave_shift(int rows, size_t bytes, const LaunchShape &shape);
void write_batch_desc(void *slot, int idx, int rows, int k, const int *order, const void *const *in,
                      void *const *out, size_t bytes, const LaunchShape &shape);
hipError_t launch_apply_batch(int rows, int k, const uint8_t *coef, int coef_stride, const void *descs_dev,
                              int n_chunks, size_t max_bytes, const LaunchShape &shape, hipStream_t stream);

struct RdpPlan;
// RDP: accumulate the stripe syndromes from the shards the plan reads and
// form the plan's outputs from them, stripe by stripe.  shards[] is indexed
// by shard id (0..k-1 data, k row parity, k+1 diagonal parity); cell_bytes is
// a power of two >= 16 and shard_bytes a multiple of (p-1)*cell_bytes.
hipError_t launch_rdp(const RdpPlan &plan, const void *const *shards, size_t shard_bytes,
                      size_t cell_bytes, const LaunchShape &shape, hipStream_t stream);

// RDP, many chunks in one launch: descriptors of kBatchDescBytes each, written
// with write_rdp_batch_desc() (false if a chunk is not whole stripes) and copied
// to the device by the caller; one plan for all chunks.
struct RdpBatchDesc {
    const uint8_t *disk[18];  // stripe disks 0..p, nullptr = not read
    uint8_t *out[2];
    uint64_t nvb;             // 8-byte vectors per row summed over the chunk's stripes
    uint32_t nx_shift;
    uint32_t pad;
};
static_assert(sizeof(RdpBatchDesc) == kBatchDescBytes, "both descriptor kinds share the batch object's slots");
bool write_rdp_batch_desc(void *slot, int idx, const RdpPlan &plan, const void *const *shards, size_t shard_bytes,
                          size_t cell_bytes, const LaunchShape &shape);
hipError_t launch_rdp_batch(const RdpPlan &plan, const void *descs_dev, int n_chunks, size_t max_bytes,
                            size_t cell_bytes, const LaunchShape &shape, hipStream_t stream);

// RDP over a paged pool: a cell is one page (a power of two >= 1 KiB), a stripe
// p-1 consecutive page slots of a plane (n_slots a multiple of p-1).  shards[]
// is indexed by shard id like the contiguous form; each is a table row or a
// dense buffer laid out [plane][slot][page].
hipError_t launch_rdp_paged(const RdpPlan &plan, const void *const *plane_base_dev, int n_planes, size_t page_bytes,
                            int64_t pages_per_plane, const int32_t *table_dev, int table_stride, int n_slots,
                            const PagedStream *shards, const LaunchShape &shape, hipStream_t stream);

}  // namespace gs
