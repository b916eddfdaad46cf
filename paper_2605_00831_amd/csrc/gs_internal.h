// Definitions shared by the translation units of the library (not public).
#pragma once
#include <hip/hip_runtime_api.h>
#include <cstdint>
#include <vector>

#include "gs_gf.h"
#include "gs_launch.h"
#include "gs_rdp.h"

struct gs_code {
    int k = 0, m = 0, kind = 0;
    gs::Matrix P;  // m x k parity block, row-major (empty for RDP)
    gs::RdpPlan rdp_encode;  // RDP only
    size_t rdp_cell = 0;     // RDP only: bytes per cell
    bool is_rdp() const { return kind == 2; }
};

namespace gs {

extern thread_local int g_last_hip_error;
int hip_status(hipError_t e);
// status for the exception in flight (call inside a catch block): no C++
// exception may cross the C boundary
int caught();
LaunchShape current_shape();

int apply_matrix(int rows, int cols, const uint8_t *C, const void *const *in, void *const *out,
                 size_t bytes, hipStream_t stream);
int check_erasures(const gs_code *code, const int *erased, int n_erased, std::vector<uint8_t> &lost);
// shard ids a rebuild of `erased` reads (any code kind); validates the list
int shards_read(const gs_code *code, const int *erased, int n_erased, std::vector<int> &read);
// true when an output range [out[r], +bytes) shares a byte with an input range or another output
bool outputs_overlap(const void *const *in, int n_in, void *const *out, int n_out, size_t bytes);
// pointer / alignment / stripe / overlap checks of one encode or one rebuild (`read` from shards_read)
int check_encode_args(const gs_code *code, const void *const *data, void *const *parity, size_t shard_bytes);
int check_rebuild_args(const gs_code *code, void *const *shards, const std::vector<int> &read, const int *erased,
                       int n_erased, size_t shard_bytes);
// rebuild with a matrix from decode_matrix (any code but RDP): checks the pointers, then launches
int apply_rebuild(const gs_code *code, const std::vector<uint8_t> &R, const std::vector<int> &survivors,
                  void *const *shards, const int *erased, int n_erased, size_t shard_bytes, hipStream_t stream);
int decode_matrix(const gs_code *code, const int *erased, int n_erased, std::vector<uint8_t> &R,
                  std::vector<int> &survivors);

// A window of a paged KV pool: n_slots page slots per plane, their page ids at
// table[row * table_stride + slot].
struct PagedView {
    const void *const *plane_base;  // device array of n_planes device pointers
    int n_planes;
    size_t page_bytes;
    int64_t pages_per_plane;
    const int32_t *table;           // device; entry of row 0 at the window's first slot
    int table_stride;
    int n_slots;
};
int check_paged_geometry(const void *const *plane_base, int n_planes, size_t page_bytes, int64_t pages_per_plane,
                         const int32_t *table, int pages_per_shard, bool *empty);
int apply_matrix_paged(int rows, int cols, const uint8_t *C, const PagedView &v, const PagedStream *in,
                       const PagedStream *out, hipStream_t stream);
// the same two operations for any code kind (RDP included: a cell is a page)
int check_rdp_paged(const gs_code *code, size_t page_bytes, int n_slots);
int encode_paged_view(const gs_code *code, const PagedView &v, const PagedStream *parity_out, hipStream_t stream);
int rebuild_paged_view(const gs_code *code, const std::vector<uint8_t> &R, const std::vector<int> &surv, const PagedView &v,
                       const PagedStream *parity_in, const PagedStream *parity_out, const int *erased, int n_erased,
                       hipStream_t stream);
int rebuild_paged(const gs_code *code, const std::vector<uint8_t> &R, const std::vector<int> &surv, const PagedView &v,
                  const PagedStream *parity_in, const PagedStream *parity_out, const int *erased, int n_erased,
                  hipStream_t stream);

}  // namespace gs
