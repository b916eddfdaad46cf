// C ABI of the erasure-code library: argument checking, code construction,
// decode matrices, and the splitting of wide codes into kernel launches.
#include "../../include/ghostserve_ec.h"

#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <atomic>
#include <cstring>
#include <memory>
#include <new>
#include <vector>

#include "gs_gf.h"
#include "gs_internal.h"
#include "gs_launch.h"

namespace gs {

thread_local int g_last_hip_error = 0;

// Launch-shape knobs, defaults chosen by measurement on MI355X; see
// gs_set_launch_shape().  The four knobs live in one atomic word, so a launch
// that runs while another thread changes them sees either the old or the new
// set, never a mixture; every setting gives the same bytes.
static constexpr LaunchShape kDefaultShape = {0, 1, 1, 5, 1, 1};  // unroll 0: chosen per kernel family

static constexpr uint64_t pack_shape(const LaunchShape &s)
{
    return static_cast<uint64_t>(static_cast<uint8_t>(s.unroll)) | (static_cast<uint64_t>(static_cast<uint8_t>(s.nontemporal)) << 8) |
           (static_cast<uint64_t>(static_cast<uint8_t>(s.interleave_shift)) << 16) |
           (static_cast<uint64_t>(s.occupancy_cap ? 1u : 0u) << 24) | (static_cast<uint64_t>(static_cast<uint32_t>(s.size_forms) & 3u) << 25) |
           (static_cast<uint64_t>(static_cast<uint32_t>(s.tiles_per_wg)) << 32);
}

static std::atomic<uint64_t> g_shape{pack_shape(kDefaultShape)};

LaunchShape current_shape()
{
    const uint64_t w = g_shape.load(std::memory_order_relaxed);
    LaunchShape s;
    s.unroll = static_cast<int>(w & 0xFF);
    s.nontemporal = static_cast<int>((w >> 8) & 0xFF);
    s.interleave_shift = static_cast<int>((w >> 16) & 0xFF);
    s.occupancy_cap = static_cast<int>((w >> 24) & 1);
    s.size_forms = static_cast<int>((w >> 25) & 3);
    s.tiles_per_wg = static_cast<int>(w >> 32);
    return s;
}

// power-code encodes go through the Horner kernel unless switched off
static std::atomic<bool> g_power_horner{true};

int hip_status(hipError_t e)
{
    if (e == hipSuccess) return GS_OK;
    g_last_hip_error = static_cast<int>(e);
    return e == hipErrorOutOfMemory ? GS_ENOMEM : GS_EHIP;
}

int caught()
{
    try {
        throw;
    } catch (const std::bad_alloc &) {
        return GS_ENOMEM;
    } catch (...) {
        return GS_EINVAL;
    }
}

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// out[r] = XOR_j C[r][j] (x) in[j] for an arbitrary rows x cols matrix: row
// groups of up to 4, column groups of up to 16, later column groups accumulate.
int apply_matrix(int rows, int cols, const uint8_t *C, const void *const *in, void *const *out,
                 size_t bytes, hipStream_t stream)
{
    const LaunchShape shape = current_shape();
    for (int r0 = 0; r0 < rows; r0 += kLaunchMaxM) {
        const int nr = std::min(kLaunchMaxM, rows - r0);
        for (int c0 = 0; c0 < cols; c0 += kLaunchMaxK) {
            const int nc = std::min(kLaunchMaxK, cols - c0);
            const hipError_t e = launch_apply(nr, nc, C + static_cast<size_t>(r0) * cols + c0, cols,
                                              in + c0, out + r0, bytes, c0 != 0, shape, stream);
            if (e != hipSuccess) return hip_status(e);
        }
    }
    return GS_OK;
}

// paged form of apply_matrix: streams are table rows or dense buffers
int apply_matrix_paged(int rows, int cols, const uint8_t *C, const PagedView &v, const PagedStream *in,
                       const PagedStream *out, hipStream_t stream)
{
    const LaunchShape shape = current_shape();
    for (int r0 = 0; r0 < rows; r0 += kLaunchMaxM) {
        const int nr = std::min(kLaunchMaxM, rows - r0);
        for (int c0 = 0; c0 < cols; c0 += kLaunchMaxK) {
            const int nc = std::min(kLaunchMaxK, cols - c0);
            const hipError_t e = launch_apply_paged(nr, nc, C + static_cast<size_t>(r0) * cols + c0, cols, v.plane_base,
                                                    v.n_planes, v.page_bytes, v.pages_per_plane, v.table,
                                                    v.table_stride, v.n_slots, in + c0, out + r0, c0 != 0, shape, stream);
            if (e != hipSuccess) return hip_status(e);
        }
    }
    return GS_OK;
}

// Geometry checks shared by the paged entry points.  GS_OK with *empty set
// means there is nothing to do.
int check_paged_geometry(const void *const *plane_base, int n_planes, size_t page_bytes, int64_t pages_per_plane,
                         const int32_t *table, int pages_per_shard, bool *empty)
{
    *empty = false;
    if (plane_base == nullptr || table == nullptr) return GS_EINVAL;
    if (n_planes < 0 || n_planes > 65535 || pages_per_shard < 0 || pages_per_plane < 0) return GS_EINVAL;
    if (page_bytes == 0 || page_bytes % 16 != 0) return GS_EINVAL;
    if ((page_bytes / 16) * static_cast<uint64_t>(pages_per_shard) >= (1ull << 32)) return GS_EINVAL;
    if (n_planes == 0 || pages_per_shard == 0) {
        *empty = true;
        return GS_OK;
    }
    return pages_per_plane == 0 ? GS_EINVAL : GS_OK;
}

// Rebuild over a paged view with a matrix from decode_matrix: surviving data
// shards are gathered from their pages, surviving parity comes from
// parity_in[i] (dense), a lost data shard is scattered into the pages of its
// table row, a lost parity shard goes to parity_out[i] (dense).
int rebuild_paged(const gs_code *code, const std::vector<uint8_t> &R, const std::vector<int> &surv, const PagedView &v,
                  const PagedStream *parity_in, const PagedStream *parity_out, const int *erased, int n_erased,
                  hipStream_t stream)
{
    const int k = code->k;
    std::vector<PagedStream> in(k), out(n_erased);
    for (int j = 0; j < k; ++j) {
        if (surv[j] < k) {
            in[j] = PagedStream{surv[j], nullptr};
        } else {
            in[j] = parity_in[surv[j] - k];
            if (in[j].dense == nullptr || !aligned16(in[j].dense)) return GS_EINVAL;
            in[j].table_row = -1;
        }
    }
    for (int x = 0; x < n_erased; ++x) {
        if (erased[x] < k) {
            out[x] = PagedStream{erased[x], nullptr};
        } else {
            out[x] = parity_out[erased[x] - k];
            if (out[x].dense == nullptr || !aligned16(out[x].dense)) return GS_EINVAL;
            out[x].table_row = -1;
        }
    }
    return apply_matrix_paged(n_erased, k, R.data(), v, in.data(), out.data(), stream);
}

// RDP over a paged pool: a cell is a page, a stripe p-1 consecutive slots of a plane
int check_rdp_paged(const gs_code *code, size_t page_bytes, int n_slots)
{
    if (page_bytes != code->rdp_cell || page_bytes < 1024) return GS_EINVAL;
    if (n_slots % (code->rdp_encode.p - 1) != 0) return GS_EINVAL;
    // one launch covers 16 GiB per stripe row of a plane (p = 3: 32 GiB of a shard per plane)
    if (static_cast<uint64_t>(n_slots) / (code->rdp_encode.p - 1) * page_bytes >= (16ull << 30)) return GS_EINVAL;
    return GS_OK;
}

static int rdp_paged(const gs_code *code, const RdpPlan &plan, const PagedView &v, const PagedStream *parity_in,
                     const PagedStream *parity_out, hipStream_t stream)
{
    const int k = code->k;
    PagedStream shards[kRdpMaxDisks];
    for (int j = 0; j < k; ++j) shards[j] = PagedStream{j, nullptr};
    for (int i = 0; i < 2; ++i) {
        bool produced = false;
        for (int s : plan.outputs) produced = produced || s == k + i;
        shards[k + i] = produced ? parity_out[i] : parity_in[i];
        shards[k + i].table_row = -1;
    }
    // every dense buffer the plan touches must be there
    for (int j = 0; j <= plan.p; ++j) {
        const int s = plan.shard_of_disk[j];
        if (s >= k && (shards[s].dense == nullptr || !aligned16(shards[s].dense))) return GS_EINVAL;
    }
    for (int s : plan.outputs)
        if (s >= k && (shards[s].dense == nullptr || !aligned16(shards[s].dense))) return GS_EINVAL;
    return hip_status(launch_rdp_paged(plan, v.plane_base, v.n_planes, v.page_bytes, v.pages_per_plane, v.table,
                                       v.table_stride, v.n_slots, shards, current_shape(), stream));
}

// Encode over a paged view, any code kind: data shards are table rows 0..k-1,
// parity goes to the dense streams parity_out[0..m).
int encode_paged_view(const gs_code *code, const PagedView &v, const PagedStream *parity_out, hipStream_t stream)
{
    for (int i = 0; i < code->m; ++i)
        if (parity_out[i].dense == nullptr || !aligned16(parity_out[i].dense)) return GS_EINVAL;
    if (code->is_rdp()) {
        const int rc = check_rdp_paged(code, v.page_bytes, v.n_slots);
        if (rc != GS_OK) return rc;
        return rdp_paged(code, code->rdp_encode, v, parity_out, parity_out, stream);
    }
    std::vector<PagedStream> in(code->k);
    for (int j = 0; j < code->k; ++j) in[j] = PagedStream{j, nullptr};
    return apply_matrix_paged(code->m, code->k, code->P.data(), v, in.data(), parity_out, stream);
}

// Rebuild over a paged view, any code kind.  R and surv come from decode_matrix
// (unused for RDP, whose plan is made here).
int rebuild_paged_view(const gs_code *code, const std::vector<uint8_t> &R, const std::vector<int> &surv, const PagedView &v,
                       const PagedStream *parity_in, const PagedStream *parity_out, const int *erased, int n_erased,
                       hipStream_t stream)
{
    if (!code->is_rdp()) return rebuild_paged(code, R, surv, v, parity_in, parity_out, erased, n_erased, stream);
    const int rc = check_rdp_paged(code, v.page_bytes, v.n_slots);
    if (rc != GS_OK) return rc;
    RdpPlan plan;
    if (!rdp_plan(code->k, erased, n_erased, plan)) return GS_ESINGULAR;
    return rdp_paged(code, plan, v, parity_in, parity_out, stream);
}

int check_erasures(const gs_code *code, const int *erased, int n_erased, std::vector<uint8_t> &lost)
{
    const int n = code->k + code->m;
    lost.assign(n, 0);
    if (n_erased < 0 || (n_erased > 0 && erased == nullptr)) return GS_EINVAL;
    for (int x = 0; x < n_erased; ++x) {
        if (erased[x] < 0 || erased[x] >= n || lost[erased[x]]) return GS_EINVAL;
        lost[erased[x]] = 1;
    }
    return n_erased > code->m ? GS_ETOOMANY : GS_OK;
}

int decode_matrix(const gs_code *code, const int *erased, int n_erased, std::vector<uint8_t> &R,
                  std::vector<int> &survivors)
{
    const int k = code->k;
    std::vector<uint8_t> lost;
    const int rc = check_erasures(code, erased, n_erased, lost);
    if (rc != GS_OK) return rc;
    survivors.clear();
    for (int r = 0; r < k + code->m && static_cast<int>(survivors.size()) < k; ++r)
        if (!lost[r]) survivors.push_back(r);
    // A = the survivors' rows of [I ; P]
    Matrix A(static_cast<size_t>(k) * k, 0);
    for (int r = 0; r < k; ++r) {
        const int s = survivors[r];
        if (s < k) A[r * k + s] = 1;
        else std::memcpy(&A[r * k], &code->P[static_cast<size_t>(s - k) * k], k);
    }
    if (!invert_in_place(k, A)) return GS_ESINGULAR;
    R.assign(static_cast<size_t>(n_erased) * k, 0);
    for (int x = 0; x < n_erased; ++x) {
        const int r = erased[x];
        if (r < k) {
            std::memcpy(&R[static_cast<size_t>(x) * k], &A[static_cast<size_t>(r) * k], k);
        } else {
            const uint8_t *prow = &code->P[static_cast<size_t>(r - k) * k];
            for (int c = 0; c < k; ++c) {
                uint8_t s = 0;
                for (int t = 0; t < k; ++t) s ^= gf_mul(prow[t], A[t * k + c]);
                R[static_cast<size_t>(x) * k + c] = s;
            }
        }
    }
    return GS_OK;
}

int shards_read(const gs_code *code, const int *erased, int n_erased, std::vector<int> &read)
{
    read.clear();
    if (code->is_rdp()) {
        std::vector<uint8_t> lost;
        const int rc = check_erasures(code, erased, n_erased, lost);
        if (rc != GS_OK || n_erased == 0) return rc;
        RdpPlan plan;
        if (!rdp_plan(code->k, erased, n_erased, plan)) return GS_ESINGULAR;
        for (int j = 0; j <= plan.p; ++j)
            if (plan.shard_of_disk[j] >= 0) read.push_back(plan.shard_of_disk[j]);
        return GS_OK;
    }
    std::vector<uint8_t> R;
    return decode_matrix(code, erased, n_erased, R, read);
}

// true when the byte ranges [a, a+n) and [b, b+n) share a byte
static bool ranges_meet(const void *a, const void *b, size_t n)
{
    const uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b);
    return x < y ? y - x < n : x - y < n;
}

// An output buffer of a call may overlap neither an input nor another output:
// the kernels read and write tile by tile in no fixed order.
bool outputs_overlap(const void *const *in, int n_in, void *const *out, int n_out, size_t bytes)
{
    for (int r = 0; r < n_out; ++r) {
        for (int j = 0; j < n_in; ++j)
            if (ranges_meet(out[r], in[j], bytes)) return true;
        for (int q = 0; q < r; ++q)
            if (ranges_meet(out[r], out[q], bytes)) return true;
    }
    return false;
}

int check_encode_args(const gs_code *code, const void *const *data, void *const *parity, size_t shard_bytes)
{
    if (shard_bytes == 0) return GS_OK;
    for (int j = 0; j < code->k; ++j)
        if (data[j] == nullptr || !aligned16(data[j])) return GS_EINVAL;
    for (int i = 0; i < code->m; ++i)
        if (parity[i] == nullptr || !aligned16(parity[i])) return GS_EINVAL;
    if (code->is_rdp() && shard_bytes % (code->rdp_cell * (code->rdp_encode.p - 1)) != 0) return GS_EINVAL;
    if (outputs_overlap(data, code->k, parity, code->m, shard_bytes)) return GS_EINVAL;
    return GS_OK;
}

int check_rebuild_args(const gs_code *code, void *const *shards, const std::vector<int> &read, const int *erased,
                       int n_erased, size_t shard_bytes)
{
    if (n_erased == 0 || shard_bytes == 0) return GS_OK;
    for (int s : read)
        if (shards[s] == nullptr || !aligned16(shards[s])) return GS_EINVAL;
    for (int x = 0; x < n_erased; ++x)
        if (shards[erased[x]] == nullptr || !aligned16(shards[erased[x]])) return GS_EINVAL;
    if (code->is_rdp() && shard_bytes % (code->rdp_cell * (code->rdp_encode.p - 1)) != 0) return GS_EINVAL;
    const void *in[256];  // k + m <= 256
    void *out[256];
    int n_in = 0;
    for (int s : read) in[n_in++] = shards[s];
    for (int x = 0; x < n_erased; ++x) out[x] = shards[erased[x]];
    if (outputs_overlap(in, n_in, out, n_erased, shard_bytes)) return GS_EINVAL;
    return GS_OK;
}

// the launches of a rebuild whose matrix is already known (not RDP)
int apply_rebuild(const gs_code *code, const std::vector<uint8_t> &R, const std::vector<int> &survivors,
                  void *const *shards, const int *erased, int n_erased, size_t shard_bytes, hipStream_t stream)
{
    if (n_erased == 0 || shard_bytes == 0) return GS_OK;
    const int rc = check_rebuild_args(code, shards, survivors, erased, n_erased, shard_bytes);
    if (rc != GS_OK) return rc;
    std::vector<const void *> in(code->k);
    std::vector<void *> out(n_erased);
    for (int j = 0; j < code->k; ++j) in[j] = shards[survivors[j]];
    for (int x = 0; x < n_erased; ++x) out[x] = shards[erased[x]];
    return apply_matrix(n_erased, code->k, R.data(), in.data(), out.data(), shard_bytes, stream);
}

static int rdp_reconstruct(const gs_code *code, void *const *shards, const int *erased, int n_erased,
                           size_t shard_bytes, hipStream_t stream)
{
    std::vector<uint8_t> lost;
    const int rc = check_erasures(code, erased, n_erased, lost);
    if (rc != GS_OK) return rc;
    if (n_erased == 0 || shard_bytes == 0) return GS_OK;
    if (shard_bytes % (code->rdp_cell * (code->rdp_encode.p - 1)) != 0) return GS_EINVAL;
    RdpPlan plan;
    if (!rdp_plan(code->k, erased, n_erased, plan)) return GS_ESINGULAR;
    for (int j = 0; j <= plan.p; ++j) {
        const int s = plan.shard_of_disk[j];
        if (s >= 0 && (shards[s] == nullptr || !aligned16(shards[s]))) return GS_EINVAL;
    }
    const void *in[kRdpMaxDisks];
    void *out[2];
    int n_in = 0, n_out = 0;
    for (int j = 0; j <= plan.p; ++j)
        if (plan.shard_of_disk[j] >= 0) in[n_in++] = shards[plan.shard_of_disk[j]];
    for (int s : plan.outputs) {
        if (shards[s] == nullptr || !aligned16(shards[s])) return GS_EINVAL;
        out[n_out++] = shards[s];
    }
    if (outputs_overlap(in, n_in, out, n_out, shard_bytes)) return GS_EINVAL;
    return hip_status(launch_rdp(plan, shards, shard_bytes, code->rdp_cell, current_shape(), stream));
}

}  // namespace gs

using namespace gs;

extern "C" {

int gs_make_code(int k, int m, int kind, gs_code **out)
try {
    if (out == nullptr) return GS_EINVAL;
    *out = nullptr;
    if (k < 1 || m < 1 || k + m > 256) return GS_EINVAL;
    if (kind != GS_CAUCHY && kind != GS_VANDERMONDE && kind != GS_RDP && kind != GS_POWER) return GS_EINVAL;
    if (kind == GS_RDP && (m != 2 || k > kRdpMaxPrime - 1)) return GS_EINVAL;
    if (kind == GS_POWER && m > 3) return GS_EINVAL;  // beyond that the power matrix is not MDS
    std::unique_ptr<gs_code> c(new gs_code);
    c->k = k;
    c->m = m;
    c->kind = kind;
    if (kind == GS_RDP) {
        const int parity_ids[2] = {k, k + 1};
        rdp_plan(k, parity_ids, 2, c->rdp_encode);
        c->rdp_cell = GS_RDP_DEFAULT_CELL;
    }
    else if (kind == GS_POWER) c->P = power_parity_block(k, m);
    else c->P = kind == GS_CAUCHY ? cauchy_parity_block(k, m) : vandermonde_parity_block(k, m);
    *out = c.release();
    return GS_OK;
}
catch (...) {
    return caught();
}

void gs_free_code(gs_code *code) { delete code; }

int gs_code_params(const gs_code *code, int *k, int *m)
{
    if (code == nullptr) return GS_EINVAL;
    if (k) *k = code->k;
    if (m) *m = code->m;
    return GS_OK;
}

int gs_make_rdp_code(int k, size_t cell_bytes, gs_code **out)
try {
    if (out == nullptr) return GS_EINVAL;
    *out = nullptr;
    if (cell_bytes < 16 || (cell_bytes & (cell_bytes - 1)) != 0) return GS_EINVAL;
    const int rc = gs_make_code(k, 2, GS_RDP, out);
    if (rc == GS_OK) (*out)->rdp_cell = cell_bytes;
    return rc;
}
catch (...) {
    return caught();
}

int gs_rdp_cell_bytes(const gs_code *code, size_t *cell_out)
{
    if (code == nullptr || cell_out == nullptr || !code->is_rdp()) return GS_EINVAL;
    *cell_out = code->rdp_cell;
    return GS_OK;
}

int gs_rdp_prime(const gs_code *code, int *p_out)
{
    if (code == nullptr || p_out == nullptr || !code->is_rdp()) return GS_EINVAL;
    *p_out = code->rdp_encode.p;
    return GS_OK;
}

int gs_rdp_plan(const gs_code *code, const int *missing, int n_missing, int *read_out, int *n_read_out,
                uint32_t *syndrome_mask_out)
try {
    if (code == nullptr || !code->is_rdp() || read_out == nullptr || n_read_out == nullptr ||
        syndrome_mask_out == nullptr)
        return GS_EINVAL;
    RdpPlan plan;
    if (n_missing == 0) {
        plan = code->rdp_encode;
    } else {
        std::vector<uint8_t> lost;
        const int rc = check_erasures(code, missing, n_missing, lost);
        if (rc != GS_OK) return rc;
        if (!rdp_plan(code->k, missing, n_missing, plan)) return GS_ESINGULAR;
    }
    int n = 0;
    for (int j = 0; j <= plan.p; ++j)
        if (plan.shard_of_disk[j] >= 0) read_out[n++] = plan.shard_of_disk[j];
    *n_read_out = n;
    std::copy(plan.syndrome_mask.begin(), plan.syndrome_mask.end(), syndrome_mask_out);
    return GS_OK;
}
catch (...) {
    return caught();
}

int gs_code_matrix(const gs_code *code, uint8_t *P_out)
{
    if (code == nullptr || P_out == nullptr || code->is_rdp()) return GS_EINVAL;
    std::memcpy(P_out, code->P.data(), code->P.size());
    return GS_OK;
}

int gs_decode_matrix(const gs_code *code, const int *erased, int n_erased, uint8_t *R_out,
                     int *survivors_out)
try {
    if (code == nullptr || code->is_rdp()) return GS_EINVAL;
    std::vector<uint8_t> R;
    std::vector<int> surv;
    const int rc = decode_matrix(code, erased, n_erased, R, surv);
    if (rc != GS_OK) return rc;
    if (R_out && !R.empty()) std::memcpy(R_out, R.data(), R.size());
    if (survivors_out) std::copy(surv.begin(), surv.end(), survivors_out);
    return GS_OK;
}
catch (...) {
    return caught();
}

int gs_encode(const gs_code *code, const void *const *data, void *const *parity, size_t shard_bytes,
              void *stream)
try {
    if (code == nullptr || data == nullptr || parity == nullptr) return GS_EINVAL;
    if (shard_bytes == 0) return GS_OK;
    const int rc = check_encode_args(code, data, parity, shard_bytes);
    if (rc != GS_OK) return rc;
    if (code->is_rdp()) {
        std::vector<const void *> shards(data, data + code->k);
        shards.push_back(parity[0]);
        shards.push_back(parity[1]);
        return hip_status(launch_rdp(code->rdp_encode, shards.data(), shard_bytes, code->rdp_cell, current_shape(),
                                         static_cast<hipStream_t>(stream)));
    }
    if (code->kind == GS_POWER && g_power_horner.load(std::memory_order_relaxed) && code->m >= 2 && code->k <= kLaunchMaxK)
        return hip_status(launch_horner(code->m, code->k, code->P.data(), code->k, data, parity, shard_bytes,
                                        current_shape(), static_cast<hipStream_t>(stream)));
    return apply_matrix(code->m, code->k, code->P.data(), data, parity, shard_bytes,
                        static_cast<hipStream_t>(stream));
}
catch (...) {
    return caught();
}

int gs_encode_paged(const gs_code *code, const void *const *plane_base, int n_planes, size_t page_bytes,
                    int64_t pages_per_plane, const int32_t *table, int pages_per_shard,
                    void *const *parity, void *stream)
try {
    if (code == nullptr || parity == nullptr) return GS_EINVAL;
    bool empty;
    const int rc = check_paged_geometry(plane_base, n_planes, page_bytes, pages_per_plane, table, pages_per_shard, &empty);
    if (rc != GS_OK || empty) return rc;
    std::vector<PagedStream> out(code->m);
    for (int i = 0; i < code->m; ++i) out[i] = PagedStream{-1, parity[i]};
    const PagedView v{plane_base, n_planes, page_bytes, pages_per_plane, table, pages_per_shard, pages_per_shard};
    return encode_paged_view(code, v, out.data(), static_cast<hipStream_t>(stream));
}
catch (...) {
    return caught();
}

int gs_reconstruct_paged(const gs_code *code, const void *const *plane_base, int n_planes, size_t page_bytes,
                         int64_t pages_per_plane, const int32_t *table, int pages_per_shard,
                         void *const *parity, const int *erased, int n_erased, void *stream)
try {
    if (code == nullptr || parity == nullptr) return GS_EINVAL;
    bool empty;
    const int rc0 = check_paged_geometry(plane_base, n_planes, page_bytes, pages_per_plane, table, pages_per_shard, &empty);
    if (rc0 != GS_OK) return rc0;
    std::vector<uint8_t> R;
    std::vector<int> surv;
    const int rc = code->is_rdp() ? shards_read(code, erased, n_erased, surv) : decode_matrix(code, erased, n_erased, R, surv);
    if (rc != GS_OK) return rc;
    if (n_erased == 0 || empty) return GS_OK;
    std::vector<PagedStream> dense(code->m);
    for (int i = 0; i < code->m; ++i) dense[i] = PagedStream{-1, parity[i]};
    const PagedView v{plane_base, n_planes, page_bytes, pages_per_plane, table, pages_per_shard, pages_per_shard};
    return rebuild_paged_view(code, R, surv, v, dense.data(), dense.data(), erased, n_erased, static_cast<hipStream_t>(stream));
}
catch (...) {
    return caught();
}

int gs_reconstruct(const gs_code *code, void *const *shards, const int *erased, int n_erased,
                   size_t shard_bytes, void *stream)
try {
    if (code == nullptr || shards == nullptr) return GS_EINVAL;
    if (code->is_rdp()) return rdp_reconstruct(code, shards, erased, n_erased, shard_bytes, static_cast<hipStream_t>(stream));
    std::vector<uint8_t> R;
    std::vector<int> surv;
    const int rc = decode_matrix(code, erased, n_erased, R, surv);
    if (rc != GS_OK) return rc;
    return apply_rebuild(code, R, surv, shards, erased, n_erased, shard_bytes, static_cast<hipStream_t>(stream));
}
catch (...) {
    return caught();
}

const char *gs_strerror(int status)
{
    switch (status) {
        case GS_OK: return "ok";
        case GS_EINVAL: return "invalid argument";
        case GS_ENOMEM: return "out of memory";
        case GS_ETOOMANY: return "more erasures than parity shards";
        case GS_ESINGULAR: return "survivor matrix is singular";
        case GS_EHIP: return "HIP runtime error";
        case GS_ELIMIT: return "beyond the fixed capacity of an entry point that allocates nothing";
        default: return "unknown status";
    }
}

int gs_last_hip_error(void) { return g_last_hip_error; }

int gs_coef_words(int c, uint32_t *words_out)
{
    if (c < 0 || c > 255 || words_out == nullptr) return GS_EINVAL;
    const CoefWords w = split_tables(static_cast<uint8_t>(c));
    for (int i = 0; i < 5; ++i) words_out[i] = w.w[i];
    return GS_OK;
}

int gs_set_launch_shape(int unroll, int tiles_per_wg, int nontemporal, int interleave_shift)
{
    LaunchShape s = kDefaultShape;
    if (unroll > 0) {
        if (unroll != 1 && unroll != 2 && unroll != 4) return GS_EINVAL;
        s.unroll = unroll;
    }
    if (tiles_per_wg > 0) s.tiles_per_wg = tiles_per_wg;  // any positive int fits the packed word
    if (nontemporal >= 0) s.nontemporal = nontemporal ? 1 : 0;
    if (interleave_shift >= 0) {
        if (interleave_shift > 10) return GS_EINVAL;
        s.interleave_shift = interleave_shift;
    }
    // the occupancy and kernel-form switches are knobs of their own: keep what they say
    uint64_t old = g_shape.load(std::memory_order_relaxed), next;
    do {
        s.occupancy_cap = static_cast<int>((old >> 24) & 1);
        s.size_forms = static_cast<int>((old >> 25) & 3);
        next = pack_shape(s);
    } while (!g_shape.compare_exchange_weak(old, next, std::memory_order_relaxed));
    return GS_OK;
}

int gs_set_occupancy_cap(int enable)
{
    uint64_t old = g_shape.load(std::memory_order_relaxed), next;
    do {
        next = enable ? (old | (1ull << 24)) : (old & ~(1ull << 24));
    } while (!g_shape.compare_exchange_weak(old, next, std::memory_order_relaxed));
    return GS_OK;
}

int gs_set_size_forms(int mode)
{
    if (mode < 0 || mode > 2) return GS_EINVAL;
    uint64_t old = g_shape.load(std::memory_order_relaxed), next;
    do {
        next = (old & ~(3ull << 25)) | (static_cast<uint64_t>(mode) << 25);
    } while (!g_shape.compare_exchange_weak(old, next, std::memory_order_relaxed));
    return GS_OK;
}

int gs_set_power_horner(int enable)
{
    g_power_horner.store(enable != 0, std::memory_order_relaxed);
    return GS_OK;
}

}  // extern "C"
