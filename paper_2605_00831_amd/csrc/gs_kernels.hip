// HIP kernels for gfx950: apply a small GF(2^8) matrix to k byte streams.
//
//   out[r][t] = XOR_j  C[r][j] (x) in[j][t]          r < rows <= 4, j < k <= 16
//
// Encode uses C = the code's parity block (Alg. 1, EC.encode); reconstruct
// uses C = the rebuild matrix of the erasure pattern (Alg. 2, EC.reconstruct).
// The KV cache is consumed as raw bytes (Section 4.1: reversible integer view
// of FP16), so there is no conversion pass before or after.
//
// Shape of the computation on CDNA4:
//   * the path is HBM-bound, so every lane moves 16-byte vectors with
//     consecutive lanes on consecutive addresses (1 KiB per wavefront per
//     load); a tile is 256 lanes x U vectors per stream;
//   * the 1 KiB pieces of a shard are dealt to workgroups with an interleave
//     that keeps every XCD on one residue class of pieces (see "Work
//     distribution" below) -- worth 8-10 points of HBM peak on MI355X;
//   * the streams are taken one at a time (load a stream's piece, fold it into
//     the accumulators), and bulk launches limit the workgroups per CU to 3
//     or 4 through an LDS reservation: many wavefronts with one short burst of
//     loads each serve the memory better than fewer with long bursts;
//   * multiplication by a constant is linear over GF(2), so it is evaluated
//     as three byte-table lookups on the bit fields [2:0], [5:3], [7:6] of
//     each byte, four bytes at a time with v_perm_b32 (an 8-byte table fits
//     the instruction's two source registers); the tables arrive as kernel
//     arguments and are read with scalar loads;
//   * a matrix row of all ones (row 0 of the parity block; the one-parity
//     code) is a plain XOR and skips the lookups;
//   * the power code P[r][j] = 2^(r*j) has a second encode kernel that
//     evaluates its rows by Horner's rule with a packed multiply-by-2 and no
//     tables (fewer vector instructions; HBM-bound like the table kernel).
#include <hip/hip_runtime.h>
#include "gs_gf.h"
#include "gs_launch.h"

namespace gs {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct ApplyArgs {
    const uint8_t *in[kLaunchMaxK];
    uint8_t *out[kLaunchMaxM];
    uint32_t tab[kLaunchMaxM][kLaunchMaxK][8];  // 5 words used per coefficient
    uint64_t nvec;        // whole 16-byte vectors per stream
    uint32_t tail;        // trailing bytes after the last whole vector (0..15)
    int32_t k;            // streams in this launch
    int32_t accumulate;   // XOR into the existing outputs
    uint32_t tiles_per_wg;
    uint32_t nx_shift;    // log2 of the interleave modulus (0 = plain consecutive tiles)
    // Kernels with an XOR row: that row takes streams [0, n_xor) only, and before the stores the
    // accumulators of the rows in `fold` (bit r = row r, r >= 1) are XORed into it.  An encode has
    // n_xor = k and fold = 0; a rebuild whose matrix has a row that differs from the XOR of some of
    // its other rows only by zeros and ones (see plan_fold) runs with the XOR shortcut this way.
    int32_t n_xor;
    uint32_t fold;
};

static_assert(sizeof(BatchDesc) == kBatchDescBytes, "descriptor size is part of the internal interface");

struct BatchArgs {
    const BatchDesc *descs;  // device array, one per blockIdx.y
    uint32_t tab[kLaunchMaxM][kLaunchMaxK][8];
    int32_t k;
};

struct PagedArgs {
    const uint8_t *const *plane_base;  // device array [n_planes]
    const int32_t *table;              // device [shards][pps]
    // every stream is either paged (table row >= 0) or contiguous in the dense
    // parity layout [plane][slot][page] (row < 0, pointer used)
    const uint8_t *in_ptr[kLaunchMaxK];
    int32_t in_row[kLaunchMaxK];
    uint32_t in_stride[kLaunchMaxK];   // dense streams: 16-byte vectors from one plane to the next
    uint8_t *out[kLaunchMaxM];
    int32_t out_row[kLaunchMaxM];
    uint32_t out_stride[kLaunchMaxM];
    uint32_t tab[kLaunchMaxM][kLaunchMaxK][8];
    uint64_t vecs_per_plane;   // slots * vpp, < 2^32
    uint64_t pages_per_plane;  // valid page ids are [0, pages_per_plane)
    uint32_t vpp;              // 16-byte vectors per page
    int32_t vpp_shift;         // log2(vpp) if a power of two, else -1
    uint32_t table_stride;     // entries from one table row to the next (>= slots of this launch)
    int32_t k;
    int32_t accumulate;
    uint32_t tiles_per_wg;
    uint32_t nx_shift;         // log2 of the piece interleave modulus
    uint32_t mixed;            // 0: inputs are consecutive table rows, outputs dense
    uint32_t small_form;       // host side only: a launch that does not fill the chip may take its own kernel form
};

template <bool NT>
__device__ __forceinline__ u32x4 load16(const uint8_t *base, uint64_t vec)
{
    const u32x4 *p = reinterpret_cast<const u32x4 *>(base) + vec;

    if (NT) return __builtin_nontemporal_load(p);
    return *p;
}

template <bool NT>
__device__ __forceinline__ void store16(uint8_t *base, uint64_t vec, u32x4 v)
{
    u32x4 *p = reinterpret_cast<u32x4 *>(base) + vec;
    if (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// The same two accesses for a 1 KiB piece: `piece` (first vector of the piece)
// is the same for every lane of the wavefront, so base + piece is scalar
// arithmetic and the only per-lane part of the address is the 32-bit lane
// offset -- the scalar-base + vector-offset form of the memory instructions,
// which needs no 64-bit address arithmetic and no address registers per stream.
template <bool NT>
__device__ __forceinline__ u32x4 load_piece(const uint8_t *base, uint64_t piece, uint32_t lane)
{
    const u32x4 *p = reinterpret_cast<const u32x4 *>(base) + piece;
    if (NT) return __builtin_nontemporal_load(p + lane);
    return p[lane];
}

template <bool NT>
__device__ __forceinline__ void store_piece(uint8_t *base, uint64_t piece, uint32_t lane, u32x4 v)
{
    u32x4 *p = reinterpret_cast<u32x4 *>(base) + piece;
    if (NT) __builtin_nontemporal_store(v, p + lane);
    else p[lane] = v;
}

// c (x) each of the four bytes of d, given the five table words of c.
// v_perm_b32 picks, per selector byte s in 0..7, byte s of the 64-bit value
// {first operand : second operand}.
__device__ __forceinline__ uint32_t mul4(const uint32_t *t, uint32_t s0, uint32_t s1, uint32_t s2)
{
    return __builtin_amdgcn_perm(t[1], t[0], s0) ^ __builtin_amdgcn_perm(t[3], t[2], s1) ^
           __builtin_amdgcn_perm(t[4], t[4], s2);
}

// same product for a single byte, without the permute instruction
__device__ __forceinline__ uint32_t mul1(const uint32_t *t, uint32_t x)
{
    const uint64_t t0 = (static_cast<uint64_t>(t[1]) << 32) | t[0];
    const uint64_t t1 = (static_cast<uint64_t>(t[3]) << 32) | t[2];
    return static_cast<uint32_t>((t0 >> (8 * (x & 7))) ^ (t1 >> (8 * ((x >> 3) & 7))) ^
                                 (t[4] >> (8 * (x >> 6)))) & 0xFFu;
}

// The accumulators are plain dwords.  pin() is an empty asm that makes the
// compiler materialise the value at that point: without it the XOR chains of
// all streams are reassociated into one wide tree whose leaves (every lookup
// result of a tile) are alive at once, which costs hundreds of registers.
__device__ __forceinline__ void pin(uint32_t &v) { asm volatile("" : "+v"(v)); }

struct Acc4 { uint32_t c[4]; };

__device__ __forceinline__ u32x4 to_vec(const Acc4 &a) { return u32x4{a.c[0], a.c[1], a.c[2], a.c[3]}; }
__device__ __forceinline__ Acc4 from_vec(u32x4 v) { return Acc4{{v[0], v[1], v[2], v[3]}}; }

// acc[r][u] ^= C[r][j] (x) x[u] for all rows
// (SKIP0: the stream is not part of the XOR row)
template <int M, bool ROW0_XOR, int U, bool SKIP0 = false>
__device__ __forceinline__ void mac(Acc4 (&acc)[M][U], const u32x4 (&x)[U],
                                    const uint32_t (&tab)[kLaunchMaxM][kLaunchMaxK][8], int j)
{
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint32_t d = x[u][c];
            if (ROW0_XOR && !SKIP0) {
                acc[0][u].c[c] ^= d;
                pin(acc[0][u].c[c]);
            }
            if (M > (ROW0_XOR ? 1 : 0)) {
                const uint32_t s0 = d & 0x07070707u;
                const uint32_t s1 = (d >> 3) & 0x07070707u;
                const uint32_t s2 = (d >> 6) & 0x03030303u;
#pragma unroll
                for (int r = (ROW0_XOR ? 1 : 0); r < M; ++r) {
                    acc[r][u].c[c] ^= mul4(tab[r][j], s0, s1, s2);
                    pin(acc[r][u].c[c]);
                }
            }
        }
    }
}

// 2 (x) each of the four bytes of x: shift left inside every byte and fold the
// bit shifted out of a byte back in as the field polynomial's low part, 0x1D.
__device__ __forceinline__ uint32_t times2(uint32_t x)
{
    const uint32_t hi = x & 0x80808080u;
    return ((x ^ hi) << 1) ^ ((hi >> 7) * 0x1Du);
}

// One Horner step of the power code P[r][j] = 2^(r*j), streams taken from the
// last to the first: acc[r] = 2^r (x) acc[r] ^ x.  No tables, and the work per
// row does not depend on the coefficients.
template <int M, int U>
__device__ __forceinline__ void horner_step(Acc4 (&acc)[M][U], const u32x4 (&x)[U])
{
    static_assert(M >= 2 && M <= 3, "power code rows");
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint32_t d = x[u][c];
            acc[0][u].c[c] ^= d;
            pin(acc[0][u].c[c]);
            acc[1][u].c[c] = times2(acc[1][u].c[c]) ^ d;
            pin(acc[1][u].c[c]);
            if (M > 2) {
                acc[2][u].c[c] = times2(times2(acc[2][u].c[c])) ^ d;
                pin(acc[2][u].c[c]);
            }
        }
    }
}

// One tile over contiguous streams: each lane handles the U vectors v[0..U).
// FULL tiles (every lane in range) carry no predication at all; only tiles
// that reach past the end of the shard take the predicated form.
// S names where the stream pointers and the length live: the kernel arguments
// (ApplyArgs) or a per-chunk descriptor in device memory (BatchDesc).
// HORNER: the matrix is the power code's and is evaluated by horner_step over
// the streams in descending order instead of through the tables.
// KB: how many streams' loads are issued together before their arithmetic.
template <int M, bool ROW0_XOR, int U, bool NT, bool FULL, bool HORNER, int KB, class S>
__device__ __forceinline__ void contig_tile(const S &s, const uint32_t (&tab)[kLaunchMaxM][kLaunchMaxK][8],
                                            int k, int accumulate, int n_xor, uint32_t fold,
                                            const uint64_t (&piece)[U], uint32_t lane)
{
    // piece[u]: first vector of this wavefront's u-th piece (wavefront-uniform)
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) ok[u] = FULL || piece[u] + lane < s.nvec;

    Acc4 acc[M][U];
#pragma unroll
    for (int r = 0; r < M; ++r)
#pragma unroll
        for (int u = 0; u < U; ++u) acc[r][u] = Acc4{{0, 0, 0, 0}};
    if (accumulate) {
#pragma unroll
        for (int r = 0; r < M; ++r)
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (ok[u]) acc[r][u] = from_vec(load_piece<NT>(s.out[r], piece[u], lane));
    }

    // KB = 1, one stream at a time, is the bulk form: a wavefront has the U loads of one stream in
    // flight, does that stream's arithmetic, and goes on to the next stream.  Overlap comes from the
    // other wavefronts of the CU (12 to 16 of them, see the LDS reservation of the launchers).
    // Issuing the loads of two or four streams together, which looks like the obvious way to keep
    // more bytes in flight, is 1 to 5 points of HBM peak slower for every code shape once the chip is
    // full.  A launch that does not fill the chip is the other way round: its time is the k memory
    // round trips of a wavefront one after the other, and KB = 4 makes them k/4.
    int j = 0;
    if constexpr (KB > 1) {
        for (; j + KB <= k; j += KB) {
            u32x4 x[KB][U];
#pragma unroll
            for (int b = 0; b < KB; ++b) {
                const uint8_t *src = s.in[HORNER ? k - 1 - (j + b) : j + b];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    x[b][u] = u32x4{0, 0, 0, 0};
                    if (ok[u]) x[b][u] = load_piece<NT>(src, piece[u], lane);
                }
            }
#pragma unroll
            for (int b = 0; b < KB; ++b) {
                if constexpr (HORNER) horner_step<M, U>(acc, x[b]);
                else mac<M, ROW0_XOR, U>(acc, x[b], tab, j + b);
            }
        }
    }
    // the bulk form of a kernel with an XOR row and more rows: the streams that row takes come first
    constexpr bool kFolds = ROW0_XOR && !HORNER && KB == 1 && M > 1;
    const int first_end = kFolds ? n_xor : k;
    for (; j < first_end; ++j) {
        const uint8_t *src = s.in[HORNER ? k - 1 - j : j];
        u32x4 x[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            x[u] = u32x4{0, 0, 0, 0};
            if (ok[u]) x[u] = load_piece<NT>(src, piece[u], lane);
        }
        if constexpr (HORNER) horner_step<M, U>(acc, x);
        else mac<M, ROW0_XOR, U>(acc, x, tab, j);
    }
    if constexpr (kFolds) {
        for (; j < k; ++j) {
            u32x4 x[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                x[u] = u32x4{0, 0, 0, 0};
                if (ok[u]) x[u] = load_piece<NT>(s.in[j], piece[u], lane);
            }
            mac<M, true, U, true>(acc, x, tab, j);
        }
#pragma unroll
        for (int r = 1; r < M; ++r)
            if (fold & (1u << r)) {
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int c = 0; c < 4; ++c) acc[0][u].c[c] ^= acc[r][u].c[c];
            }
    }

#pragma unroll
    for (int r = 0; r < M; ++r)
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (ok[u]) store_piece<NT>(s.out[r], piece[u], lane, to_vec(acc[r][u]));
}

// Register budget of a kernel variant, as the occupancy (wavefronts per SIMD)
// the allocator must still be able to reach.  The allocator fills whatever
// budget it is given and runs over it into scratch memory for the widest
// variants, so those get a larger budget (BATCH: pointers and lengths come
// from a descriptor in memory, which costs a few registers more).  How many
// wavefronts really share a CU is decided at launch (LDS reservation).
template <int M, bool ROW0_XOR, int U, bool BATCH = false>
constexpr int kWavesPerEu()
{
    if (U == 1) return (BATCH && M >= 2) ? 5 : 8;             // 102 resp. 64 VGPRs
    if (!ROW0_XOR && (M >= 3 || (BATCH && M >= 2))) return 3;  // 170 VGPRs
    return 4;                                                  // 128 VGPRs
}

// Work distribution.  A shard is cut into 1 KiB pieces (one 16-byte vector per
// lane of a wavefront).  Workgroups are dealt to the 8 XCDs round-robin by
// index, and HBM throughput is best when a given XCD keeps touching the same
// 1 KiB residue class of the address space.  So a tile (one workgroup, 4
// wavefronts x U pieces) is not 4*U consecutive pieces: with interleave
// modulus NX = 2^nx_shift, tile t = g*NX + r takes the pieces
//     (g*4U + q)*NX + r,   q = 0..4U-1,
// i.e. every NX-th piece inside a super-tile of NX*4U pieces, wavefront w
// taking q = w*U .. w*U+U-1.  All NX tiles of a super-tile together cover it
// exactly once.  nx_shift = 0 gives plain consecutive tiles.
template <int M, bool ROW0_XOR, int U, bool NT, bool HORNER, int KB = 1, class S>
__device__ __forceinline__ void contig_streams(const S &s, const uint32_t (&tab)[kLaunchMaxM][kLaunchMaxK][8],
                                               int k, int accumulate, uint32_t tiles_per_wg, bool last_wg,
                                               int n_xor, uint32_t fold = 0)
{
    const uint32_t tid = threadIdx.x;
    // the wavefront's index is the same in all of its lanes: say so, which keeps everything derived
    // from it in scalar registers
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63u;
    constexpr uint32_t kPieces = (kThreads / 64) * U;  // pieces per tile
    const uint32_t nx_shift = s.nx_shift;
    const uint64_t nvec = s.nvec;
    const uint64_t first_tile = static_cast<uint64_t>(blockIdx.x) * tiles_per_wg;
    const uint64_t nx_mask = (1ull << nx_shift) - 1;

    for (uint32_t tt = 0; tt < tiles_per_wg; ++tt) {
        const uint64_t t = first_tile + tt;
        const uint64_t g = t >> nx_shift, r = t & nx_mask;
        // first vector of the super-tile; nothing to do once it is past the end
        const uint64_t super_first = ((g * kPieces) << nx_shift) * 64;
        if (super_first >= nvec) break;
        uint64_t piece[U];
#pragma unroll
        for (int u = 0; u < U; ++u) piece[u] = (((g * kPieces + wave * U + u) << nx_shift) + r) << 6;
        const uint64_t super_end = (((g + 1) * kPieces) << nx_shift) * 64;
        if (super_end <= nvec)
            contig_tile<M, ROW0_XOR, U, NT, true, HORNER, KB>(s, tab, k, accumulate, n_xor, fold, piece, lane);
        else
            contig_tile<M, ROW0_XOR, U, NT, false, HORNER, KB>(s, tab, k, accumulate, n_xor, fold, piece, lane);
    }

    // trailing bytes of a shard whose length is not a multiple of 16: one
    // lane per byte, in the last workgroup
    const uint32_t tail = s.tail;
    if (tail != 0 && last_wg && tid < tail) {
        const uint64_t t = nvec * 16 + tid;
#pragma unroll
        for (int r = 0; r < M; ++r) {
            uint8_t *dst = s.out[r];
            uint32_t sum = accumulate ? dst[t] : 0u;
            for (int j = 0; j < k; ++j) {
                const uint32_t xb = s.in[j][t];
                sum ^= mul1(tab[r][j], xb);  // row 0 too: its table holds the row's own coefficients
            }
            dst[t] = static_cast<uint8_t>(sum);
        }
    }
}

template <int M, bool ROW0_XOR, int U, bool NT>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(kWavesPerEu<M, ROW0_XOR, U>(), 8)))
void apply_contig_kernel(const ApplyArgs a)
{
    contig_streams<M, ROW0_XOR, U, NT, false>(a, a.tab, a.k, a.accumulate, a.tiles_per_wg, blockIdx.x == gridDim.x - 1,
                                              a.n_xor, a.fold);
}

// The same for launches that do not fill the chip (a chunk of a few MiB, a
// decode step): four streams' loads issued together, see contig_tile.
template <int M, bool ROW0_XOR, bool NT>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(kWavesPerEu<M, ROW0_XOR, 2>(), 8)))
void apply_contig_small_kernel(const ApplyArgs a)
{
    contig_streams<M, ROW0_XOR, 2, NT, false, 4>(a, a.tab, a.k, a.accumulate, a.tiles_per_wg, blockIdx.x == gridDim.x - 1, a.k);
}

// Power-code encode by Horner's rule (rows 1, 2^j, 4^j): same tiles, same
// loads and stores, no table lookups.  The tables are still passed: the up to
// 15 bytes after the last whole vector go through the per-byte path.
template <int M, int U, bool NT, int KB = 1>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(kWavesPerEu<M, true, U>(), 8)))
void horner_contig_kernel(const ApplyArgs a)
{
    contig_streams<M, true, U, NT, true, KB>(a, a.tab, a.k, 0, a.tiles_per_wg, blockIdx.x == gridDim.x - 1, a.k);
}

// Many independent chunks in one launch (one request's chunk, or one chunk of
// a long prefill, each): blockIdx.y is the chunk, its pointers and length come
// from a descriptor array in device memory, read with scalar loads through the
// constant address space (descriptors are never written while the kernel runs).
typedef const BatchDesc __attribute__((address_space(4))) *ConstDesc;

template <int M, bool ROW0_XOR, int U, bool NT>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(kWavesPerEu<M, ROW0_XOR, U, true>(), 8)))
void apply_batch_kernel(const BatchArgs a)
{
    ConstDesc d = (ConstDesc)a.descs + blockIdx.y;
    contig_streams<M, ROW0_XOR, U, NT, false>(*d, a.tab, a.k, 0, 1u, blockIdx.x == gridDim.x - 1, a.k);
}

// The grouped launch when all its chunks together do not fill the chip.
template <int M, bool ROW0_XOR, bool NT>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(kWavesPerEu<M, ROW0_XOR, 2, true>(), 8)))
void apply_batch_small_kernel(const BatchArgs a)
{
    ConstDesc d = (ConstDesc)a.descs + blockIdx.y;
    contig_streams<M, ROW0_XOR, 2, NT, false, 4>(*d, a.tab, a.k, 0, 1u, blockIdx.x == gridDim.x - 1, a.k);
}

// One tile of the paged gather.  A lane whose vector index is past the end of
// the plane, or whose page id is outside the plane, reads vector 0 / page 0
// instead (always a valid address) and its value is replaced by zero, so the
// loads need no branches.
//
// WAVE_PAGE: the page size is a multiple of 1 KiB, so the 64 lanes of a piece
// share one page.  The slot is then wavefront-uniform and the table entry is
// fetched with a scalar load through the constant address space (the table is
// never written while the kernel runs), which takes the per-lane divide and
// the vector table loads off the critical path.
typedef const int32_t __attribute__((address_space(4))) *ConstTable;

// MIXED: streams may be table rows or dense buffers on either side (paged
// reconstruct).  Without it (paged encode) input j is table row in_row[0]+j
// and every output is dense, which keeps the per-stream kind tests and one
// dependent scalar load off the latency-bound decode-step path.
template <int M, bool ROW0_XOR, int U, bool NT, bool WAVE_PAGE, bool MIXED, int KB>
__device__ __forceinline__ void paged_tile(const PagedArgs &a, const uint8_t *pbase, uint32_t plane,
                                           const uint64_t (&vv)[U])
{
    bool ok[U];
    uint32_t v[U], slot[U], off[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        ok[u] = vv[u] < a.vecs_per_plane;
        v[u] = ok[u] ? static_cast<uint32_t>(vv[u]) : 0u;
        if (WAVE_PAGE) {
            // vecs_per_plane is a multiple of 64 here, so ok[u] and the slot are uniform
            const uint32_t first = __builtin_amdgcn_readfirstlane(v[u]);
            slot[u] = a.vpp_shift >= 0 ? (first >> a.vpp_shift) : (first / a.vpp);
        } else {
            slot[u] = a.vpp_shift >= 0 ? (v[u] >> a.vpp_shift) : (v[u] / a.vpp);
        }
        off[u] = v[u] - slot[u] * a.vpp;
    }

    Acc4 acc[M][U];
#pragma unroll
    for (int r = 0; r < M; ++r)
#pragma unroll
        for (int u = 0; u < U; ++u) acc[r][u] = Acc4{{0, 0, 0, 0}};
    // page id of table row `row` at this lane's slot, or -1 if out of range
    auto page_of = [&](int32_t row, int u) -> int64_t {
        const uint64_t entry = static_cast<uint64_t>(row) * a.table_stride + slot[u];
        const int64_t page = WAVE_PAGE ? ((ConstTable)a.table)[entry] : a.table[entry];
        return static_cast<uint64_t>(page) < a.pages_per_plane ? page : -1;
    };
    // stream j at vector u: from its page, or from the dense layout
    const int32_t first_row = a.in_row[0];
    // No branch on the kind of stream: base and index are selected (the kind is wavefront-uniform), so
    // the compiler is free to hoist the next stream's lookup and load.  A dense stream still looks up
    // table row 0, which is always there, and ignores the entry.
    auto gather = [&](int j, int u) -> u32x4 {
        const int32_t row = MIXED ? a.in_row[j] : first_row + j;
        const bool dense = MIXED && row < 0;
        const int64_t page = page_of(dense ? 0 : row, u);
        const bool valid = ok[u] && (dense || page >= 0);
        const uint8_t *base = dense ? a.in_ptr[j] : pbase;
        const uint64_t idx = dense ? static_cast<uint64_t>(plane) * a.in_stride[j] + v[u]
                                   : static_cast<uint64_t>(page) * a.vpp + off[u];
        const u32x4 x = load16<NT>(base, valid ? idx : 0ull);
        return valid ? x : u32x4{0, 0, 0, 0};
    };
    // where output r of vector u lives; nullptr if it must not be touched
    auto out_at = [&](int r, int u) -> u32x4 * {
        const int32_t row = MIXED ? a.out_row[r] : -1;
        if (row < 0) return reinterpret_cast<u32x4 *>(a.out[r]) + static_cast<uint64_t>(plane) * a.out_stride[r] + v[u];
        const int64_t page = page_of(row, u);
        if (page < 0) return nullptr;
        return reinterpret_cast<u32x4 *>(const_cast<uint8_t *>(pbase)) + static_cast<uint64_t>(page) * a.vpp + off[u];
    };

    if (a.accumulate) {
#pragma unroll
        for (int r = 0; r < M; ++r)
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const u32x4 *src = out_at(r, u);
                if (ok[u] && src != nullptr) acc[r][u] = from_vec(NT ? __builtin_nontemporal_load(src) : *src);
            }
    }

    // one stream at a time, or KB streams' loads together in a launch that does not fill the chip,
    // as in the contiguous kernel
    int j = 0;
    if constexpr (KB > 1) {
        for (; j + KB <= a.k; j += KB) {
            u32x4 x[KB][U];
#pragma unroll
            for (int b = 0; b < KB; ++b)
#pragma unroll
                for (int u = 0; u < U; ++u) x[b][u] = gather(j + b, u);
#pragma unroll
            for (int b = 0; b < KB; ++b) mac<M, ROW0_XOR, U>(acc, x[b], a.tab, j + b);
        }
    }
    for (; j < a.k; ++j) {
        u32x4 x[U];
#pragma unroll
        for (int u = 0; u < U; ++u) x[u] = gather(j, u);
        mac<M, ROW0_XOR, U>(acc, x, a.tab, j);
    }

#pragma unroll
    for (int r = 0; r < M; ++r)
#pragma unroll
        for (int u = 0; u < U; ++u) {
            u32x4 *dst = out_at(r, u);
            if (ok[u] && dst != nullptr) {
                if (NT) __builtin_nontemporal_store(to_vec(acc[r][u]), dst);
                else *dst = to_vec(acc[r][u]);
            }
        }
}

// Paged gather: blockIdx.y is the plane; blockIdx.x walks the plane's
// slots * vpp vectors in the same interleaved 1 KiB pieces as the
// contiguous kernel (gridDim.x is a multiple of the interleave modulus, so the
// piece residue still names the XCD).  Each lane finds its page slot, looks
// the page id up in every shard's table row, and reads from that page.
template <int M, bool ROW0_XOR, int U, bool WAVE_PAGE, bool MIXED, int KB = 1>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(kWavesPerEu<M, ROW0_XOR, U>(), 8)))
void apply_paged_kernel(const PagedArgs a)
{
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63u;
    constexpr uint32_t kPieces = (kThreads / 64) * U;
    const uint32_t plane = blockIdx.y;
    const uint8_t *pbase = a.plane_base[plane];
    const uint64_t first_tile = static_cast<uint64_t>(blockIdx.x) * a.tiles_per_wg;
    const uint64_t nx_mask = (1ull << a.nx_shift) - 1;

    for (uint32_t tt = 0; tt < a.tiles_per_wg; ++tt) {
        const uint64_t t = first_tile + tt;
        const uint64_t g = t >> a.nx_shift, r = t & nx_mask;
        if (((g * kPieces) << a.nx_shift) * 64 >= a.vecs_per_plane) break;
        uint64_t v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = ((((g * kPieces + wave * U + u) << a.nx_shift) + r) << 6) + lane;
        paged_tile<M, ROW0_XOR, U, true, WAVE_PAGE, MIXED, KB>(a, pbase, plane, v);
    }
}

// ------------------------------------------------------------------ host side

// table words for every constant, built once
struct CoefTable {
    CoefWords c[256];
    CoefTable()
    {
        for (unsigned v = 0; v < 256; ++v) c[v] = split_tables(static_cast<uint8_t>(v));
    }
};

static const CoefTable &coef_table()
{
    static const CoefTable t;
    return t;
}

// Row order of a launch: if some row of the coefficient slice is all ones it
// is moved to position 0 so that the XOR shortcut applies.
struct RowPlan {
    int order[kLaunchMaxM];
    bool row0_xor;
};

static RowPlan plan_rows(int rows, int k, const uint8_t *coef, int coef_stride)
{
    RowPlan p;
    for (int r = 0; r < kLaunchMaxM; ++r) p.order[r] = r;
    p.row0_xor = false;
    for (int r = 0; r < rows && !p.row0_xor; ++r) {
        bool ones = true;
        for (int j = 0; j < k; ++j) ones = ones && coef[r * coef_stride + j] == 1;
        if (ones) {
            p.order[0] = r;
            p.order[r] = 0;
            p.row0_xor = true;
        }
    }
    return p;
}

// table block of a launch, rows in plan order
template <typename Args>
static void fill_tables(Args &a, const RowPlan &p, int rows, int k, const uint8_t *coef, int coef_stride)
{
    const CoefTable &ct = coef_table();
    for (int r = 0; r < kLaunchMaxM; ++r)
        for (int j = 0; j < kLaunchMaxK; ++j) {
            const unsigned c = (r < rows && j < k) ? coef[p.order[r] * coef_stride + j] : 0u;
            for (int i = 0; i < 5; ++i) a.tab[r][j][i] = ct.c[c].w[i];
            a.tab[r][j][5] = a.tab[r][j][6] = a.tab[r][j][7] = 0;
        }
}

// tables and output pointers of a launch; returns true when row 0 is all ones
template <typename Args>
static bool fill_rows(Args &a, int rows, int k, const uint8_t *coef, int coef_stride, void *const *out)
{
    const RowPlan p = plan_rows(rows, k, coef, coef_stride);
    fill_tables(a, p, rows, k, coef, coef_stride);
    for (int r = 0; r < kLaunchMaxM; ++r) a.out[r] = r < rows ? static_cast<uint8_t *>(out[p.order[r]]) : nullptr;
    return p.row0_xor;
}

template <template <int, bool, int, bool> class Launcher, typename Args>
static hipError_t dispatch(int rows, bool row0_xor, int unroll, bool nt, const Args &a, dim3 grid, size_t lds,
                           hipStream_t stream)
{
#define GS_CASE_U(M_, X_, U_)                                                   \
    if (unroll == U_) {                                                         \
        if (nt) return Launcher<M_, X_, U_, true>::go(a, grid, lds, stream);    \
        return Launcher<M_, X_, U_, false>::go(a, grid, lds, stream);           \
    }
#define GS_CASE_MX(M_, X_)  \
    if (rows == M_ && row0_xor == X_) { GS_CASE_U(M_, X_, 1) GS_CASE_U(M_, X_, 2) }
    if (rows == 1 && row0_xor == false) { GS_CASE_U(1, false, 4) }
    if (rows == 1 && row0_xor == true) { GS_CASE_U(1, true, 4) }
    GS_CASE_MX(1, false) GS_CASE_MX(1, true)
    GS_CASE_MX(2, false) GS_CASE_MX(2, true)
    GS_CASE_MX(3, false) GS_CASE_MX(3, true)
    GS_CASE_MX(4, false) GS_CASE_MX(4, true)
#undef GS_CASE_MX
#undef GS_CASE_U
    return hipErrorInvalidValue;
}

template <int M, bool X, int U, bool NT>
struct ContigLauncher {
    static hipError_t go(const ApplyArgs &a, dim3 grid, size_t lds, hipStream_t stream)
    {
        hipLaunchKernelGGL((apply_contig_kernel<M, X, U, NT>), grid, dim3(kThreads), lds, stream, a);
        return hipGetLastError();
    }
};

// launches of at most kSmallWorkgroups workgroups at two vectors per lane
template <int M, bool X, int U, bool NT>
struct ContigSmallLauncher {
    static hipError_t go(const ApplyArgs &a, dim3 grid, size_t lds, hipStream_t stream)
    {
        if constexpr (U == 2)
            hipLaunchKernelGGL((apply_contig_small_kernel<M, X, NT>), grid, dim3(kThreads), lds, stream, a);
        else
            hipLaunchKernelGGL((apply_contig_kernel<M, X, U, NT>), grid, dim3(kThreads), lds, stream, a);
        return hipGetLastError();
    }
};

// the paged kernels always use the streaming cache policy (NT is ignored)
template <int M, bool X, int U, bool NT>
struct PagedLauncher {
    template <bool WAVE_PAGE, bool MIXED>
    static void launch(const PagedArgs &a, dim3 grid, size_t lds, hipStream_t stream)
    {
        if constexpr (U == 1) {
            if (a.small_form && a.k > 1 && static_cast<uint64_t>(grid.x) * grid.y <= kSmallWorkgroups) {
                hipLaunchKernelGGL((apply_paged_kernel<M, X, U, WAVE_PAGE, MIXED, 4>), grid, dim3(kThreads), lds, stream, a);
                return;
            }
        }
        hipLaunchKernelGGL((apply_paged_kernel<M, X, U, WAVE_PAGE, MIXED>), grid, dim3(kThreads), lds, stream, a);
    }
    static hipError_t go(const PagedArgs &a, dim3 grid, size_t lds, hipStream_t stream)
    {
        const bool wave_page = a.vpp % 64 == 0;
        if (a.mixed) wave_page ? launch<true, true>(a, grid, lds, stream) : launch<false, true>(a, grid, lds, stream);
        else wave_page ? launch<true, false>(a, grid, lds, stream) : launch<false, false>(a, grid, lds, stream);
        return hipGetLastError();
    }
};

// Vectors per lane.  0 (the default) picks what measured best: 2 for contiguous
// streams, 1 for the paged gather, where the extra workgroups hide the table
// lookup that precedes every load (+2 to +5 points of HBM peak on bulk pools).
// 4 vectors per lane exist only for the single-row kernels; wider ones would spill.
static int sane_unroll(int u, int rows, int automatic = 2)
{
    if (u == 4 && rows > 1) return 2;
    return (u == 1 || u == 2 || u == 4) ? u : automatic;
}

// workgroups along x, and tiles per workgroup raised if needed so that the
// grid stays below the launch limit on total threads per dimension
static void grid_for(uint64_t tiles, uint32_t &tiles_per_wg, uint32_t &wgs)
{
    constexpr uint64_t kMaxWgs = 1u << 22;
    if (tiles_per_wg < 1) tiles_per_wg = 1;
    uint64_t n = (tiles + tiles_per_wg - 1) / tiles_per_wg;
    if (n > kMaxWgs) {
        tiles_per_wg = static_cast<uint32_t>((tiles + kMaxWgs - 1) / kMaxWgs);
        n = (tiles + tiles_per_wg - 1) / tiles_per_wg;
    }
    wgs = static_cast<uint32_t>(n ? n : 1);
}

// Interleave modulus (shrunk for short streams so that no tile is idle) and the
// tile count rounded up to whole super-tiles.
static void interleave_for(uint64_t nvec, int unroll, int wanted_shift, uint32_t &nx_shift, uint64_t &tiles)
{
    nx_shift = wanted_shift >= 0 && wanted_shift <= 10 ? static_cast<uint32_t>(wanted_shift) : 5u;
    const uint64_t tile = static_cast<uint64_t>(kThreads) * unroll;
    while (nx_shift > 0 && (tile << nx_shift) > nvec) --nx_shift;
    const uint64_t super = tile << nx_shift;
    tiles = ((nvec + super - 1) / super) << nx_shift;
}

// LDS reservation of a bulk launch of the contiguous kernel at two vectors per lane: workgroups
// per CU by kernel variant, from sweeps inside one process over 0.5 to 16 GiB shards, 1+1 to 16+4,
// encode and rebuilds of one to four shards.  The lighter the arithmetic per load, the fewer
// wavefronts: one-row kernels run best with three workgroups (12 wavefronts) per CU, two- and
// three-row kernels with four, four-row kernels and a lone stream with all eight.  The reservation
// starts to pay once a launch fills the chip several times over: from 6144 workgroups (48 MiB
// shards) for kernels of two and more rows (+1 to +2 points there, +2 to +4 from 12288), from
// 12288 for one-row kernels (below that they lose 0.5 to 4 points to it).
static size_t contig_reservation(const LaunchShape &shape, int unroll, int rows, bool row0_xor, int k, uint64_t workgroups)
{
    if (!shape.occupancy_cap || unroll != 2) return 0;
    if (workgroups < (rows == 1 ? kCapMinWorkgroupsOneRow : kCapMinWorkgroupsRows)) return 0;
    switch (rows) {
        case 1: return lds_for_workgroups_per_cu(k == 1 ? 0 : k == 2 ? 4 : 3);
        case 2: return lds_for_workgroups_per_cu(row0_xor && k >= 8 ? 3 : 4);
        case 3: return lds_for_workgroups_per_cu(!row0_xor && k > 8 ? 0 : 4);
        default: return lds_for_workgroups_per_cu(k == 1 ? 3 : 0);
    }
}

hipError_t launch_apply(int rows, int k, const uint8_t *coef, int coef_stride,
                        const void *const *in, void *const *out, size_t bytes,
                        bool accumulate, const LaunchShape &shape, hipStream_t stream)
{
    if (rows < 1 || rows > kLaunchMaxM || k < 1 || k > kLaunchMaxK) return hipErrorInvalidValue;
    if (bytes == 0) return hipSuccess;
    ApplyArgs a;
    bool row0_xor = fill_rows(a, rows, k, coef, coef_stride, out);
    for (int j = 0; j < kLaunchMaxK; ++j) a.in[j] = j < k ? static_cast<const uint8_t *>(in[j]) : nullptr;
    a.n_xor = k;
    a.fold = 0;
    a.nvec = bytes / 16;
    a.tail = static_cast<uint32_t>(bytes % 16);
    a.k = k;
    a.accumulate = accumulate ? 1 : 0;
    const int unroll = sane_unroll(shape.unroll, rows);
    uint32_t nx_shift;
    uint64_t tiles;
    interleave_for(a.nvec, unroll, shape.interleave_shift, nx_shift, tiles);
    uint32_t tpw = shape.tiles_per_wg > 0 ? static_cast<uint32_t>(shape.tiles_per_wg) : 1u, wgs = 1;
    grid_for(tiles, tpw, wgs);
    a.tiles_per_wg = tpw;
    a.nx_shift = nx_shift;
    if (shape.size_forms && unroll == 2 && tpw == 1 && k > 1 && (wgs <= kSmallWorkgroups || shape.size_forms == 2)) {
        // (mode 2: every contiguous launch in this form, with the reservation of its size, for comparison)
        const size_t lds_small = wgs <= kSmallWorkgroups ? 0 : contig_reservation(shape, unroll, rows, row0_xor, k, wgs);
        return dispatch<ContigSmallLauncher>(rows, row0_xor, unroll, shape.nontemporal != 0, a, dim3(wgs), lds_small, stream);
    }
    // Three and four lookup rows keep the vector ALU busy 70 to 80 % of the time at the HBM rate; with one
    // of them turned into an XOR row the rebuild of three shards runs at the rate of the 8+3 encode.
    // (Measured: 8+3 less three 82 -> 83.5 to 84.5 %, 16+3 80 -> 83.6 %, 8+4 less four 79.5 -> 81 to 82.7 %, 16+4
    // 73 -> 79 %.  Two-row rebuilds are HBM-bound either way -- level at k = 4 and 16, 1 to 2 points worse
    // folded at k = 8 -- and stay as they are; a launch that accumulates into its outputs cannot fold,
    // its accumulators start from the previous contents.)
    if (shape.size_forms == 1 && !row0_xor && rows >= 3 && !accumulate) {
        const XorFold f = find_xor_fold(rows, k, coef, coef_stride);
        if (f.found) {
            RowPlan p;
            for (int r = 0; r < kLaunchMaxM; ++r) p.order[r] = f.order[r];
            p.row0_xor = true;
            uint8_t permuted[kLaunchMaxM * kLaunchMaxK];
            for (int r = 0; r < rows; ++r)
                for (int j = 0; j < k; ++j) permuted[r * kLaunchMaxK + j] = coef[r * coef_stride + f.perm[j]];
            fill_tables(a, p, rows, k, permuted, kLaunchMaxK);
            for (int r = 0; r < rows; ++r) a.out[r] = static_cast<uint8_t *>(out[f.order[r]]);
            for (int j = 0; j < k; ++j) a.in[j] = static_cast<const uint8_t *>(in[f.perm[j]]);
            a.n_xor = f.n_xor;
            a.fold = f.fold;
            row0_xor = true;
        }
    }
    const size_t lds = tpw == 1 ? contig_reservation(shape, unroll, rows, row0_xor, k, wgs) : 0;
    return dispatch<ContigLauncher>(rows, row0_xor, unroll, shape.nontemporal != 0, a, dim3(wgs), lds, stream);
}

hipError_t launch_horner(int rows, int k, const uint8_t *coef, int coef_stride, const void *const *in,
                         void *const *out, size_t bytes, const LaunchShape &shape, hipStream_t stream)
{
    if (rows < 2 || rows > 3 || k < 1 || k > kLaunchMaxK) return hipErrorInvalidValue;
    // the kernel hard-wires the matrix: refuse anything but 2^(r*j)
    for (int r = 0; r < rows; ++r) {
        uint8_t g = 1, want = 1;
        for (int i = 0; i < r; ++i) g = gf_mul(g, 2);
        for (int j = 0; j < k; ++j) {
            if (coef[r * coef_stride + j] != want) return hipErrorInvalidValue;
            want = gf_mul(want, g);
        }
    }
    if (bytes == 0) return hipSuccess;
    ApplyArgs a;
    fill_rows(a, rows, k, coef, coef_stride, out);  // row 0 is all ones, so the row order is kept
    for (int j = 0; j < kLaunchMaxK; ++j) a.in[j] = j < k ? static_cast<const uint8_t *>(in[j]) : nullptr;
    a.nvec = bytes / 16;
    a.tail = static_cast<uint32_t>(bytes % 16);
    a.k = k;
    a.accumulate = 0;
    a.n_xor = k;
    a.fold = 0;
    const int unroll = sane_unroll(shape.unroll, rows);
    uint32_t nx_shift;
    uint64_t tiles;
    interleave_for(a.nvec, unroll, shape.interleave_shift, nx_shift, tiles);
    uint32_t tpw = shape.tiles_per_wg > 0 ? static_cast<uint32_t>(shape.tiles_per_wg) : 1u, wgs = 1;
    grid_for(tiles, tpw, wgs);
    a.tiles_per_wg = tpw;
    a.nx_shift = nx_shift;
    const bool nt = shape.nontemporal != 0;
    // no lookups, a few shifts and XORs per load: three workgroups per CU for every k
    const size_t lds = (shape.occupancy_cap && unroll == 2 && tpw == 1 && wgs >= kCapMinWorkgroupsRows)
                           ? lds_for_workgroups_per_cu(3) : 0;
    if (shape.size_forms && unroll == 2 && tpw == 1 && wgs <= kSmallWorkgroups) {  // does not fill the chip: four streams' loads together
        if (rows == 2) {
            if (nt) hipLaunchKernelGGL((horner_contig_kernel<2, 2, true, 4>), dim3(wgs), dim3(kThreads), 0, stream, a);
            else hipLaunchKernelGGL((horner_contig_kernel<2, 2, false, 4>), dim3(wgs), dim3(kThreads), 0, stream, a);
        } else {
            if (nt) hipLaunchKernelGGL((horner_contig_kernel<3, 2, true, 4>), dim3(wgs), dim3(kThreads), 0, stream, a);
            else hipLaunchKernelGGL((horner_contig_kernel<3, 2, false, 4>), dim3(wgs), dim3(kThreads), 0, stream, a);
        }
        return hipGetLastError();
    }
#define GS_HORNER(M_, U_)                                                                                       \
    if (rows == M_ && unroll == U_) {                                                                           \
        if (nt) hipLaunchKernelGGL((horner_contig_kernel<M_, U_, true>), dim3(wgs), dim3(kThreads), lds, stream, a); \
        else hipLaunchKernelGGL((horner_contig_kernel<M_, U_, false>), dim3(wgs), dim3(kThreads), lds, stream, a);   \
        return hipGetLastError();                                                                               \
    }
    GS_HORNER(2, 1) GS_HORNER(2, 2) GS_HORNER(3, 1) GS_HORNER(3, 2)
#undef GS_HORNER
    return hipErrorInvalidValue;
}

template <int M, bool X, int U, bool NT>
struct BatchLauncher {
    static hipError_t go(const BatchArgs &a, dim3 grid, size_t lds, hipStream_t stream)
    {
        hipLaunchKernelGGL((apply_batch_kernel<M, X, U, NT>), grid, dim3(kThreads), lds, stream, a);
        return hipGetLastError();
    }
};

template <int M, bool X, int U, bool NT>
struct BatchSmallLauncher {
    static hipError_t go(const BatchArgs &a, dim3 grid, size_t lds, hipStream_t stream)
    {
        if constexpr (U == 2)
            hipLaunchKernelGGL((apply_batch_small_kernel<M, X, NT>), grid, dim3(kThreads), lds, stream, a);
        else
            hipLaunchKernelGGL((apply_batch_kernel<M, X, U, NT>), grid, dim3(kThreads), lds, stream, a);
        return hipGetLastError();
    }
};

size_t batch_desc_bytes() { return sizeof(BatchDesc); }

void batch_row_order(int rows, int k, const uint8_t *coef, int coef_stride, int *order)
{
    const RowPlan p = plan_rows(rows, k, coef, coef_stride);
    for (int r = 0; r < kLaunchMaxM; ++r) order[r] = p.order[r];
}

uint32_t batch_interleave_shift(int rows, size_t bytes, const LaunchShape &shape)
{
    uint32_t nx_shift;
    uint64_t tiles;
    interleave_for(bytes / 16, sane_unroll(shape.unroll, rows), shape.interleave_shift, nx_shift, tiles);
    return nx_shift;
}

void write_batch_desc(void *slot, int idx, int rows, int k, const int *order, const void *const *in,
                      void *const *out, size_t bytes, const LaunchShape &shape)
{
    BatchDesc &d = static_cast<BatchDesc *>(slot)[idx];
    for (int j = 0; j < kLaunchMaxK; ++j) d.in[j] = j < k ? static_cast<const uint8_t *>(in[j]) : nullptr;
    for (int r = 0; r < kLaunchMaxM; ++r) d.out[r] = r < rows ? static_cast<uint8_t *>(out[order[r]]) : nullptr;
    d.nvec = bytes / 16;
    d.tail = static_cast<uint32_t>(bytes % 16);
    d.nx_shift = batch_interleave_shift(rows, bytes, shape);
}

hipError_t launch_apply_batch(int rows, int k, const uint8_t *coef, int coef_stride, const void *descs_dev,
                              int n_chunks, size_t max_bytes, const LaunchShape &shape, hipStream_t stream)
{
    if (rows < 1 || rows > kLaunchMaxM || k < 1 || k > kLaunchMaxK) return hipErrorInvalidValue;
    if (n_chunks < 1 || n_chunks > 65535) return hipErrorInvalidValue;
    if (max_bytes == 0) return hipSuccess;
    BatchArgs a;
    const RowPlan p = plan_rows(rows, k, coef, coef_stride);
    fill_tables(a, p, rows, k, coef, coef_stride);
    a.descs = static_cast<const BatchDesc *>(descs_dev);
    a.k = k;
    const int unroll = sane_unroll(shape.unroll, rows);
    uint32_t nx_shift;
    uint64_t tiles;
    interleave_for(max_bytes / 16, unroll, shape.interleave_shift, nx_shift, tiles);
    uint32_t tpw = 1, wgs = 1;
    grid_for(tiles, tpw, wgs);
    if (tpw != 1) return hipErrorInvalidValue;  // chunks this large go through launch_apply
    // the grouped kernel runs with four workgroups per CU from 4096 workgroups on, whatever the code:
    // +1 to +3 points of HBM peak for every chunk mix tried, where three help some and ruin others
    const size_t lds = (shape.occupancy_cap && unroll == 2 && static_cast<uint64_t>(wgs) * n_chunks >= 4096)
                           ? lds_for_workgroups_per_cu(4) : 0;
    // all chunks together do not fill the chip (512 workgroups: 1.4 to 3.1 us less from launch to idle; at
    // 1024 the two forms are level)
    if (shape.size_forms && unroll == 2 && k > 1 && static_cast<uint64_t>(wgs) * n_chunks <= kSmallWorkgroups / 2)
        return dispatch<BatchSmallLauncher>(rows, p.row0_xor, unroll, shape.nontemporal != 0, a,
                                            dim3(wgs, static_cast<uint32_t>(n_chunks)), lds, stream);
    return dispatch<BatchLauncher>(rows, p.row0_xor, unroll, shape.nontemporal != 0, a,
                                   dim3(wgs, static_cast<uint32_t>(n_chunks)), lds, stream);
}

hipError_t launch_apply_paged(int rows, int k, const uint8_t *coef, int coef_stride,
                              const void *const *plane_base_dev, int n_planes,
                              size_t page_bytes, int64_t pages_per_plane,
                              const int32_t *table_dev, int table_stride, int n_slots,
                              const PagedStream *in, const PagedStream *out, bool accumulate,
                              const LaunchShape &shape, hipStream_t stream)
{
    if (rows < 1 || rows > kLaunchMaxM || k < 1 || k > kLaunchMaxK) return hipErrorInvalidValue;
    if (n_planes < 1 || n_planes > 65535 || page_bytes == 0 || page_bytes % 16 != 0) return hipErrorInvalidValue;
    if (n_slots < 1 || pages_per_plane < 1 || table_stride < n_slots) return hipErrorInvalidValue;
    const uint64_t vpp = page_bytes / 16;
    const uint64_t vecs = vpp * static_cast<uint64_t>(n_slots);
    if (vpp >= (1ull << 32) || vecs >= (1ull << 32)) return hipErrorInvalidValue;
    // vectors from plane to plane of a dense stream: its own stride, or densely packed
    auto dense_stride = [&](const PagedStream &s, uint32_t &stride) {
        if (s.plane_stride_bytes == 0) {
            stride = static_cast<uint32_t>(vecs);
            return true;
        }
        if (s.plane_stride_bytes % 16 != 0 || s.plane_stride_bytes / 16 < vecs || s.plane_stride_bytes / 16 >= (1ull << 32))
            return false;
        stride = static_cast<uint32_t>(s.plane_stride_bytes / 16);
        return true;
    };
    PagedArgs a;
    const RowPlan p = plan_rows(rows, k, coef, coef_stride);
    fill_tables(a, p, rows, k, coef, coef_stride);
    for (int j = 0; j < kLaunchMaxK; ++j) {
        a.in_row[j] = j < k ? in[j].table_row : -1;
        a.in_ptr[j] = j < k ? static_cast<const uint8_t *>(in[j].dense) : nullptr;
        a.in_stride[j] = 0;
        if (j < k && in[j].table_row < 0 && !dense_stride(in[j], a.in_stride[j])) return hipErrorInvalidValue;
    }
    for (int r = 0; r < kLaunchMaxM; ++r) {
        a.out_row[r] = r < rows ? out[p.order[r]].table_row : -1;
        a.out[r] = r < rows ? static_cast<uint8_t *>(const_cast<void *>(out[p.order[r]].dense)) : nullptr;
        a.out_stride[r] = 0;
        if (r < rows && out[p.order[r]].table_row < 0 && !dense_stride(out[p.order[r]], a.out_stride[r]))
            return hipErrorInvalidValue;
    }
    bool plain = true;  // the paged-encode shape: consecutive table rows in, dense buffers out
    for (int j = 0; j < k; ++j) plain = plain && in[j].table_row >= 0 && in[j].table_row == in[0].table_row + j;
    for (int r = 0; r < rows; ++r) plain = plain && out[r].table_row < 0;
    a.mixed = plain ? 0u : 1u;
    a.small_form = shape.size_forms ? 1u : 0u;
    a.plane_base = reinterpret_cast<const uint8_t *const *>(plane_base_dev);
    a.table = table_dev;
    a.vecs_per_plane = vecs;
    a.pages_per_plane = static_cast<uint64_t>(pages_per_plane < (1ll << 31) ? pages_per_plane : (1ll << 31));
    a.vpp = static_cast<uint32_t>(vpp);
    a.vpp_shift = -1;
    if ((vpp & (vpp - 1)) == 0) {
        int sft = 0;
        while ((1ull << sft) < vpp) ++sft;
        a.vpp_shift = sft;
    }
    a.table_stride = static_cast<uint32_t>(table_stride);
    a.k = k;
    a.accumulate = accumulate ? 1 : 0;
    const int unroll = sane_unroll(shape.unroll, rows, 1);
    uint32_t nx_shift;
    uint64_t tiles;
    interleave_for(vecs, unroll, shape.interleave_shift, nx_shift, tiles);
    // one tile per workgroup keeps gridDim.x a multiple of the modulus
    uint32_t tpw = 1, wgs = 1;
    grid_for(tiles, tpw, wgs);
    a.tiles_per_wg = tpw;
    a.nx_shift = nx_shift;
    // One vector per lane and one stream at a time: a wavefront has a single 1 KiB load in flight, so the
    // gather wants every wavefront the registers allow -- no LDS reservation (any costs it 10 to 25 points).
    return dispatch<PagedLauncher>(rows, p.row0_xor, unroll, shape.nontemporal != 0, a,
                                   dim3(wgs, static_cast<uint32_t>(n_planes)), 0, stream);
}

}  // namespace gs
