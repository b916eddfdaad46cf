/*
 * ghostserve_ec.h -- C ABI of the MI355X (gfx950) erasure-code hot path of
 * GhostServe's shadow checkpointing: k data shards of the KV cache produce m
 * parity shards (Fig. 1(c); Section 4.1), parity is shipped to pinned host
 * memory (Alg. 1), and up to m lost shards are rebuilt from the survivors
 * (Alg. 2).
 *
 * The code is a systematic MDS code over GF(2^8) (polynomial 0x11D): the KV
 * cache is taken as raw bytes -- the reversible integer view of FP16 values of
 * Section 4.1 -- and every byte offset is coded independently.  The paper
 * names the code family (XOR, Reed-Solomon; Section 2) but prints no field or
 * matrix, so the library fixes them: parity block P (m x k) is the Cauchy
 * matrix 1/(x_i + y_j), x_i = k+i, y_j = j, scaled so that row 0 and column 0
 * are all ones.  With m = 1 that is exactly XOR parity.
 *
 * General conventions
 *   - "DEVICE" pointers are addresses the current device can access,
 *     "HOST" pointers are ordinary host addresses, "PINNED" host pointers come
 *     from hipHostMalloc (or an equivalent page-locked allocation).  Pinned
 *     memory is mapped into the device's address space, so a PINNED pointer
 *     is accepted wherever a DEVICE pointer is: an encode whose parity[]
 *     entries are pinned buffers writes the parity over PCIe from the kernel
 *     itself, with no staging buffer and no copy.  That saves a copy launch
 *     per small step; for bulk data the pipelines below keep the kernel short
 *     and leave the transfer to the copy engine.
 *   - Pointer arrays (data[], parity[], shards[]) are HOST arrays holding
 *     DEVICE pointers; they are read during the call and may be freed on return.
 *   - The caller owns every buffer.  A gs_code owns no device memory; a
 *     gs_pipe owns its staging buffers, events and copy stream.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work; they never synchronise unless stated.
 *   - Every entry point returns GS_OK (0) or a negative gs_status; no C++
 *     exception leaves the library.  Arguments are checked before anything
 *     is enqueued: after GS_EINVAL, GS_ETOOMANY, GS_ESINGULAR or GS_ELIMIT no
 *     buffer is written.  GS_EHIP / GS_ENOMEM come from the runtime in mid-call: a call
 *     that issues several launches or copies (wide codes, pipelines, stream
 *     pools) may by then have enqueued some of them.
 *   - Shard base pointers must be 16-byte aligned; shard_bytes may be any
 *     value (the partial last chunk is masked by bounds, Section 4.2).  Bytes
 *     at offsets >= shard_bytes are neither read nor written.
 *   - An output buffer of a call may overlap neither an input nor another
 *     output of that call (of the same chunk, for the many-chunk forms):
 *     contiguous shards are checked and the call returns GS_EINVAL; pages
 *     named by a block table live in device memory and cannot be checked --
 *     a table that names one page twice among the rows a call reads and
 *     writes gives undefined bytes in that page.
 *   - A gs_code is immutable after creation and may be shared between threads.
 *     gs_pipe and gs_batch objects keep the pointer to the gs_code they
 *     were made for: free the code only after them.  Destroy an object only
 *     when the work enqueued through it on the caller's streams has finished
 *     (the destroy calls themselves wait only for the object's own copy
 *     stream and descriptor slots).  gs_free_code never touches the device.
 */
#ifndef GHOSTSERVE_EC_H
#define GHOSTSERVE_EC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gs_code gs_code;
typedef struct gs_pipe gs_pipe;
typedef struct gs_step_graph gs_step_graph;
typedef struct gs_batch gs_batch;
typedef struct gs_pool gs_pool;

enum gs_status {
    GS_OK = 0,
    GS_EINVAL = -1,    /* bad argument (range, alignment, NULL, duplicate index) */
    GS_ENOMEM = -2,    /* host or device allocation failed                       */
    GS_ETOOMANY = -3,  /* more erasures than parity shards                       */
    GS_ESINGULAR = -4, /* survivor matrix not invertible (cannot happen for a code made here) */
    GS_EHIP = -5,      /* a HIP runtime call failed; see gs_last_hip_error()      */
    GS_ELIMIT = -6     /* beyond the fixed capacity of an entry point that allocates nothing */
};

enum gs_kind {
    GS_CAUCHY = 0,      /* closed form described above                                      */
    GS_VANDERMONDE = 1, /* systematic form of the Vandermonde matrix over points 0..k+m-1,
                           with the same normalisation; yields the identical matrix        */
    GS_RDP = 2,         /* row-diagonal parity: XOR-only, exactly two parity shards; see
                           the RDP section below                                           */
    GS_POWER = 3        /* P[i][j] = 2^(i*j): row 0 is XOR parity, row 1 the classic second
                           ("Q") syndrome with generator 2.  A different code from GS_CAUCHY
                           (different parity bytes); MDS only for m <= 3, so m is limited
                           to 3.  Works with every entry point.                            */
};

/* Largest code a single kernel launch covers; wider codes run as several
 * launches that accumulate (transparent to the caller). */
#define GS_LAUNCH_MAX_K 16
#define GS_LAUNCH_MAX_M 4

/* ---- code handle (host only; needs no GPU) -------------------------------
 * Section 2 (Reed-Solomon: distinct coefficients per parity symbol over a
 * Galois field) and Section 4.1 (N data : K parity, user-selectable).
 * Requires 1 <= k, 1 <= m, k + m <= 256, kind one of gs_kind; else GS_EINVAL. */
int gs_make_code(int k, int m, int kind, gs_code **out);
void gs_free_code(gs_code *code);
int gs_code_params(const gs_code *code, int *k, int *m);
/* copies the parity block, m*k bytes row-major, to HOST memory */
int gs_code_matrix(const gs_code *code, uint8_t *P_out);

/* Rebuild matrix for an erasure pattern (host only).  Shard ids 0..k-1 are
 * data, k..k+m-1 parity.  The k lowest-numbered surviving shards are used;
 * their ids go to survivors_out[k], and R_out (n_erased x k, row-major) maps
 * them to the erased shards in the order listed:
 *     erased[x] = XOR_j  R[x][j] (x) survivor_j .
 * A lost data shard r is row r of inverse(A), A the survivors' rows of
 * [I;P]; a lost parity shard k+i is P[i]*inverse(A) (Section 4.1: recovery
 * from up to K simultaneous failures).  Errors: GS_EINVAL for an index out of
 * range or listed twice, GS_ETOOMANY for n_erased > m. */
int gs_decode_matrix(const gs_code *code, const int *erased, int n_erased,
                     uint8_t *R_out, int *survivors_out);

/* ---- encode, contiguous shards --------------------------------------------
 * Alg. 1, "P_i = EC.encode(KV_i)":  for every byte offset t < shard_bytes and
 * parity row i < m,   parity[i][t] = XOR_{j<k} P[i][j] (x) data[j][t].
 *   data    HOST array of k DEVICE pointers, each shard_bytes long, read-only
 *   parity  HOST array of m DEVICE pointers, each shard_bytes long, written
 * shard_bytes == 0 is a no-op.  One fused pass: no conversion or staging
 * kernels (Section 5, kernel fusion). */
int gs_encode(const gs_code *code, const void *const *data, void *const *parity,
              size_t shard_bytes, void *stream);

/* ---- encode, shards gathered from a paged KV pool -------------------------
 * Same sum, but shard j is not contiguous: its logical byte stream is, for
 * plane p = 0..n_planes-1 and slot t = 0..pages_per_shard-1, the page_bytes
 * bytes at  plane_base[p] + table[j*pages_per_shard + t] * page_bytes,
 * and that page's parity lands at offset (p*pages_per_shard + t)*page_bytes
 * of each parity buffer.  (Paged KV cache as in PagedAttention, Section 2;
 * a plane is one layer's K or V pool, a page one block or one token slot.)
 *   plane_base       DEVICE array of n_planes DEVICE pointers (16-byte aligned)
 *   page_bytes       multiple of 16, > 0
 *   pages_per_plane  number of pages in every plane; a table entry outside
 *                    [0, pages_per_plane) contributes zero bytes (never read)
 *   table            DEVICE int32 [k][pages_per_shard]
 *   parity           HOST array of m DEVICE pointers, each
 *                    n_planes*pages_per_shard*page_bytes long
 * plane_base and table are read by the kernel when it runs, so a captured
 * launch sees their current contents on every replay.
 * Limits: n_planes <= 65535, pages_per_shard*page_bytes < 64 GiB. */
int gs_encode_paged(const gs_code *code, const void *const *plane_base, int n_planes,
                    size_t page_bytes, int64_t pages_per_plane,
                    const int32_t *table, int pages_per_shard,
                    void *const *parity, void *stream);

/* Reconstruct in the same paged geometry (Alg. 2 on a paged KV pool): data
 * shard j is the pages of table row j; parity shard i is the dense buffer
 * parity[i] in the layout gs_encode_paged writes.  A lost data shard is
 * rebuilt INTO the pages its table row names (the pages the restarted engine
 * allocated for it; entries outside [0, pages_per_plane) are skipped), a lost
 * parity shard into parity[i].  The k lowest-numbered surviving shards are
 * read; parity entries that are neither read nor written may be NULL.  Pages
 * of surviving shards are never written.  Same limits and error rules as
 * gs_encode_paged and gs_reconstruct. */
int gs_reconstruct_paged(const gs_code *code, const void *const *plane_base, int n_planes,
                         size_t page_bytes, int64_t pages_per_plane,
                         const int32_t *table, int pages_per_shard,
                         void *const *parity, const int *erased, int n_erased, void *stream);

/* ---- reconstruct -----------------------------------------------------------
 * Alg. 2, "KV = EC.reconstruct(KV, P)".
 *   shards   HOST array of k+m DEVICE pointers (0..k-1 data, k..k+m-1 parity),
 *            each shard_bytes long.  Entries listed in `erased` are outputs;
 *            the k lowest-numbered others are read; the rest are ignored and
 *            may be NULL.  Survivors are never written.
 *   erased   HOST array of n_erased distinct ids in [0, k+m)
 * n_erased == 0 is a no-op; n_erased > m gives GS_ETOOMANY. */
int gs_reconstruct(const gs_code *code, void *const *shards, const int *erased, int n_erased,
                   size_t shard_bytes, void *stream);

/* ---- checkpoint / restore pipelines (encode + parity D2H; H2D + reconstruct)
 * Alg. 1 ships each chunk's parity to host DRAM asynchronously while the next
 * chunk is produced; Alg. 2 brings parity back and reconstructs chunk by
 * chunk on streams.  A gs_pipe holds what that needs: `depth` sets of m
 * device staging buffers of chunk_bytes each, events, and a copy stream of
 * default priority.  chunk_bytes must be a positive multiple of 16, depth >= 2.
 * One pipe serves one checkpoint or restore at a time. */
int gs_pipe_create(const gs_code *code, size_t chunk_bytes, int depth, gs_pipe **out);
void gs_pipe_destroy(gs_pipe *pipe);

/* Encode `data` chunk by chunk on compute_stream into staging, and copy each
 * chunk's parity to host_parity[i] + offset on the pipe's copy stream, so the
 * copy of chunk c overlaps the encode of chunk c+1.
 *   data         HOST array of k DEVICE pointers, shard_bytes each
 *   host_parity  HOST array of m PINNED host pointers, shard_bytes each
 * Returns after enqueuing; the parity bytes are valid once gs_pipe_sync()
 * returns (or after the event gs_pipe_done_event() on another stream).  If a
 * runtime call fails part of the way (GS_EHIP), gs_pipe_sync() still waits for
 * everything that had been enqueued, so the buffers can be released safely. */
int gs_checkpoint(gs_pipe *pipe, const void *const *data, size_t shard_bytes,
                  void *const *host_parity, void *compute_stream);

/* Rebuild the erased shards chunk by chunk.  Parity shards that the decode
 * needs are read from host_parity (PINNED) through the staging buffers (H2D
 * on the copy stream, overlapped with the reconstruct kernel of the previous
 * chunk); data survivors are read in place.
 *   shards       HOST array of k+m pointers; entries 0..k-1 are DEVICE data
 *                shards (outputs if erased); entries k..k+m-1 are ignored
 *                unless erased, in which case they are DEVICE outputs
 *   host_parity  HOST array of m PINNED pointers (entries for erased parity
 *                shards are ignored) */
int gs_restore(gs_pipe *pipe, void *const *shards, void *const *host_parity,
               const int *erased, int n_erased, size_t shard_bytes, void *compute_stream);

/* The same two pipelines over a paged KV pool (geometry and argument meaning
 * as in gs_encode_paged / gs_reconstruct_paged): Alg. 1 and Alg. 2 run on the
 * serving engine's paged cache (Section 5), where a chunk of tokens is a window
 * of page slots in every plane.  A chunk here is the
 *     slots_per_chunk = min(pages_per_shard, chunk_bytes / (n_planes*page_bytes))
 * next slots of every plane (chunk_bytes of the pipe; GS_EINVAL if that is
 * zero); the last chunk may be shorter.  Parity lives in host memory in the
 * dense layout gs_encode_paged writes, [plane][pages_per_shard][page_bytes], so
 * what a paged checkpoint stores equals what one gs_encode_paged call over the
 * whole table would have produced; each chunk's window of it moves with one
 * strided copy per parity shard.
 *   host_parity  HOST array of m PINNED pointers, n_planes*pages_per_shard*page_bytes each
 *   parity_out   gs_restore_paged only: HOST array of m DEVICE pointers in the
 *                same dense layout, used only for erased parity shards (may be
 *                NULL when none is erased)
 * A lost data shard is rebuilt INTO the pages its table row names.  The block
 * table and plane pointers are read by the kernels when they run and must stay
 * unchanged until the pipe has finished. */
int gs_checkpoint_paged(gs_pipe *pipe, const void *const *plane_base, int n_planes, size_t page_bytes,
                        int64_t pages_per_plane, const int32_t *table, int pages_per_shard,
                        void *const *host_parity, void *compute_stream);
int gs_restore_paged(gs_pipe *pipe, const void *const *plane_base, int n_planes, size_t page_bytes,
                     int64_t pages_per_plane, const int32_t *table, int pages_per_shard,
                     void *const *host_parity, void *const *parity_out, const int *erased, int n_erased,
                     void *compute_stream);

/* block the host until everything the pipe enqueued has finished */
int gs_pipe_sync(gs_pipe *pipe);
/* hipEvent_t (as void*) recorded after the last operation enqueued so far */
void *gs_pipe_done_event(gs_pipe *pipe);
/* Per-chunk timeline of a pipe (off by default).  With timing enabled, every
 * later gs_checkpoint / gs_restore call records timing events around each
 * chunk's kernel on the compute stream and after each chunk's copies on the
 * copy stream.  gs_pipe_chunk_times waits for the last call to finish and
 * returns, for its first min(n_chunks, max_chunks) chunks, milliseconds since
 * the call began on the compute stream: when the chunk's encode / reconstruct
 * kernel began and ended, and when its parity copy (D2H for a checkpoint, H2D
 * for a restore) ended.  Any of the three arrays may be NULL; *n_chunks_out is
 * the number of chunks of that call (0 if none was timed).  This is how the
 * overlap of Alg. 1's encode with its asynchronous PCIe copy is observed. */
int gs_pipe_set_timing(gs_pipe *pipe, int enable);
int gs_pipe_chunk_times(gs_pipe *pipe, int max_chunks, float *kernel_begin_ms, float *kernel_end_ms,
                        float *copy_end_ms, int *n_chunks_out);

/* ---- captured per-step checkpoint (Section 5: graphs for fixed-size chunks)
 * Captures gs_encode_paged (+ optional D2H of the m parity buffers into
 * host_parity, PINNED, may be NULL for no copy) once, and replays it with one
 * graph launch per decode step.  The block table and plane pointers are read
 * from device memory at replay time, so the serving engine advances a step by
 * updating them in place.  No memset nodes are recorded. */
int gs_step_graph_create(const gs_code *code, const void *const *plane_base, int n_planes,
                         size_t page_bytes, int64_t pages_per_plane,
                         const int32_t *table, int pages_per_shard,
                         void *const *parity, void *const *host_parity,
                         gs_step_graph **out);
int gs_step_graph_launch(gs_step_graph *g, void *stream);
void gs_step_graph_destroy(gs_step_graph *g);

/* ---- RDP (row-diagonal parity) -----------------------------------------------
 * The third code the paper offers (Section 2, Section 4.1): XOR-only, two
 * parity shards, any two lost shards recoverable.  1 <= k <= 16.  Geometry as
 * published for RDP: p = smallest prime >= max(3, k+1); a stripe is p-1 rows
 * of one cell per shard; data shards beyond k up to p-1 are imaginary zeros;
 * shard ids: 0..k-1 data, k row parity, k+1 diagonal parity.  Cell (i, j) of
 * the first p "disks" (data + row parity) lies on diagonal (i+j) mod p;
 * diagonal parity cell d is the XOR of diagonal d, d = 0..p-2.  As on a disk
 * array a shard holds consecutive, independent stripes: stripe s is the
 * (p-1)*cell_bytes bytes at offset s*(p-1)*cell_bytes of every shard, its
 * cell i is row i (the paper does not say how its RDP lays the KV bytes out;
 * this is the library's reading).  cell_bytes is a power of two >= 16;
 * gs_make_code(k, 2, GS_RDP) uses GS_RDP_DEFAULT_CELL, which keeps the rows of
 * a stripe inside the period of the kernels' piece interleave.
 * An RDP code works with gs_encode (parity[0] = row parity, parity[1] =
 * diagonal parity) and gs_reconstruct, with the same argument conventions,
 * except that shard_bytes must be a whole number of stripes (else GS_EINVAL).
 * The checkpoint / restore pipelines accept it when chunk_bytes is a whole
 * number of stripes.  The paged entry points (gs_encode_paged,
 * gs_reconstruct_paged, gs_checkpoint_paged, gs_restore_paged) accept it when a
 * cell is a page: page_bytes == cell_bytes (make the code with
 * gs_make_rdp_code(k, page_bytes)), page_bytes >= 1024, and pages_per_shard a
 * multiple of p-1 -- a stripe is then p-1 consecutive page slots of a plane,
 * which is the contiguous definition applied to the shard's gathered byte
 * stream, and a shard's share of one plane must be below (p-1) x 16 GiB;
 * anything else gives GS_EINVAL.  The grouped launch (gs_batch)
 * takes it too, every chunk a whole number of stripes; the allocation-free
 * grouped encode does not.  gs_code_matrix / gs_decode_matrix return GS_EINVAL
 * for it.  A single lost shard other than the diagonal parity is rebuilt from
 * the row equations alone (the diagonal parity shard is then not read and may
 * be NULL). */
#define GS_RDP_DEFAULT_CELL 32768
int gs_make_rdp_code(int k, size_t cell_bytes, gs_code **out);
int gs_rdp_prime(const gs_code *code, int *p_out);
int gs_rdp_cell_bytes(const gs_code *code, size_t *cell_out);
/* The plan the kernels execute (host only; lets the planning be checked
 * without a GPU).  The device first accumulates, per stripe, the syndromes
 * SR[i] = XOR of row i over the shards read among data and row parity, and
 * SD[d] = XOR of diagonal d over those shards plus diagonal-parity cell d (if
 * read); every missing cell is then the XOR of a set of syndromes.
 * n_missing = 0 asks for the encode plan (both parity shards missing).
 * read_out (room for 18 shard ids) lists the shards that are read;
 * syndrome_mask_out (room for 32 words) holds, for missing shard x (in the
 * order given) and row q, at [x*(p-1)+q], bit i (< p-1) set when SR[i] is part
 * of the cell and bit p-1+d when SD[d] is. */
int gs_rdp_plan(const gs_code *code, const int *missing, int n_missing, int *read_out, int *n_read_out,
                uint32_t *syndrome_mask_out);

/* ---- many chunks at once ---------------------------------------------------
 * Section 5: recovery reconstructs many chunks concurrently ("each chunk is
 * assigned to a dedicated stream"), and with continuous batching every request
 * encodes its own chunk.  Small chunks do not fill 256 CUs one launch at a
 * time, so two forms are offered.
 *
 * Grouped launch (gs_batch): all chunks go through ONE kernel launch; their
 * pointers and lengths travel in a descriptor array that the gs_batch owns
 * (device buffer + pinned host mirror, a ring of 4 slots so that consecutive
 * calls do not wait for each other).  Codes with k <= 16 and m <= 4 only
 * (RDP codes included: then every chunk must be a whole number of stripes
 * and shorter than (p-1) x 16 GiB, else GS_EINVAL with nothing enqueued),
 * max_chunks <= 65535, chunks below 16 GiB (longer ones: gs_encode).  One
 * gs_batch serves one thread at a time.  The descriptor slot is filled by the host at call time and may make the host
 * wait for the launch that used it four calls earlier, so these two calls
 * must not be made on a stream that is being captured into a graph (the
 * single-chunk entry points can be).
 *   data     HOST array of n_chunks*k DEVICE pointers, chunk-major
 *   parity   HOST array of n_chunks*m DEVICE pointers, chunk-major
 *   shards   HOST array of n_chunks*(k+m) DEVICE pointers, chunk-major, same
 *            meaning per chunk as in gs_reconstruct; one erasure pattern for
 *            all chunks (a failed device loses the same shard of every chunk)
 *   shard_bytes  HOST array of n_chunks lengths (any values, 0 = skip)
 * Results per chunk are exactly those of gs_encode / gs_reconstruct. */
int gs_batch_create(const gs_code *code, int max_chunks, gs_batch **out);
void gs_batch_destroy(gs_batch *batch);
int gs_encode_batch(gs_batch *batch, int n_chunks, const void *const *data, void *const *parity,
                    const size_t *shard_bytes, void *stream);
int gs_reconstruct_batch(gs_batch *batch, int n_chunks, void *const *shards, const int *erased,
                         int n_erased, const size_t *shard_bytes, void *stream);

/* Grouped encode that allocates nothing.  For callers that cannot call
 * hipMalloc: code under HIP graph capture, tight serving loops, harnesses that
 * forbid allocation.  Same arguments and results as gs_encode_batch without
 * the gs_batch object: the chunk descriptors live in a fixed array inside the
 * library's device image (GS_STATIC_MAX_CHUNKS descriptors, 176 KiB, held on
 * every device the library runs on until the process ends) and are written by
 * a small kernel that receives them as launch arguments, so the call enqueues
 * kernel launches only -- no allocation, no copy, no host wait -- and may be
 * captured into a graph.
 *   n_chunks > GS_STATIC_MAX_CHUNKS, or a chunk of 16 GiB or more: GS_ELIMIT,
 *   nothing enqueued.  Codes with k <= 16 and m <= 4 only, and no RDP code
 *   (else GS_EINVAL).
 * All calls on one device share that device's array, and a call overwrites
 * what the previous one left there: calls on the same stream are ordered by
 * the stream; calls that may run at the same time on different streams of one
 * device race on the array and must be ordered by the caller (an event). */
#define GS_STATIC_MAX_CHUNKS 1024
int gs_encode_batch_static(const gs_code *code, int n_chunks, const void *const *data, void *const *parity,
                           const size_t *shard_bytes, void *stream);

/* Stream pool (gs_pool): the paper's form.  Chunk c is enqueued on pool
 * stream c mod n_streams (default priority); the pool streams start after the
 * work already enqueued on `stream`, and `stream` continues only after every
 * chunk has finished.  1 <= n_streams <= 64.  Same array layouts as above. */
int gs_pool_create(int n_streams, gs_pool **out);
void gs_pool_destroy(gs_pool *pool);
int gs_encode_streams(const gs_code *code, gs_pool *pool, int n_chunks, const void *const *data,
                      void *const *parity, const size_t *shard_bytes, void *stream);
int gs_reconstruct_streams(const gs_code *code, gs_pool *pool, int n_chunks, void *const *shards,
                           const int *erased, int n_erased, const size_t *shard_bytes, void *stream);

/* ---- hybrid recovery planner (host only) -----------------------------------
 * Alg. 2 recomputes the first r chunks of the lost KV cache on the restarted
 * device while the other n-r chunks are reconstructed from the survivors and
 * the parity coming back over PCIe; r = get_recompute_units(...) is left
 * undefined by the paper.  Here it is the r in [0, n] that minimises
 *     max( recompute(r), restore(n - r) )
 * under a cost model the caller fills from its own measurements:
 *     recompute(r) = sum_{i<r} (recompute_base_s + recompute_growth_s * i)
 *                    (a chunk's prefill grows with the context before it)
 *     restore(q)   = 0 for q = 0, else restore_startup_s + the two faster of
 *                    {gather_s, h2d_s, reconstruct_s} once + q * the slowest
 *                    (a three-stage pipeline per chunk)
 * Ties go to the smaller r.  r = n means pure recomputation (short inputs).
 * All costs are seconds per chunk, finite and >= 0, else GS_EINVAL. */
typedef struct gs_recovery_costs {
    double recompute_base_s;    /* prefill of one chunk with no context before it     */
    double recompute_growth_s;  /* extra prefill time per chunk of preceding context  */
    double gather_s;            /* collect one chunk's surviving data shards          */
    double h2d_s;               /* bring one chunk's parity back from host memory     */
    double reconstruct_s;       /* reconstruct kernel on one chunk                    */
    double restore_startup_s;   /* fixed cost of starting the restore pipeline at all */
} gs_recovery_costs;
int gs_recompute_units(int n_chunks, const gs_recovery_costs *costs, int *r_out, double *makespan_out);

/* ---- diagnostics -----------------------------------------------------------*/
const char *gs_strerror(int status);
/* last hipError_t seen by the calling thread in this library (0 = none) */
int gs_last_hip_error(void);
/* The five lookup words the kernels use for multiplication by the constant c
 * (0..255): a byte x is cut into bit fields x[2:0], x[5:3], x[7:6] and
 *   c (x) x = T0[x & 7] ^ T1[(x >> 3) & 7] ^ T2[x >> 6],
 * words_out = {T0[0..3], T0[4..7], T1[0..3], T1[4..7], T2[0..3]} with table
 * entry i in byte (i & 3) of its word.  Host only; exposed so that the table
 * construction can be checked without a GPU. */
int gs_coef_words(int c, uint32_t *words_out);
/* Launch-shape knobs for benchmarking sweeps; a value <= 0 (< 0 for the last
 * two) restores that knob's default.
 *   unroll            16-byte vectors per lane per shard per tile (1, 2 or 4;
 *                     default: 2 for contiguous shards, 1 for the paged gather)
 *   tiles_per_wg      consecutive tiles one workgroup processes
 *   nontemporal       1 = streaming loads/stores, 0 = default cache policy
 *   interleave_shift  log2 of the modulus with which the contiguous kernel
 *                     deals 1 KiB pieces to workgroups (0 = consecutive
 *                     pieces, default 5; at most 10)
 * Results are identical for every setting.  Process-wide, like
 * gs_set_power_horner; both are atomic: a call running in another thread uses
 * either the old or the new setting as a whole. */
int gs_set_launch_shape(int unroll, int tiles_per_wg, int nontemporal, int interleave_shift);
/* Bulk launches of the contiguous, grouped, Horner and RDP kernels (shards
 * of 48 MiB and more, 96 MiB for one-row launches and RDP, 4096 workgroups
 * for the grouped launch; default vectors per lane and tiles per workgroup)
 * ask for 40 to 64 KiB of LDS per workgroup that the kernels never touch,
 * which keeps 4, 3 or 2 workgroups on a CU instead of 8: that moves 1 to 4
 * points more of the HBM peak.  While such a kernel runs, other kernels that need LDS find
 * little of it free on the same CUs; enable = 0 switches the reservation off
 * (process-wide and atomic like the knobs above; gs_set_launch_shape leaves it
 * as it is).  Results are identical either way.  Default: enabled. */
int gs_set_occupancy_cap(int enable);
/* Two kinds of launches run kernel forms of their own.  A launch that does
 * not fill the chip (at most 1024 workgroups: shards up to 8 MiB, a decode
 * step, a small group of chunks) issues the loads of four streams together,
 * because its time is a wavefront's memory round trips one after the other.
 * A bulk rebuild of three or four contiguous shards with the all-ones parity
 * among the survivors computes one of the lost shards as a plain XOR of
 * inputs and of the other rebuilt shards instead of by table lookups.
 * mode = 0 sends both through the general bulk form; mode = 2 runs every
 * contiguous launch, whatever its size, in the form of small launches (the
 * loads of four streams together, which is what bulk launches used before one
 * stream at a time measured faster); mode = 1 is the default.  The bytes are
 * the same in every mode, which is what the switch is for: tests compare the
 * forms, and bench.py times them side by side.  Other values: GS_EINVAL.
 * Process-wide and atomic like the knobs above; gs_set_launch_shape leaves it
 * as it is. */
int gs_set_size_forms(int mode);
/* gs_encode of a GS_POWER code with m = 2 or 3 and k <= 16 evaluates the
 * parity rows by Horner's rule (par_r = (..(d_{k-1} g + d_{k-2}) g ..) g + d_0
 * with g = 2^r; one packed multiply-by-2 per stream and row, no table
 * lookups).  enable = 0 sends those encodes through the general matrix kernel
 * instead; the parity bytes are the same either way.  Default: enabled. */
int gs_set_power_horner(int enable);

#ifdef __cplusplus
}
#endif
#endif /* GHOSTSERVE_EC_H */
