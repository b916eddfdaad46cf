/*
 * gs_oracle.c -- plain CPU oracle for the erasure-code hot path of GhostServe's
 * shadow checkpointing.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is the slow, obviously-correct statement of
 * what the GPU library must compute, bit for bit.  Only the test-suite, the
 * smoke check and the benchmark's "cpu_baseline" leg may call it; the product
 * (the HIP library) never links, loads or imports anything from this folder,
 * and this file shares no code, tables or headers with it.
 *
 * What the paper fixes (Section 2 "Erasure Coding", Section 4.1, Fig. 1(c)):
 *   - N data shards produce K parity shards (here: k data, m parity);
 *   - XOR parity is bitwise XOR across the data shards (one parity, one loss);
 *   - Reed-Solomon works over a Galois field with distinct coefficients per
 *     parity symbol and survives up to K simultaneous losses;
 *   - FP16 values are reinterpreted as fixed-width integer bit patterns, which
 *     is reversible, so recovery is lossless (here: raw bytes are the symbols);
 *   - partial last chunks are handled by bounds, parity only over active bytes.
 * What the paper leaves open and this oracle fixes by a stated reading:
 *   - field: GF(2^8) = GF(2)[x]/(x^8+x^4+x^3+x^2+1) (0x11D), generator 2;
 *   - generator matrix: systematic Vandermonde-derived code over evaluation
 *     points 0..k+m-1, normalised so that parity row 0 and parity column 0 are
 *     all ones (hence m=1 is exactly XOR parity);
 *   - decoding uses the k lowest-indexed surviving shards.
 *
 * Arithmetic here is scalar log/exp-table GF(2^8); no SIMD, no blocking, no
 * fusion: every function is the textbook definition written out.
 *
 * Parity status: every function below is pinned by tests that do not call it
 * to produce their expected values (field axioms by brute force, an
 * independent carry-less multiply, the Cauchy closed form, exhaustive MDS
 * checks, XOR reduction, impulse responses, erase-every-subset round trips,
 * explicit gathers).  Nothing here is "parity unpinned".
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <pthread.h>

#define GSO_POLY 0x11D

static uint8_t g_exp[510]; /* exp[i] = 2^i, doubled so log a + log b needs no mod */
static uint8_t g_log[256]; /* log[0] unused */
static int g_ready = 0;

/* Section 2 (Reed-Solomon "over Galois fields"): build the field by repeated
 * multiplication by x, reducing by the field polynomial when bit 8 appears. */
void gso_init(void)
{
    if (g_ready) return;
    unsigned v = 1;
    for (int i = 0; i < 255; i++) {
        g_exp[i] = (uint8_t)v;
        g_log[v] = (uint8_t)i;
        v <<= 1;
        if (v & 0x100) v ^= GSO_POLY;
    }
    for (int i = 255; i < 510; i++) g_exp[i] = g_exp[i - 255];
    g_log[0] = 0;
    g_ready = 1;
}

uint8_t gso_mul(uint8_t a, uint8_t b)
{
    gso_init();
    if (a == 0 || b == 0) return 0;
    return g_exp[(int)g_log[a] + (int)g_log[b]];
}

/* multiplicative inverse; a must be non-zero (returns 0 for 0 as a sentinel) */
uint8_t gso_inv(uint8_t a)
{
    gso_init();
    if (a == 0) return 0;
    return g_exp[(255 - (int)g_log[a]) % 255];
}

static uint8_t gso_div(uint8_t a, uint8_t b) { return gso_mul(a, gso_inv(b)); }

static uint8_t gso_pow(uint8_t a, unsigned e)
{
    /* 0^0 = 1 (needed for the Vandermonde column of constants) */
    uint8_t r = 1;
    for (unsigned i = 0; i < e; i++) r = gso_mul(r, a);
    return r;
}

/* hand the raw tables to a test */
void gso_tables(uint8_t *exp_out /*255*/, uint8_t *log_out /*256*/)
{
    gso_init();
    memcpy(exp_out, g_exp, 255);
    memcpy(log_out, g_log, 256);
}

/* the full 256x256 product table, row a, column b */
void gso_mul_table(uint8_t *out /*65536*/)
{
    for (int a = 0; a < 256; a++)
        for (int b = 0; b < 256; b++)
            out[a * 256 + b] = gso_mul((uint8_t)a, (uint8_t)b);
}

/* Gauss-Jordan inverse of an n x n matrix over the field (row-major).
 * Returns 0, or -1 if A is singular.  A is not modified. */
int gso_invert(int n, const uint8_t *A, uint8_t *Ainv)
{
    gso_init();
    uint8_t *w = (uint8_t *)malloc((size_t)n * n);
    if (!w) return -2;
    memcpy(w, A, (size_t)n * n);
    for (int r = 0; r < n; r++)
        for (int c = 0; c < n; c++) Ainv[r * n + c] = (r == c);
    for (int col = 0; col < n; col++) {
        int piv = -1;
        for (int r = col; r < n; r++)
            if (w[r * n + col]) { piv = r; break; }
        if (piv < 0) { free(w); return -1; }
        if (piv != col)
            for (int c = 0; c < n; c++) {
                uint8_t t = w[col * n + c]; w[col * n + c] = w[piv * n + c]; w[piv * n + c] = t;
                t = Ainv[col * n + c]; Ainv[col * n + c] = Ainv[piv * n + c]; Ainv[piv * n + c] = t;
            }
        uint8_t s = gso_inv(w[col * n + col]);
        for (int c = 0; c < n; c++) {
            w[col * n + c] = gso_mul(w[col * n + c], s);
            Ainv[col * n + c] = gso_mul(Ainv[col * n + c], s);
        }
        for (int r = 0; r < n; r++) {
            if (r == col) continue;
            uint8_t f = w[r * n + col];
            if (!f) continue;
            for (int c = 0; c < n; c++) {
                w[r * n + c] ^= gso_mul(f, w[col * n + c]);
                Ainv[r * n + c] ^= gso_mul(f, Ainv[col * n + c]);
            }
        }
    }
    free(w);
    return 0;
}

/* Generator of the systematic code G = [I_k ; P], P is m x k (row-major).
 *
 * Route (deliberately the long way round): Vandermonde matrix V[r][c] = r^c
 * over the evaluation points r = 0..k+m-1 (field elements), made systematic by
 * G' = V * inverse(V[0:k]); the bottom m rows of G' are the raw parity block.
 * It is then normalised: each column divided by its row-0 entry, then each row
 * divided by its column-0 entry, so that P[0][*] = P[*][0] = 1.  Scaling rows
 * and columns by non-zero constants keeps every square minor non-zero, so the
 * code stays MDS, and with m = 1 the parity is the plain XOR of the data
 * (Section 2, XOR coding).  Returns 0, -1 on bad (k, m). */
int gso_generator(int k, int m, uint8_t *P)
{
    gso_init();
    if (k < 1 || m < 1 || k + m > 256) return -1;
    int n = k + m;
    uint8_t *V = (uint8_t *)malloc((size_t)n * k);
    uint8_t *Vt = (uint8_t *)malloc((size_t)k * k);
    uint8_t *Vi = (uint8_t *)malloc((size_t)k * k);
    uint8_t *raw = (uint8_t *)malloc((size_t)m * k);
    if (!V || !Vt || !Vi || !raw) { free(V); free(Vt); free(Vi); free(raw); return -2; }
    for (int r = 0; r < n; r++)
        for (int c = 0; c < k; c++) V[r * k + c] = gso_pow((uint8_t)r, (unsigned)c);
    memcpy(Vt, V, (size_t)k * k);
    int rc = gso_invert(k, Vt, Vi);
    if (rc == 0) {
        for (int i = 0; i < m; i++)
            for (int j = 0; j < k; j++) {
                uint8_t s = 0;
                for (int t = 0; t < k; t++) s ^= gso_mul(V[(k + i) * k + t], Vi[t * k + j]);
                raw[i * k + j] = s;
            }
        /* column scaling: row 0 becomes all ones */
        for (int j = 0; j < k; j++) {
            uint8_t d = raw[0 * k + j];
            for (int i = 0; i < m; i++) raw[i * k + j] = gso_div(raw[i * k + j], d);
        }
        /* row scaling: column 0 becomes all ones */
        for (int i = 0; i < m; i++) {
            uint8_t d = raw[i * k + 0];
            for (int j = 0; j < k; j++) P[i * k + j] = gso_div(raw[i * k + j], d);
        }
    }
    free(V); free(Vt); free(Vi); free(raw);
    return rc;
}

/* Encode (Alg. 1, "P_i = EC.encode(KV_i)"): for every byte offset t < S and
 * every parity row i:  parity[i][t] = XOR_j  P[i][j] (x) data[j][t].
 * Bytes at offsets >= S are neither read nor written (partial last chunk). */
void gso_encode(int k, int m, const uint8_t *P,
                const uint8_t *const *data, uint8_t *const *parity, size_t S)
{
    gso_init();
    for (size_t t = 0; t < S; t++)
        for (int i = 0; i < m; i++) {
            uint8_t s = 0;
            for (int j = 0; j < k; j++) s ^= gso_mul(P[i * k + j], data[j][t]);
            parity[i][t] = s;
        }
}

/* Paged encode.  Shard j's logical byte stream is, for plane p = 0..n_planes-1
 * and page slot t = 0..pages_per_shard-1, the page_bytes bytes starting at
 * plane_base[p] + table[j*pages_per_shard + t] * page_bytes; that page lands
 * at parity offset (p*pages_per_shard + t) * page_bytes.  (Paged KV cache:
 * Section 2 mentions PagedAttention; the layout is this build's reading.) */
void gso_encode_paged(int k, int m, const uint8_t *P,
                      const uint8_t *const *plane_base, int n_planes, size_t page_bytes,
                      const int32_t *table, int pages_per_shard,
                      uint8_t *const *parity)
{
    gso_init();
    for (int p = 0; p < n_planes; p++)
        for (int t = 0; t < pages_per_shard; t++)
            for (size_t b = 0; b < page_bytes; b++) {
                size_t off = ((size_t)p * pages_per_shard + t) * page_bytes + b;
                for (int i = 0; i < m; i++) {
                    uint8_t s = 0;
                    for (int j = 0; j < k; j++) {
                        size_t page = (size_t)table[(size_t)j * pages_per_shard + t];
                        s ^= gso_mul(P[i * k + j], plane_base[p][page * page_bytes + b]);
                    }
                    parity[i][off] = s;
                }
            }
}

/* validate an erasure list; 0 ok, -1 bad index / duplicate, -3 more than m */
static int gso_check_erased(int k, int m, const int *erased, int e, uint8_t *lost /*k+m*/)
{
    memset(lost, 0, (size_t)(k + m));
    if (e < 0) return -1;
    for (int x = 0; x < e; x++) {
        if (erased[x] < 0 || erased[x] >= k + m) return -1;
        if (lost[erased[x]]) return -1;
        lost[erased[x]] = 1;
    }
    if (e > m) return -3;
    return 0;
}

/* row r of G = [I_k ; P] */
static void gso_g_row(int k, const uint8_t *P, int r, uint8_t *row)
{
    if (r < k) for (int c = 0; c < k; c++) row[c] = (c == r);
    else       for (int c = 0; c < k; c++) row[c] = P[(r - k) * k + c];
}

/* The k lowest-indexed surviving shards and the inverse of their k x k
 * generator sub-matrix A.  Returns 0, -1/-3 for a bad list, -4 if singular. */
static int gso_survivor_inverse(int k, int m, const uint8_t *P, const int *erased, int e,
                                int *survivors /*k*/, uint8_t *Ainv /*k*k*/)
{
    uint8_t lost[256];
    int rc = gso_check_erased(k, m, erased, e, lost);
    if (rc) return rc;
    int n = 0;
    for (int r = 0; r < k + m && n < k; r++)
        if (!lost[r]) survivors[n++] = r;
    uint8_t *A = (uint8_t *)malloc((size_t)k * k);
    if (!A) return -2;
    for (int r = 0; r < k; r++) gso_g_row(k, P, survivors[r], A + (size_t)r * k);
    rc = gso_invert(k, A, Ainv);
    free(A);
    return rc == -1 ? -4 : rc;
}

/* Rebuild matrix R (e x k): erased[x] = XOR_j R[x][j] (x) survivor_j.
 * A lost data shard r is row r of inverse(A); a lost parity shard k+i is
 * P[i] * inverse(A). */
int gso_decode_matrix(int k, int m, const uint8_t *P, const int *erased, int e,
                      uint8_t *R /*e*k*/, int *survivors /*k*/)
{
    gso_init();
    uint8_t *Ainv = (uint8_t *)malloc((size_t)k * k);
    if (!Ainv) return -2;
    int rc = gso_survivor_inverse(k, m, P, erased, e, survivors, Ainv);
    if (rc == 0)
        for (int x = 0; x < e; x++) {
            int r = erased[x];
            for (int c = 0; c < k; c++) {
                if (r < k) R[x * k + c] = Ainv[r * k + c];
                else {
                    uint8_t s = 0;
                    for (int t = 0; t < k; t++) s ^= gso_mul(P[(r - k) * k + t], Ainv[t * k + c]);
                    R[x * k + c] = s;
                }
            }
        }
    free(Ainv);
    return rc;
}

/* Reconstruct (Alg. 2, "KV = EC.reconstruct(KV, P)").  shards[0..k-1] are the
 * data shards, shards[k..k+m-1] the parity shards; the entries named in
 * `erased` are outputs, everything else is read-only.  Per byte offset: solve
 * for all k data bytes from the k lowest-indexed survivors (d = inverse(A)*s),
 * write the lost data bytes, and re-encode any lost parity byte from d. */
int gso_reconstruct(int k, int m, const uint8_t *P, uint8_t *const *shards,
                    const int *erased, int e, size_t S)
{
    gso_init();
    if (e == 0) return 0;
    int survivors[256];
    uint8_t *Ainv = (uint8_t *)malloc((size_t)k * k);
    uint8_t *d = (uint8_t *)malloc((size_t)k);
    if (!Ainv || !d) { free(Ainv); free(d); return -2; }
    int rc = gso_survivor_inverse(k, m, P, erased, e, survivors, Ainv);
    if (rc == 0)
        for (size_t t = 0; t < S; t++) {
            for (int r = 0; r < k; r++) {
                uint8_t s = 0;
                for (int c = 0; c < k; c++) s ^= gso_mul(Ainv[r * k + c], shards[survivors[c]][t]);
                d[r] = s;
            }
            for (int x = 0; x < e; x++) {
                int r = erased[x];
                if (r < k) shards[r][t] = d[r];
                else {
                    uint8_t s = 0;
                    for (int c = 0; c < k; c++) s ^= gso_mul(P[(r - k) * k + c], d[c]);
                    shards[r][t] = s;
                }
            }
        }
    free(Ainv); free(d);
    return rc;
}

/* ---- the same encode over an even byte-range split on several threads ----
 * Used only to time the oracle on all host cores; each thread runs gso_encode
 * unchanged on its own byte range. */
struct gso_job {
    int k, m; const uint8_t *P;
    const uint8_t *const *data; uint8_t *const *parity;
    size_t lo, hi;
};

static void *gso_worker(void *arg)
{
    struct gso_job *j = (struct gso_job *)arg;
    const uint8_t *d[256]; uint8_t *p[256];
    for (int x = 0; x < j->k; x++) d[x] = j->data[x] + j->lo;
    for (int x = 0; x < j->m; x++) p[x] = j->parity[x] + j->lo;
    gso_encode(j->k, j->m, j->P, d, p, j->hi - j->lo);
    return NULL;
}

int gso_encode_mt(int k, int m, const uint8_t *P,
                  const uint8_t *const *data, uint8_t *const *parity, size_t S, int nthreads)
{
    gso_init();
    if (nthreads < 1) nthreads = 1;
    if (nthreads > 256) nthreads = 256;
    pthread_t th[256]; struct gso_job jobs[256];
    size_t per = (S + (size_t)nthreads - 1) / (size_t)nthreads;
    int started = 0;
    for (int t = 0; t < nthreads; t++) { /* every byte range first: the inline fallback below needs them all */
        size_t lo = (size_t)t * per, hi = lo + per;
        if (lo > S) lo = S;
        if (hi > S) hi = S;
        jobs[t] = (struct gso_job){k, m, P, data, parity, lo, hi};
    }
    for (int t = 0; t < nthreads; t++) {
        if (pthread_create(&th[t], NULL, gso_worker, &jobs[t]) != 0) break;
        started++;
    }
    for (int t = 0; t < started; t++) pthread_join(th[t], NULL);
    /* a thread that could not be started: its range and the later ones are done here, so the result is complete */
    for (int t = started; t < nthreads; t++) gso_worker(&jobs[t]);
    return 0;
}

/* ---- hybrid recovery planner (Alg. 2, get_recompute_units) -----------------
 * The paper names the function but never defines it.  Reading: recompute the
 * first r chunks while the other n-r are restored through a three-stage
 * pipeline (gather survivors, parity H2D, reconstruct); pick the r in [0, n]
 * with the smallest max(recompute(r), restore(n-r)), smallest r on a tie.
 * The oracle evaluates every r with the sums written out term by term. */
struct gso_costs { double base, growth, gather, h2d, reconstruct, startup; };

static double gso_recompute(const struct gso_costs *c, int r)
{
    double t = 0.0;
    for (int i = 0; i < r; i++) t += c->base + c->growth * (double)i;
    return t;
}

static double gso_restore(const struct gso_costs *c, int q)
{
    if (q <= 0) return 0.0;
    double slow = c->gather;
    if (c->h2d > slow) slow = c->h2d;
    if (c->reconstruct > slow) slow = c->reconstruct;
    double once = c->gather + c->h2d + c->reconstruct - slow;
    double t = c->startup + once;
    for (int i = 0; i < q; i++) t += slow;
    return t;
}

int gso_recompute_units(int n, const struct gso_costs *c, double *makespan_out)
{
    int best = 0;
    double best_t = -1.0;
    for (int r = 0; r <= n; r++) {
        double a = gso_recompute(c, r), b = gso_restore(c, n - r);
        double t = a > b ? a : b;
        if (best_t < 0.0 || t < best_t) { best_t = t; best = r; }
    }
    if (makespan_out) *makespan_out = best_t < 0.0 ? 0.0 : best_t;
    return best;
}

/* ---- the power code, an alternative generator -------------------------------
 * P[i][j] = 2^(i*j) (exponent taken mod 255): parity row i is the evaluation
 * of the data polynomial at 2^i.  Row 0 is XOR parity; rows 0 and 1 are the
 * familiar P and Q syndromes.  Every square minor on rows {0,1,2} is of
 * Vandermonde type in the distinct elements 2^j, hence non-zero, so the code
 * is MDS for m <= 3; with four rows it is not (2^(3*85) = 2^(3*0)). */
int gso_power_generator(int k, int m, uint8_t *P)
{
    gso_init();
    if (k < 1 || k > 255 || m < 1 || m > 3) return -1;
    for (int i = 0; i < m; i++)
        for (int j = 0; j < k; j++) P[i * k + j] = g_exp[(i * j) % 255];
    return 0;
}
