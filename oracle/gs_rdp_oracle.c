/*
 * gs_rdp_oracle.c -- plain CPU oracle for Row-Diagonal Parity (RDP), the
 * XOR-only double-parity code that GhostServe offers next to XOR and
 * Reed-Solomon (Section 2 and Section 4.1 of the paper name it and cite
 * Corbett et al., "Row-Diagonal Parity for Double Disk Failure Correction";
 * the geometry below is that publication's, restated).
 *
 * TEST INFRASTRUCTURE, like gs_oracle.c: never linked or imported by the HIP
 * library, shares no code with it.
 *
 * Geometry.  p is a prime > 2.  A stripe has p-1 rows and p+1 "disks":
 *   disks 0 .. p-2   data   (only the first k hold real shards; the others
 *                            are imaginary all-zero disks when k < p-1)
 *   disk  p-1        row parity
 *   disk  p          diagonal parity
 * A disk block ("cell") is B bytes.  As on a disk array, a shard holds many
 * stripes one after the other: stripe s of a shard is the (p-1)*B bytes at
 * offset s*(p-1)*B, and its cell i is row i.  Stripes are independent.  (The
 * paper does not say how its RDP maps the KV bytes to stripes; consecutive
 * stripes of fixed-size cells is this build's reading, and the cell size is a
 * parameter.)  Block (i, j), j <= p-1, lies on diagonal (i+j) mod p; diagonal
 * p-1 is the one diagonal that is not stored.
 *   row parity      R[i] = XOR_{j<=p-2} D[i][j]
 *   diagonal parity Q[d] = XOR of all blocks (i, j), i <= p-2, j <= p-1, with
 *                          (i+j) mod p = d,          for d = 0 .. p-2
 * Reconstruction follows the publication's procedure: a lost diagonal-parity
 * disk is re-encoded; a single lost data/row disk comes from the row
 * equations; two lost disks among 0..p-1 are rebuilt by the diagonal walk
 * (use a diagonal that misses one of the two disks to get a block of the
 * other, then that block's row to get a block of the first, and so on, two
 * chains, each ending at the unstored diagonal).
 *
 * Pins (tests/test_oracle_rdp.py): row parity == numpy XOR; the diagonal
 * parity against two stripes worked by hand from the definition above (p = 3
 * and p = 5, expected bytes written out in the test) and, for every k <= 16,
 * against a definition-direct numpy construction that never calls this file
 * -- a flipped diagonal direction, a row-parity disk left out of the
 * diagonals or another unstored diagonal fails them; generator matrix read
 * out by impulses and checked for rank over GF(2) under every pair of lost
 * disks (independent elimination); exhaustive search for the unique
 * completion on the smallest stripe; round trips over every pair of disks for
 * every k <= 16.  What stays unchecked: that the definition restated above is
 * the cited publication's (it is not available to this build); by the
 * authors' own description (row parity plus diagonal parity over the data and
 * row-parity disks, one diagonal dropped) it is.
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static int is_prime(int n)
{
    if (n < 2) return 0;
    for (int d = 2; d * d <= n; d++)
        if (n % d == 0) return 0;
    return 1;
}

/* smallest prime p >= max(3, k+1): room for k data disks */
int gso_rdp_prime(int k)
{
    int p = k + 1 < 3 ? 3 : k + 1;
    while (!is_prime(p)) p++;
    return p;
}

static void xor_into(uint8_t *dst, const uint8_t *src, size_t n)
{
    for (size_t t = 0; t < n; t++) dst[t] ^= src[t];
}

/* block (row i) of disk j, or NULL for an imaginary zero disk */
static uint8_t *blk(uint8_t *const *disk, int k, int p, size_t B, int i, int j)
{
    if (j < k) return disk[j] + (size_t)i * B;            /* data shard j        */
    if (j < p - 1) return NULL;                           /* imaginary zero disk */
    return disk[k + (j - (p - 1))] + (size_t)i * B;       /* row / diagonal parity */
}

/* one stripe: disk[0..k-1] data, disk[k] row parity, disk[k+1] diagonal parity,
 * each (p-1)*B bytes */
static void encode_stripe(int k, int p, uint8_t *const *disk, size_t B)
{
    memset(disk[k], 0, (size_t)(p - 1) * B);
    memset(disk[k + 1], 0, (size_t)(p - 1) * B);
    for (int i = 0; i < p - 1; i++)
        for (int j = 0; j < k; j++) xor_into(blk(disk, k, p, B, i, p - 1), blk(disk, k, p, B, i, j), B);
    for (int i = 0; i < p - 1; i++)
        for (int j = 0; j <= p - 1; j++) {
            int d = (i + j) % p;
            const uint8_t *b = blk(disk, k, p, B, i, j);
            if (d == p - 1 || b == NULL) continue;
            xor_into(blk(disk, k, p, B, d, p), b, B);
        }
}

/* Shards of S bytes = S / ((p-1)*B) stripes of cells of B bytes.
 * Returns 0, -1 if S is not a whole number of stripes or k is out of range. */
int gso_rdp_encode(int k, uint8_t *const *disk, size_t S, size_t B)
{
    if (k < 1 || k > 254 || B == 0) return -1;
    int p = gso_rdp_prime(k);
    size_t stripe = (size_t)(p - 1) * B;
    if (S % stripe) return -1;
    uint8_t *at[256];
    for (size_t off = 0; off < S; off += stripe) {
        for (int j = 0; j < k + 2; j++) at[j] = disk[j] + off;
        encode_stripe(k, p, at, B);
    }
    return 0;
}

/* recompute block (i, j) from its row: XOR of the other p-1 blocks of row i among disks 0..p-1 */
static void from_row(uint8_t *const *disk, int k, int p, size_t B, int i, int j)
{
    uint8_t *dst = blk(disk, k, p, B, i, j);
    memset(dst, 0, B);
    for (int c = 0; c <= p - 1; c++) {
        const uint8_t *b = blk(disk, k, p, B, i, c);
        if (c != j && b) xor_into(dst, b, B);
    }
}

/* recompute block (i, j) from its diagonal d = (i+j) mod p (d != p-1):
 * diagonal parity block d XOR the other blocks of that diagonal */
static void from_diagonal(uint8_t *const *disk, int k, int p, size_t B, int i, int j)
{
    int d = (i + j) % p;
    uint8_t *dst = blk(disk, k, p, B, i, j);
    memcpy(dst, blk(disk, k, p, B, d, p), B);
    for (int c = 0; c <= p - 1; c++) {
        int r = ((d - c) % p + p) % p;
        if (c == j || r == p - 1) continue;
        const uint8_t *b = blk(disk, k, p, B, r, c);
        if (b) xor_into(dst, b, B);
    }
}

/* one stripe; lost[] holds stripe disk numbers among 0..p-1 */
static void reconstruct_stripe(int k, int p, uint8_t *const *disk, size_t B, const int *lost, int n, int diag_lost)
{
    if (n == 1) {
        for (int i = 0; i < p - 1; i++) from_row(disk, k, p, B, i, lost[0]);
    } else if (n == 2) {
        /* diagonal walk.  Diagonal d has no block on disk (d+1) mod p.  Start each
         * chain on the diagonal that misses one lost disk, alternate diagonal and
         * row steps, stop when the next diagonal is the unstored one. */
        for (int s = 0; s < 2; s++) {
            int a = lost[s], b = lost[1 - s];          /* first diagonal misses disk a */
            int d = ((a - 1) % p + p) % p;
            while (d != p - 1) {
                int i = ((d - b) % p + p) % p;         /* row of diagonal d on disk b */
                from_diagonal(disk, k, p, B, i, b);
                from_row(disk, k, p, B, i, a);
                d = (i + a) % p;                       /* diagonal of the block just rebuilt */
            }
        }
    }
    if (diag_lost) {
        /* re-encode the diagonal parity from the (now complete) stripe */
        memset(disk[k + 1], 0, (size_t)(p - 1) * B);
        for (int i = 0; i < p - 1; i++)
            for (int j = 0; j <= p - 1; j++) {
                int d = (i + j) % p;
                const uint8_t *b = blk(disk, k, p, B, i, j);
                if (d == p - 1 || b == NULL) continue;
                xor_into(blk(disk, k, p, B, d, p), b, B);
            }
    }
}

/* erased: shard indices in [0, k+2) (k = row parity, k+1 = diagonal parity).
 * Returns 0; -1 bad arguments; -3 more than two erasures. */
int gso_rdp_reconstruct(int k, uint8_t *const *disk, const int *erased, int e, size_t S, size_t B)
{
    if (k < 1 || k > 254 || e < 0 || B == 0) return -1;
    int p = gso_rdp_prime(k);
    size_t stripe = (size_t)(p - 1) * B;
    if (S % stripe) return -1;
    int lost[2] = {-1, -1}, n = 0, diag_lost = 0;
    for (int x = 0; x < e; x++) {
        if (erased[x] < 0 || erased[x] > k + 1) return -1;
        for (int y = 0; y < x; y++)
            if (erased[y] == erased[x]) return -1;
    }
    if (e > 2) return -3;
    for (int x = 0; x < e; x++) {
        if (erased[x] == k + 1) diag_lost = 1;
        else lost[n++] = erased[x] < k ? erased[x] : p - 1;   /* stripe disk number */
    }
    uint8_t *at[256];
    for (size_t off = 0; off < S; off += stripe) {
        for (int j = 0; j < k + 2; j++) at[j] = disk[j] + off;
        reconstruct_stripe(k, p, at, B, lost, n, diag_lost);
    }
    return 0;
}
