// Host-side GF(2^8) arithmetic, matrices and lookup-table construction for the
// HIP erasure-code library.  Field: GF(2)[x]/(x^8+x^4+x^3+x^2+1).
//
// Multiplication is the bitwise shift-and-reduce product; there are no
// logarithm tables anywhere in the library.
#pragma once
#include <cstdint>
#include <vector>

namespace gs {

constexpr unsigned kFieldPoly = 0x11D;

// a*b by shift-and-reduce (Russian-peasant form)
inline uint8_t gf_mul(uint8_t a, uint8_t b)
{
    unsigned acc = 0, aa = a, bb = b;
    while (bb) {
        if (bb & 1u) acc ^= aa;
        bb >>= 1;
        aa <<= 1;
        if (aa & 0x100u) aa ^= kFieldPoly;
    }
    return static_cast<uint8_t>(acc);
}

// a^(2^8-2) by square-and-multiply; 0 maps to 0
inline uint8_t gf_inv(uint8_t a)
{
    uint8_t result = 1, base = a;
    for (unsigned e = 254; e; e >>= 1) {
        if (e & 1u) result = gf_mul(result, base);
        base = gf_mul(base, base);
    }
    return a ? result : 0;
}

using Matrix = std::vector<uint8_t>;  // row-major

// Parity block (m x k) by the normalised Cauchy closed form.
Matrix cauchy_parity_block(int k, int m);
// Parity block (m x k) from the systematic form of the Vandermonde matrix
// over points 0..k+m-1, with the same normalisation.
Matrix vandermonde_parity_block(int k, int m);
// Parity block (m x k) of the power code: P[i][j] = 2^(i*j).  Row 0 and
// column 0 are all ones.  MDS for every k <= 255 only when m <= 3.
Matrix power_parity_block(int k, int m);
// In-place inversion of an n x n matrix by elimination on [A | I].
// Returns false if A is singular.
bool invert_in_place(int n, Matrix &a);

// Split-lookup words for multiplication by the constant c.  A byte x is cut
// into bit fields x[2:0], x[5:3], x[7:6]; since multiplication by c is linear
// over GF(2),  c*x = T0[x & 7] ^ T1[(x >> 3) & 7] ^ T2[x >> 6]  with
//   T0[i] = c*i,  T1[i] = c*(8 i),  T2[i] = c*(64 i).
// Words: {T0[0..3], T0[4..7], T1[0..3], T1[4..7], T2[0..3]}, little-endian
// bytes, i.e. entry i of a table sits in byte (i & 3) of word (i >> 2).
struct CoefWords { uint32_t w[5]; };
CoefWords split_tables(uint8_t c);

// A rebuild matrix has no all-ones row, but when the all-ones parity row is
// among the survivors one of the lost data shards is the XOR of that parity
// with all the other data shards, rebuilt ones included.  In terms of the
// matrix R (rows x k, rows <= 4, k <= 16): some row r0 and some set T of other
// rows satisfy
//     R[r0] = v + sum of R[t], t in T,   with every v[j] zero or one,
// so out[r0] = XOR of the inputs with v[j] = 1, XORed with the outputs of the
// rows in T: one XOR per input byte instead of a table lookup.  The result
// puts r0 first (order: position -> row of R), the inputs with v[j] = 1 first
// (perm: position -> column of R; n_xor of them) and names T by row positions
// (bit p of fold, p >= 1).  The smallest T is taken; found = false if there
// is no such row.
struct XorFold {
    bool found;
    int order[4];
    int perm[16];
    int n_xor;
    uint32_t fold;
};
XorFold find_xor_fold(int rows, int k, const uint8_t *coef, int coef_stride);

}  // namespace gs
