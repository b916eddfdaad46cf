#include "gs_gf.h"

namespace gs {

static uint8_t gf_div(uint8_t a, uint8_t b) { return gf_mul(a, gf_inv(b)); }

// Scale columns so row 0 is all ones, then rows so column 0 is all ones.
static void normalise(int k, int m, Matrix &p)
{
    for (int j = 0; j < k; ++j) {
        const uint8_t s = gf_inv(p[j]);
        for (int i = 0; i < m; ++i) p[i * k + j] = gf_mul(p[i * k + j], s);
    }
    for (int i = 0; i < m; ++i) {
        const uint8_t s = gf_inv(p[i * k]);
        for (int j = 0; j < k; ++j) p[i * k + j] = gf_mul(p[i * k + j], s);
    }
}

Matrix cauchy_parity_block(int k, int m)
{
    // 1/(x_i + y_j) with x_i = k+i, y_j = j; x and y ranges are disjoint, so no
    // denominator vanishes.  Any square minor of a Cauchy matrix is non-zero,
    // and scaling rows and columns keeps that, so [I;P] is MDS.
    Matrix p(static_cast<size_t>(m) * k);
    for (int i = 0; i < m; ++i)
        for (int j = 0; j < k; ++j)
            p[i * k + j] = gf_inv(static_cast<uint8_t>((k + i) ^ j));
    normalise(k, m, p);
    return p;
}

Matrix vandermonde_parity_block(int k, int m)
{
    // Row of the systematic generator for evaluation point x (a parity point)
    // is the vector of Lagrange basis values L_j(x) over the data points
    // y_0..y_{k-1}:  L_j(x) = prod_{l != j} (x - y_l) / (y_j - y_l).
    Matrix p(static_cast<size_t>(m) * k);
    for (int i = 0; i < m; ++i) {
        const uint8_t x = static_cast<uint8_t>(k + i);
        for (int j = 0; j < k; ++j) {
            uint8_t num = 1, den = 1;
            for (int l = 0; l < k; ++l) {
                if (l == j) continue;
                num = gf_mul(num, static_cast<uint8_t>(x ^ l));
                den = gf_mul(den, static_cast<uint8_t>(j ^ l));
            }
            p[i * k + j] = gf_div(num, den);
        }
    }
    normalise(k, m, p);
    return p;
}

Matrix power_parity_block(int k, int m)
{
    // row i holds the powers of g_i = 2^i: 1, g_i, g_i^2, ...
    Matrix p(static_cast<size_t>(m) * k);
    uint8_t g = 1;  // 2^i
    for (int i = 0; i < m; ++i) {
        uint8_t v = 1;
        for (int j = 0; j < k; ++j) {
            p[i * k + j] = v;
            v = gf_mul(v, g);
        }
        g = gf_mul(g, 2);
    }
    return p;
}

// full product table for the matrix routines, filled once from the bitwise multiply
struct ProductTable {
    uint8_t v[256][256];
    ProductTable()
    {
        for (int a = 0; a < 256; ++a)
            for (int b = 0; b < 256; ++b) v[a][b] = gf_mul(static_cast<uint8_t>(a), static_cast<uint8_t>(b));
    }
};

static const ProductTable &products()
{
    static const ProductTable t;
    return t;
}

bool invert_in_place(int n, Matrix &a)
{
    const ProductTable &pt = products();
    // augmented elimination: w = [A | I], n x 2n
    const int w2 = 2 * n;
    Matrix w(static_cast<size_t>(n) * w2, 0);
    for (int r = 0; r < n; ++r) {
        for (int c = 0; c < n; ++c) w[r * w2 + c] = a[r * n + c];
        w[r * w2 + n + r] = 1;
    }
    for (int col = 0; col < n; ++col) {
        int piv = col;
        while (piv < n && w[piv * w2 + col] == 0) ++piv;
        if (piv == n) return false;
        if (piv != col)
            for (int c = 0; c < w2; ++c) { uint8_t t = w[col * w2 + c]; w[col * w2 + c] = w[piv * w2 + c]; w[piv * w2 + c] = t; }
        const uint8_t s = gf_inv(w[col * w2 + col]);
        if (s != 1)
            for (int c = col; c < w2; ++c) w[col * w2 + c] = pt.v[s][w[col * w2 + c]];
        for (int r = 0; r < n; ++r) {
            const uint8_t f = w[r * w2 + col];
            if (r == col || f == 0) continue;
            for (int c = col; c < w2; ++c) w[r * w2 + c] ^= pt.v[f][w[col * w2 + c]];
        }
    }
    for (int r = 0; r < n; ++r)
        for (int c = 0; c < n; ++c) a[r * n + c] = w[r * w2 + n + c];
    return true;
}

CoefWords split_tables(uint8_t c)
{
    CoefWords t{};
    for (unsigned i = 0; i < 8; ++i) {
        t.w[0 + (i >> 2)] |= static_cast<uint32_t>(gf_mul(c, static_cast<uint8_t>(i))) << (8 * (i & 3));
        t.w[2 + (i >> 2)] |= static_cast<uint32_t>(gf_mul(c, static_cast<uint8_t>(i << 3))) << (8 * (i & 3));
    }
    for (unsigned i = 0; i < 4; ++i)
        t.w[4] |= static_cast<uint32_t>(gf_mul(c, static_cast<uint8_t>(i << 6))) << (8 * i);
    return t;
}

XorFold find_xor_fold(int rows, int k, const uint8_t *coef, int coef_stride)
{
    XorFold best;
    best.found = false;
    best.n_xor = 0;
    best.fold = 0;
    for (int r = 0; r < 4; ++r) best.order[r] = r;
    for (int j = 0; j < 16; ++j) best.perm[j] = j;
    if (rows < 1 || rows > 4 || k < 1 || k > 16) return best;
    int best_size = rows + 1;
    for (int r0 = 0; r0 < rows; ++r0)
        for (uint32_t T = 0; T < (1u << rows); ++T) {
            if (T & (1u << r0)) continue;
            const int size = __builtin_popcount(T);
            if (size >= best_size) continue;
            uint8_t v[16];
            bool zero_one = true;
            for (int j = 0; j < k && zero_one; ++j) {
                v[j] = coef[r0 * coef_stride + j];
                for (int t = 0; t < rows; ++t)
                    if (T & (1u << t)) v[j] ^= coef[t * coef_stride + j];
                zero_one = v[j] <= 1;
            }
            if (!zero_one) continue;
            best.found = true;
            best_size = size;
            best.order[0] = r0;
            best.fold = 0;
            int pos = 1;
            for (int r = 0; r < rows; ++r)
                if (r != r0) {
                    if (T & (1u << r)) best.fold |= 1u << pos;
                    best.order[pos++] = r;
                }
            int n = 0;
            for (int j = 0; j < k; ++j)
                if (v[j] == 1) best.perm[n++] = j;
            best.n_xor = n;
            for (int j = 0; j < k; ++j)
                if (v[j] == 0) best.perm[n++] = j;
        }
    return best;
}

}  // namespace gs
