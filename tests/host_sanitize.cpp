// Host-only exercise of the library's field / matrix code under
// AddressSanitizer + UndefinedBehaviorSanitizer (built and run by
// tests/test_host_sanitize.py with g++; no HIP involved).
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../paper_2605_00831_amd/csrc/gs_gf.cpp"
#include "../paper_2605_00831_amd/csrc/gs_plan.cpp"
#include "../paper_2605_00831_amd/csrc/gs_rdp.cpp"

using namespace gs;

static int fail(const char *what, int a, int b)
{
    std::printf("FAIL %s (%d, %d)\n", what, a, b);
    return 1;
}

int main()
{
    // field: inverse and distributivity on every element
    for (int a = 1; a < 256; ++a)
        if (gf_mul(static_cast<uint8_t>(a), gf_inv(static_cast<uint8_t>(a))) != 1) return fail("inverse", a, 0);
    for (int a = 0; a < 256; ++a)
        for (int b = 0; b < 256; ++b)
            if (gf_mul(a, b) != gf_mul(b, a) || gf_mul(a, b ^ 0x5A) != (gf_mul(a, b) ^ gf_mul(a, 0x5A)))
                return fail("axioms", a, b);
    // both generator routes agree, are normalised, and every k x k mix of identity
    // and parity rows taken below is invertible with A * inverse(A) = I
    for (int k = 1; k <= 40; k += 3)
        for (int m = 1; m <= 7; ++m) {
            Matrix c = cauchy_parity_block(k, m), v = vandermonde_parity_block(k, m);
            if (c != v) return fail("routes differ", k, m);
            for (int j = 0; j < k; ++j) if (c[j] != 1) return fail("row 0", k, m);
            for (int i = 0; i < m; ++i) if (c[i * k] != 1) return fail("col 0", k, m);
            const int use = m < k ? m : k;  // replace the first `use` identity rows by parity rows
            Matrix A(static_cast<size_t>(k) * k, 0);
            for (int r = 0; r < k; ++r) {
                if (r < use) for (int col = 0; col < k; ++col) A[r * k + col] = c[r * k + col];
                else A[r * k + r] = 1;
            }
            Matrix Ai = A;
            if (!invert_in_place(k, Ai)) return fail("singular", k, m);
            for (int r = 0; r < k; ++r)
                for (int col = 0; col < k; ++col) {
                    uint8_t s = 0;
                    for (int t = 0; t < k; ++t) s ^= gf_mul(A[r * k + t], Ai[t * k + col]);
                    if (s != (r == col)) return fail("A*Ainv", k, m);
                }
        }
    // extremes of the parameter range
    if (cauchy_parity_block(255, 1).size() != 255 || cauchy_parity_block(1, 255).size() != 255) return fail("extremes", 0, 0);
    Matrix sing = {1, 2, 1, 2};
    if (invert_in_place(2, sing)) return fail("singular not detected", 0, 0);
    // lookup words reproduce the product for every constant and byte
    for (int c = 0; c < 256; ++c) {
        const CoefWords w = split_tables(static_cast<uint8_t>(c));
        for (int x = 0; x < 256; ++x) {
            auto byte = [&](int word, int idx) { return (w.w[word + (idx >> 2)] >> (8 * (idx & 3))) & 0xFFu; };
            const unsigned got = byte(0, x & 7) ^ byte(2, (x >> 3) & 7) ^ byte(4, x >> 6);
            if (got != gf_mul(static_cast<uint8_t>(c), static_cast<uint8_t>(x))) return fail("split tables", c, x);
        }
    }
    // RDP planning for every code width and every one- and two-shard loss: masks stay inside the
    // 2(p-1) syndrome bits, disk ids inside the shard range, and lost shards are never read
    for (int k = 1; k <= 16; ++k) {
        const int n = k + 2;
        for (int a = 0; a < n; ++a)
            for (int b = a; b < n; ++b) {
                const int missing[2] = {a, b};
                const int n_missing = a == b ? 1 : 2;
                RdpPlan plan;
                if (!rdp_plan(k, missing, n_missing, plan)) return fail("rdp plan singular", k, a * 100 + b);
                const int rows = plan.p - 1;
                if (plan.p != rdp_prime(k) || static_cast<int>(plan.outputs.size()) != n_missing) return fail("rdp plan shape", k, a);
                if (static_cast<int>(plan.syndrome_mask.size()) != n_missing * rows) return fail("rdp mask count", k, a);
                for (uint32_t mask : plan.syndrome_mask)
                    if (rows < 16 && (mask >> (2 * rows)) != 0) return fail("rdp mask range", k, a);
                for (int j = 0; j <= plan.p; ++j) {
                    const int sh = plan.shard_of_disk[j];
                    if (sh < -1 || sh >= n || sh == a || sh == b) return fail("rdp disk", k, j);
                }
            }
        const int three[3] = {0, 1, 2};
        RdpPlan plan;
        if (k >= 1 && rdp_plan(k, three, 3, plan)) return fail("rdp accepted three losses", k, 0);
    }
    // planner: the answer is inside [0, n] and its makespan is the smaller of the neighbours'
    for (int n = 0; n <= 40; n += 5) {
        const gs_recovery_costs costs = {0.01 + 0.001 * n, 0.0005, 0.002, 0.004, 0.001, 0.003};
        int r = -1;
        double t = -1.0;
        if (gs_recompute_units(n, &costs, &r, &t) != GS_OK || r < 0 || r > n || !(t >= 0.0)) return fail("planner", n, r);
    }
    // The XOR fold of a rebuild matrix: for every loss of three or four shards of several codes, rebuild
    // matrix from the k lowest survivors, then the plan applied to random bytes the way the kernel applies
    // it (XOR row over the first n_xor permuted inputs, lookup rows, fold) against the plain product.
    {
        unsigned rng = 12345;
        auto next = [&]() { rng = rng * 1664525u + 1013904223u; return static_cast<uint8_t>(rng >> 24); };
        const int shapes[][2] = {{4, 3}, {8, 3}, {6, 4}, {16, 4}, {5, 4}};
        for (const auto &km : shapes) {
            const int k = km[0], m = km[1], n = k + m;
            const Matrix P = cauchy_parity_block(k, m);
            auto g = [&](int row, int col) -> uint8_t { return row < k ? (row == col) : P[(row - k) * k + col]; };
            int with_p0 = 0, found_with_p0 = 0;
            for (unsigned pat = 0; pat < (1u << n); ++pat) {
                const int e = __builtin_popcount(pat);
                if (e < 3 || e > m) continue;
                std::vector<int> lost, surv;
                for (int r = 0; r < n; ++r) {
                    if (pat & (1u << r)) lost.push_back(r);
                    else if (static_cast<int>(surv.size()) < k) surv.push_back(r);
                }
                Matrix A(static_cast<size_t>(k) * k);
                for (int r = 0; r < k; ++r)
                    for (int c = 0; c < k; ++c) A[r * k + c] = g(surv[r], c);
                if (!invert_in_place(k, A)) return fail("survivors singular", k, static_cast<int>(pat));
                Matrix R(static_cast<size_t>(e) * k, 0);
                for (int r = 0; r < e; ++r)
                    for (int c = 0; c < k; ++c)
                        for (int t = 0; t < k; ++t) R[r * k + c] ^= gf_mul(g(lost[r], t), A[t * k + c]);
                const XorFold f = find_xor_fold(e, k, R.data(), k);
                bool data_lost = false, p0_used = false;
                for (int r : lost) data_lost = data_lost || r < k;
                for (int r : surv) p0_used = p0_used || r == k;
                if (data_lost && p0_used) {
                    ++with_p0;
                    found_with_p0 += f.found;
                }
                if (!f.found) continue;
                if (f.n_xor < 0 || f.n_xor > k || (f.fold & 1u) || (f.fold >> e)) return fail("fold plan range", k, static_cast<int>(pat));
                uint8_t x[16], want[4], acc[4] = {0, 0, 0, 0};
                for (int j = 0; j < k; ++j) x[j] = next();
                for (int r = 0; r < e; ++r) {
                    want[r] = 0;
                    for (int j = 0; j < k; ++j) want[r] ^= gf_mul(R[r * k + j], x[j]);
                }
                for (int jj = 0; jj < k; ++jj) {
                    const uint8_t xp = x[f.perm[jj]];
                    if (jj < f.n_xor) acc[0] ^= xp;
                    for (int pos = 1; pos < e; ++pos) acc[pos] ^= gf_mul(R[f.order[pos] * k + f.perm[jj]], xp);
                }
                for (int pos = 1; pos < e; ++pos)
                    if (f.fold & (1u << pos)) acc[0] ^= acc[pos];
                for (int pos = 0; pos < e; ++pos)
                    if (acc[pos] != want[f.order[pos]]) return fail("fold plan result", k, static_cast<int>(pat));
            }
            // whenever the all-ones parity row is used and a data shard is lost there is such a row
            if (with_p0 == 0 || found_with_p0 != with_p0) return fail("fold not found", with_p0, found_with_p0);
        }
        // an encode matrix has its all-ones row found with nothing to fold; a matrix without structure has none
        const Matrix P = cauchy_parity_block(8, 3);
        const XorFold enc = find_xor_fold(3, 8, P.data(), 8);
        if (!enc.found || enc.order[0] != 0 || enc.n_xor != 8 || enc.fold != 0) return fail("encode fold", enc.n_xor, enc.fold);
        const uint8_t none[2 * 3] = {2, 3, 4, 5, 7, 9};
        if (find_xor_fold(2, 3, none, 3).found) return fail("fold in a matrix without one", 0, 0);
    }
    std::printf("OK\n");
    return 0;
}
