#include "gs_rdp.h"

#include <algorithm>
#include <bitset>

namespace gs {

int rdp_prime(int k)
{
    int p = std::max(3, k + 1);
    for (;; ++p) {
        bool prime = true;
        for (int d = 2; d * d <= p; ++d)
            if (p % d == 0) { prime = false; break; }
        if (prime) return p;
    }
}

// Stripe disks: 0..p-2 data (k real, the rest imaginary zeros), p-1 row parity,
// p diagonal parity.  Shard id <-> stripe disk.
static int disk_of_shard(int k, int p, int shard) { return shard < k ? shard : (shard == k ? p - 1 : p); }

RdpPlan rdp_encode_plan(int k)
{
    RdpPlan plan;
    const int p = plan.p = rdp_prime(k), rows = p - 1;
    for (int j = 0; j < k; ++j) plan.inputs.push_back(j);
    plan.outputs = {k, k + 1};
    plan.mask.assign(static_cast<size_t>(k) * rows, 0);
    // data block (i, j) is part of row parity block i, of its own diagonal
    // (i+j) mod p, and -- through row parity block i, which sits on disk p-1 --
    // of diagonal (i+p-1) mod p; diagonal p-1 is not stored
    for (int j = 0; j < k; ++j)
        for (int i = 0; i < rows; ++i) {
            uint32_t m = 1u << i;
            const int d_own = (i + j) % p, d_via_row = (i + p - 1) % p;
            if (d_own != p - 1) m ^= 1u << (rows + d_own);
            if (d_via_row != p - 1) m ^= 1u << (rows + d_via_row);
            plan.mask[static_cast<size_t>(j) * rows + i] = m;
        }
    return plan;
}

bool rdp_decode_plan(int k, const int *lost, int n_lost, RdpPlan &plan)
{
    const int p = plan.p = rdp_prime(k), rows = p - 1;
    constexpr int kMaxKnown = (kRdpMaxPrime + 1) * kRdpMaxRows;
    using Known = std::bitset<kMaxKnown>;
    // variable numbering: unknown u = x*rows + r for block r of lost[x];
    // known block (disk, row) -> disk*rows + row (imaginary disks are zero: dropped)
    int lost_disk[2] = {-1, -1};
    for (int x = 0; x < n_lost; ++x) lost_disk[x] = disk_of_shard(k, p, lost[x]);
    auto unknown_of = [&](int disk, int row) {
        for (int x = 0; x < n_lost; ++x)
            if (lost_disk[x] == disk) return x * rows + row;
        return -1;
    };
    auto real = [&](int disk) { return disk < k || disk >= p - 1; };

    struct Eq { uint32_t unk = 0; Known known; };
    std::vector<Eq> eqs;
    auto add_block = [&](Eq &e, int disk, int row) {
        if (!real(disk)) return;
        const int u = unknown_of(disk, row);
        if (u >= 0) e.unk ^= 1u << u;
        else e.known.flip(static_cast<size_t>(disk) * rows + row);
    };
    for (int i = 0; i < rows; ++i) {  // row equations first: a single lost disk then never needs the diagonals
        Eq e;
        for (int j = 0; j <= p - 1; ++j) add_block(e, j, i);
        eqs.push_back(e);
    }
    for (int d = 0; d < rows; ++d) {  // stored diagonals 0..p-2
        Eq e;
        for (int c = 0; c <= p - 1; ++c) {
            const int r = ((d - c) % p + p) % p;
            if (r != p - 1) add_block(e, c, r);
        }
        add_block(e, p, d);
        eqs.push_back(e);
    }
    // Gauss-Jordan over GF(2) on the unknown columns
    const int nu = n_lost * rows;
    std::vector<int> pivot_eq(nu, -1);
    size_t next = 0;
    for (int u = 0; u < nu; ++u) {
        size_t piv = next;
        while (piv < eqs.size() && !(eqs[piv].unk >> u & 1u)) ++piv;
        if (piv == eqs.size()) return false;
        std::swap(eqs[next], eqs[piv]);
        for (size_t q = 0; q < eqs.size(); ++q)
            if (q != next && (eqs[q].unk >> u & 1u)) {
                eqs[q].unk ^= eqs[next].unk;
                eqs[q].known ^= eqs[next].known;
            }
        pivot_eq[u] = static_cast<int>(next++);
    }
    // collect the disks that are actually read, in shard order
    Known any;
    for (int u = 0; u < nu; ++u) any |= eqs[pivot_eq[u]].known;
    plan.inputs.clear();
    plan.outputs.assign(lost, lost + n_lost);
    for (int shard = 0; shard < k + 2; ++shard) {
        const int disk = disk_of_shard(k, p, shard);
        bool used = false;
        for (int r = 0; r < rows; ++r) used = used || any.test(static_cast<size_t>(disk) * rows + r);
        if (used) plan.inputs.push_back(shard);
    }
    plan.mask.assign(plan.inputs.size() * rows, 0);
    for (size_t s = 0; s < plan.inputs.size(); ++s) {
        const int disk = disk_of_shard(k, p, plan.inputs[s]);
        for (int r = 0; r < rows; ++r)
            for (int u = 0; u < nu; ++u)
                if (eqs[pivot_eq[u]].known.test(static_cast<size_t>(disk) * rows + r))
                    plan.mask[s * rows + r] |= 1u << u;
    }
    return true;
}

}  // namespace gs
