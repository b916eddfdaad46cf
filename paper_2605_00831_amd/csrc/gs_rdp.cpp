#include "gs_rdp.h"

#include <algorithm>

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

static int disk_of_shard(int k, int p, int shard) { return shard < k ? shard : (shard == k ? p - 1 : p); }

bool rdp_plan(int k, const int *missing, int n_missing, RdpPlan &plan)
{
    if (k < 1 || k > kRdpMaxPrime - 1 || n_missing < 1 || n_missing > 2) return false;  // RDP rebuilds at most two
    const int p = plan.p = rdp_prime(k), rows = p - 1;
    int lost_disk[2] = {-1, -1};
    for (int x = 0; x < n_missing; ++x) lost_disk[x] = disk_of_shard(k, p, missing[x]);
    auto unknown_of = [&](int disk, int row) {
        for (int x = 0; x < n_missing; ++x)
            if (lost_disk[x] == disk) return x * rows + row;
        return -1;
    };
    // One equation per syndrome: the XOR of the unknown cells it covers equals
    // the syndrome (the known cells are already inside the syndrome).
    struct Eq { uint32_t unk = 0, syn = 0; };
    std::vector<Eq> eqs(2 * rows);
    for (int i = 0; i < rows; ++i) {  // row equations first
        Eq &e = eqs[i];
        e.syn = 1u << i;
        for (int j = 0; j <= p - 1; ++j) {
            const int u = unknown_of(j, i);
            if (u >= 0) e.unk ^= 1u << u;
        }
    }
    for (int d = 0; d < rows; ++d) {  // stored diagonals
        Eq &e = eqs[rows + d];
        e.syn = 1u << (rows + d);
        for (int c = 0; c <= p - 1; ++c) {
            const int r = ((d - c) % p + p) % p;
            if (r == p - 1) continue;
            const int u = unknown_of(c, r);
            if (u >= 0) e.unk ^= 1u << u;
        }
        const int u = unknown_of(p, d);
        if (u >= 0) e.unk ^= 1u << u;
    }
    // Gauss-Jordan over GF(2)
    const int nu = n_missing * rows;
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
                eqs[q].syn ^= eqs[next].syn;
            }
        pivot_eq[u] = static_cast<int>(next++);
    }
    plan.outputs.assign(missing, missing + n_missing);
    plan.syndrome_mask.assign(nu, 0);
    plan.needs_diagonals = false;
    for (int u = 0; u < nu; ++u) {
        plan.syndrome_mask[u] = eqs[pivot_eq[u]].syn;
        if (eqs[pivot_eq[u]].syn >> rows) plan.needs_diagonals = true;
    }
    // disks that are read: every real disk that is not being produced; the
    // diagonal-parity disk only when some diagonal syndrome is used
    for (int j = 0; j < kRdpMaxDisks; ++j) plan.shard_of_disk[j] = -1;
    for (int shard = 0; shard < k + 2; ++shard) {
        const int disk = disk_of_shard(k, p, shard);
        bool produced = false;
        for (int x = 0; x < n_missing; ++x) produced = produced || missing[x] == shard;
        if (produced || (disk == p && !plan.needs_diagonals)) continue;
        plan.shard_of_disk[disk] = shard;
    }
    return true;
}

}  // namespace gs
