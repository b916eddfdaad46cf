// Row-diagonal parity (RDP): XOR-only double parity.  Host-side planning.
//
// Every RDP operation (encode, any rebuild) is done in two steps on the
// device: (1) accumulate the 2(p-1) syndromes of a stripe from the shards that
// are present -- SR[i], the XOR of row i over disks 0..p-1, and SD[d], the XOR
// of stored diagonal d over disks 0..p-1 plus diagonal-parity cell d -- which
// needs no per-case information beyond which disks are present; (2) form each
// missing cell as the XOR of a set of syndromes.  The plan carries those sets.
#pragma once
#include <cstdint>
#include <vector>

namespace gs {

constexpr int kRdpMaxPrime = 17;                 // k <= 16 data shards
constexpr int kRdpMaxRows = kRdpMaxPrime - 1;
constexpr int kRdpMaxDisks = kRdpMaxPrime + 1;   // stripe disks 0..p

int rdp_prime(int k);  // smallest prime >= max(3, k+1)

struct RdpPlan {
    int p = 0;
    // shard id held by stripe disk j (0..p-2 data, p-1 row parity, p diagonal
    // parity), or -1 if that disk is imaginary, missing, or not needed
    int shard_of_disk[kRdpMaxDisks];
    std::vector<int> outputs;         // shard ids written (1 or 2), in the caller's order
    // for output x and row q, at [x*(p-1)+q]: bit i (< p-1) = SR[i] is part of
    // the cell, bit p-1+d = SD[d] is part of it
    std::vector<uint32_t> syndrome_mask;
    bool needs_diagonals = false;     // some mask uses an SD bit
};

// shard ids: 0..k-1 data, k row parity, k+1 diagonal parity.
// missing: the shards to produce (encode = {k, k+1}); returns false if singular.
bool rdp_plan(int k, const int *missing, int n_missing, RdpPlan &plan);

}  // namespace gs
