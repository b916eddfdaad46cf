// Row-diagonal parity (RDP): XOR-only double parity.  Host-side planning:
// which surviving blocks each output block is the XOR of.
#pragma once
#include <cstdint>
#include <vector>

namespace gs {

constexpr int kRdpMaxPrime = 17;                       // k <= 16 data shards
constexpr int kRdpMaxRows = kRdpMaxPrime - 1;
constexpr int kRdpMaxInputs = kRdpMaxPrime + 1;        // shards read by one launch

int rdp_prime(int k);  // smallest prime >= max(3, k+1)

// A plan: `inputs` are the shard ids that are read; `outputs` the shard ids
// that are written (1 or 2); mask[s*(p-1)+row] has bit (x*(p-1)+r) set when
// block `row` of inputs[s] is part of the XOR that gives block r of outputs[x].
struct RdpPlan {
    int p = 0;
    std::vector<int> inputs, outputs;
    std::vector<uint32_t> mask;
};

// shard ids: 0..k-1 data, k row parity, k+1 diagonal parity
RdpPlan rdp_encode_plan(int k);
// lost: 1 or 2 distinct shard ids; returns false if the system is singular
bool rdp_decode_plan(int k, const int *lost, int n_lost, RdpPlan &plan);

}  // namespace gs
