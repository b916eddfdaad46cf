"""GPU parity at the largest sizes one MI355X holds: a one-million-token context of the
8B-shaped KV cache (4 shards of 32 GiB + 2 parity shards = 192 GiB resident, the upper end of
the paper's long-context scaling experiment, Section 6.4), and shards of 44 GiB, past the point
where one workgroup takes several tiles.

Nothing of this size can be cloned or shipped to the host, so the checks are
  - seeded windows (shard ends, both sides of every 4 GiB multiple that fits, random offsets
    with odd lengths) byte for byte against the oracle on the same bytes copied to the host;
  - the XOR-fold invariant over the whole buffers (fold of parity == oracle encode of the folds);
  - rebuild: 64-bit word sums and XOR folds of the lost shards, taken before they are wiped,
    must come back exactly, as must their windows.
"""
import numpy as np
import pytest

import oracle
from paper_2605_00831_amd import inputs

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

FOLD = 4096
GiB = 1 << 30


@pytest.fixture(scope="module")
def gs():
    from paper_2605_00831_amd import binding
    binding.lib()
    binding.gs_set_launch_shape()
    return binding


def xor_fold(t, piece=2 * GiB):
    """XOR of all FOLD-byte blocks of a uint8 device tensor, piece by piece (little extra memory)."""
    acc = torch.zeros(FOLD // 8, dtype=torch.int64, device=t.device)
    for off in range(0, t.numel(), piece):
        x = t[off:off + piece].view(torch.int64).reshape(-1, FOLD // 8)
        while x.shape[0] > 1:
            n = x.shape[0]
            if n % 2:
                acc ^= x[n - 1]
                x = x[:n - 1]
                n -= 1
            x = x[: n // 2] ^ x[n // 2:]
        acc ^= x[0]
    return acc.view(torch.uint8).cpu().numpy()


def word_sum(t, piece=4 * GiB):
    """sum of the shard's 64-bit words modulo 2^64"""
    s = 0
    for off in range(0, t.numel(), piece):
        s = (s + int(t[off:off + piece].view(torch.int64).sum().item())) & ((1 << 64) - 1)
    return s


def windows(S, seed):
    rng = np.random.default_rng(seed)
    w = [(0, 65536 + 7), (S - 65536 - 3, 65536 + 3)]
    for mult in range(4 * GiB, S, 4 * GiB):
        w.append((mult - 4099, 8200))
    for _ in range(6):
        n = int(rng.integers(1, 100000))
        w.append((int(rng.integers(0, S - n)), n))
    return w


def fill(buf, seed):
    """bf16 N(0,1) bytes, generated on the device in 1 GiB pieces"""
    g = torch.Generator(device="cuda").manual_seed(seed)
    for off in range(0, buf.numel(), GiB):
        n = min(GiB, buf.numel() - off)
        buf[off:off + n].view(torch.bfloat16).copy_(torch.randn(n // 2, generator=g, device="cuda", dtype=torch.float32))


def run(gs, k, m, S, lost, seed):
    torch.cuda.empty_cache()  # earlier tests' blocks would otherwise count as in use
    free, _ = torch.cuda.mem_get_info()
    need = (k + m) * S + 24 * GiB
    if free < need:
        pytest.skip("needs %.0f GiB of free device memory" % (need / 2**30))
    shards = [torch.empty(S, dtype=torch.uint8, device="cuda") for _ in range(k + m)]
    for j in range(k):
        fill(shards[j], seed + j)
    for i in range(m):
        shards[k + i].fill_(0xEE)
    data, parity = shards[:k], shards[k:]
    code = gs.gs_make_code(k, m)
    P = oracle.generator(k, m)
    gs.gs_encode(code, data, parity, S)
    torch.cuda.synchronize()
    win = windows(S, seed)
    for off, n in win:
        host = [np.ascontiguousarray(d[off:off + n].cpu().numpy()) for d in data]
        want = oracle.encode(P, host, nthreads=8)
        for i in range(m):
            assert np.array_equal(parity[i][off:off + n].cpu().numpy(), want[i]), (i, off, n)
    folds = [np.ascontiguousarray(xor_fold(d)) for d in data]
    want = oracle.encode(P, folds)
    pfolds = [xor_fold(p) for p in parity]
    for i in range(m):
        assert np.array_equal(pfolds[i], want[i]), "fold of parity %d differs" % i
    # lose shards: remember their digests and windows, wipe, rebuild in place, compare
    allfolds = folds + pfolds
    sums = {r: word_sum(shards[r]) for r in lost}
    keep = {r: [shards[r][off:off + n].clone() for off, n in win] for r in lost}
    for r in lost:
        shards[r].fill_(0xA5)
    gs.gs_reconstruct(code, shards, lost, S)
    torch.cuda.synchronize()
    for r in lost:
        assert word_sum(shards[r]) == sums[r], "word sum of shard %d differs" % r
        assert np.array_equal(xor_fold(shards[r]), allfolds[r]), "fold of shard %d differs" % r
        for (off, n), orig in zip(win, keep[r]):
            assert torch.equal(shards[r][off:off + n], orig), (r, off, n)
    del shards, data, parity, keep
    torch.cuda.empty_cache()


def test_one_million_token_context_of_the_8b_shape(gs):
    """1,048,576 tokens x 128 KiB = 128 GiB of KV in 4 shards of 32 GiB, m = 2."""
    run(gs, 4, 2, 32 * GiB, [1, 3], 0x67531000)


def test_shards_of_44_gib(gs):
    """k = 4, m = 1: shard offsets beyond 2^35 and more tiles than one launch has workgroups for."""
    run(gs, 4, 1, 44 * GiB, [2], 0x67532000)


def test_rdp_shards_of_34_gib(gs):
    """RDP with k = 2 (p = 3, stripes of two 32 KiB cells): shards of 34 GiB need more workgroups than one
    grid row holds.  Row parity must equal the XOR of the data shards over the whole buffers (its
    definition, computed with torch); sampled runs of whole stripes (both ends, both sides of every
    4 GiB multiple, seeded random ones) go through the RDP oracle; both data shards are then lost and
    must come back with the same digests and windows."""
    k, cell = 2, 32768
    S = 34 * GiB
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    if free < 4 * S + 24 * GiB:
        pytest.skip("needs %.0f GiB of free device memory" % ((4 * S + 24 * GiB) / 2**30))
    code = gs.gs_make_rdp_code(k, cell)
    stripe = (gs.gs_rdp_prime(code) - 1) * cell
    assert stripe == 2 * cell and S % stripe == 0
    shards = [torch.empty(S, dtype=torch.uint8, device="cuda") for _ in range(4)]
    for j in range(k):
        fill(shards[j], 0x67533000 + j)
    for t in shards[k:]:
        t.fill_(0xEE)
    gs.gs_encode(code, shards[:k], shards[k:], S)
    torch.cuda.synchronize()
    for off in range(0, S, 2 * GiB):
        a, b, p = (t[off:off + 2 * GiB].view(torch.int64) for t in (shards[0], shards[1], shards[2]))
        assert torch.equal(a ^ b, p), "row parity differs in the piece at %d" % off
    rng = np.random.default_rng(0x67533010)
    n_stripes = S // stripe
    first = [0, n_stripes - 3] + [mult // stripe - 1 for mult in range(4 * GiB, S, 4 * GiB)] + \
            [int(x) for x in rng.integers(0, n_stripes - 3, size=6)]
    win = [(s * stripe, 3 * stripe) for s in first]
    for off, n in win:
        host = [np.ascontiguousarray(t[off:off + n].cpu().numpy()) for t in shards[:k]]
        want = oracle.rdp_encode(host, cell)
        for i in range(2):
            assert np.array_equal(shards[k + i][off:off + n].cpu().numpy(), want[i]), (i, off)
    lost = [0, 1]
    sums = {r: word_sum(shards[r]) for r in lost}
    folds = {r: xor_fold(shards[r]) for r in lost}
    keep = {r: [shards[r][off:off + n].clone() for off, n in win] for r in lost}
    for r in lost:
        shards[r].fill_(0xA5)
    gs.gs_reconstruct(code, shards, lost, S)
    torch.cuda.synchronize()
    for r in lost:
        assert word_sum(shards[r]) == sums[r], "word sum of shard %d differs" % r
        assert np.array_equal(xor_fold(shards[r]), folds[r]), "fold of shard %d differs" % r
        for (off, n), orig in zip(win, keep[r]):
            assert torch.equal(shards[r][off:off + n], orig), (r, off)
    del shards, keep
    torch.cuda.empty_cache()
