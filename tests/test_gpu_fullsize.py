"""GPU parity at the full sizes of the measured workloads, in the launch
configuration bench.py times (default launch shape, one launch per call).

These tests check
  - every parity byte of the 32 GiB and 40 GiB workloads against the oracle,
    streamed through the host in 256 MiB pieces (about 15 s per workload on
    16 host threads);
  - sampled windows (shard starts and ends, both sides of the 4 GiB offset,
    seeded random offsets with odd lengths) byte for byte against the oracle
    on the same bytes copied to the host;
  - the XOR-fold invariant over the WHOLE buffers: folding a shard to a 4 KiB
    block by XOR commutes with the code, so oracle.encode(folds of data) must
    equal the folds of the GPU parity (folds computed with torch ops, which
    share nothing with the kernels);
  - reconstruct at full size: rebuilt shards equal the originals bit for bit.
"""
import numpy as np
import pytest

import oracle
from paper_2605_00831_amd import inputs

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

FOLD = 4096


@pytest.fixture(scope="module")
def gs():
    from paper_2605_00831_amd import binding
    binding.lib()
    binding.gs_set_launch_shape()
    return binding


def xor_fold(t):
    """XOR of all FOLD-byte blocks of a uint8 device tensor (length a multiple
    of FOLD and a power-of-two number of blocks times an odd factor)."""
    x = t.view(torch.int64).reshape(-1, FOLD // 8)
    while x.shape[0] > 1:
        n = x.shape[0]
        if n % 2:
            x = torch.cat([x[:1] ^ x[n - 1:], x[1:n - 1]])
            n -= 1
        x = x[: n // 2] ^ x[n // 2:]
    return x.reshape(-1).view(torch.uint8).cpu().numpy()


def windows(S, seed, count=6):
    """(offset, length) pairs inside [0, S)"""
    rng = np.random.default_rng(seed)
    w = [(0, 65536 + 7), (S - 65536 - 3, 65536 + 3)]
    if S > (1 << 32):
        w += [((1 << 32) - 4099, 8200), ((1 << 32), 4096 + 5)]
    if S > (1 << 31):
        w += [((1 << 31) - 33, 70)]
    for _ in range(count):
        n = int(rng.integers(1, 200000))
        w.append((int(rng.integers(0, S - n)), n))
    return w


def check_windows(P, data, parity, S, seed):
    k, m = P.shape[1], P.shape[0]
    for off, n in windows(S, seed):
        host = [np.ascontiguousarray(d[off:off + n].cpu().numpy()) for d in data]
        want = oracle.encode(P, host, nthreads=8)
        for i in range(m):
            got = parity[i][off:off + n].cpu().numpy()
            assert np.array_equal(got, want[i]), "parity %d differs in window at %d (+%d)" % (i, off, n)


def check_folds(P, data, parity):
    folds = [np.ascontiguousarray(xor_fold(d)) for d in data]
    want = oracle.encode(P, folds)
    for i in range(P.shape[0]):
        assert np.array_equal(xor_fold(parity[i]), want[i]), "fold of parity %d differs" % i


def check_every_byte(P, data, parity, S, piece=256 << 20):
    """The whole parity against the oracle, piece by piece: the data piece goes to the host,
    the oracle encodes it on the host cores, the result must equal the GPU's parity piece."""
    m = P.shape[0]
    for off in range(0, S, piece):
        n = min(piece, S - off)
        host = [np.ascontiguousarray(d[off:off + n].cpu().numpy()) for d in data]
        want = oracle.encode(P, host, nthreads=16)
        for i in range(m):
            got = parity[i][off:off + n].cpu().numpy()
            assert np.array_equal(got, want[i]), "parity %d differs in the piece at %d" % (i, off)


def run_bulk(gs, name):
    cfg = inputs.CONFIGS[name]
    k, m = cfg["k"], cfg["m"]
    total = inputs.config_total_bytes(name)
    S = total // k
    free, _ = torch.cuda.mem_get_info()
    need = total + m * S + 2 * S + (4 << 30)
    if free < need:
        pytest.skip("needs %.0f GiB of free device memory" % (need / 2**30))
    buf = inputs.kv_bytes_device(inputs.config_seed(name), total, cfg["dtype"], cfg["sigma"], "cuda")
    data = [buf[j * S:(j + 1) * S] for j in range(k)]
    parity = [torch.full((S,), 0xEE, dtype=torch.uint8, device="cuda") for _ in range(m)]
    code = gs.gs_make_code(k, m)
    P = oracle.generator(k, m)
    assert np.array_equal(gs.gs_code_matrix(code), P)
    gs.gs_encode(code, data, parity, S)
    torch.cuda.synchronize()
    check_windows(P, data, parity, S, inputs.config_seed(name))
    check_folds(P, data, parity)
    check_every_byte(P, data, parity, S)
    # lose two data shards (failure = flushed buffers), rebuild in place, compare
    lost = [1, k - 1]
    keep = [data[r].clone() for r in lost]
    for r in lost:
        data[r].fill_(0xA5)
    gs.gs_reconstruct(code, data + parity, lost, S)
    torch.cuda.synchronize()
    for r, orig in zip(lost, keep):
        assert torch.equal(data[r], orig), "shard %d not rebuilt bit for bit" % r
    del keep
    # lose a data shard and a parity shard
    lost = [0, k + 1]
    keep = [data[0].clone(), parity[1].clone()]
    data[0].fill_(0xA5)
    parity[1].fill_(0xA5)
    gs.gs_reconstruct(code, data + parity, lost, S)
    torch.cuda.synchronize()
    assert torch.equal(data[0], keep[0]) and torch.equal(parity[1], keep[1])


def test_llama8b_prefill_full_size(gs):
    """32 GiB bf16 N(0, 0.5), k=4 shards of 8 GiB (offsets beyond 2^32), m=2."""
    run_bulk(gs, "llama8b_prefill")


def test_llama70b_longctx_full_size(gs):
    """40 GiB bf16 N(0, 1), k=8 shards of 5 GiB, m=2."""
    run_bulk(gs, "llama70b_longctx")


def test_recovery_stress_full_size_20_seeded_patterns(gs):
    """k=8, m=3, S=512 MiB: shards 0-3 uniform bytes, shards 4-7 bf16 KV held
    in 32 KiB pages (16-token blocks) behind a permutation table and gathered
    to contiguous survivors; parity lives in pinned host memory and comes back
    H2D through the restore pipeline; 20 seeded erasure triples."""
    c = inputs.CONFIGS["recovery_stress"]
    k, m, S = c["k"], c["m"], c["shard_bytes"]
    seed = inputs.config_seed("recovery_stress")
    page = 32768
    pages = S // page
    data = [inputs.uniform_bytes_device(seed + j, S, "cuda") for j in range(4)]
    pool = inputs.kv_bytes_device(seed + 7, 4 * S, "bf16", 1.0, "cuda").view(4 * pages, page)
    table = torch.from_numpy(inputs.block_table_np(seed, 4, pages, 4 * pages)).cuda()
    data += [pool[table[j].long()].reshape(-1).contiguous() for j in range(4)]
    P = oracle.generator(k, m)
    code = gs.gs_make_code(k, m)
    parity = [torch.empty(S, dtype=torch.uint8, device="cuda") for _ in range(m)]
    gs.gs_encode(code, data, parity, S)
    torch.cuda.synchronize()
    check_windows(P, data, parity, S, seed)
    check_folds(P, data, parity)
    # the same parity through the paged entry: shards 4-7 straight from the pool
    # (k=4 sub-code check: paged encode of the KV shards equals contiguous encode of their gathers)
    code4 = gs.gs_make_code(4, 2)
    base = torch.tensor([pool.data_ptr()], dtype=torch.int64, device="cuda")
    pp = [torch.empty(S, dtype=torch.uint8, device="cuda") for _ in range(2)]
    pc = [torch.empty(S, dtype=torch.uint8, device="cuda") for _ in range(2)]
    gs.gs_encode_paged(code4, base, 1, page, 4 * pages, table, pages, pp)
    gs.gs_encode(code4, data[4:], pc, S)
    torch.cuda.synchronize()
    assert torch.equal(pp[0], pc[0]) and torch.equal(pp[1], pc[1])
    check_windows(oracle.generator(4, 2), data[4:], pp, S, seed + 1)
    del pp, pc
    # parity goes to pinned host memory; device copies are dropped
    host = [torch.empty(S, dtype=torch.uint8, pin_memory=True) for _ in range(m)]
    for i in range(m):
        host[i].copy_(parity[i])
    torch.cuda.synchronize()
    full = data + parity
    pipe = gs.gs_pipe_create(code, 64 << 20, 2)
    pats = inputs.random_erasure_patterns(seed, k + m, 3, c["patterns_full"])
    assert len(pats) == 20
    for pat in pats:
        work = []
        for r in range(k + m):
            if r in pat:
                work.append(torch.full((S,), 0xA5, dtype=torch.uint8, device="cuda"))
            elif r < k:
                work.append(full[r])
            else:
                work.append(None)          # surviving parity is only in host memory
        gs.gs_restore(pipe, work, host, list(pat), S)
        gs.gs_pipe_sync(pipe)
        torch.cuda.synchronize()
        for r in pat:
            assert torch.equal(work[r], full[r]), (pat, r)
        del work
    # one pattern also through the plain entry with parity resident
    pat = pats[0]
    work = [torch.full((S,), 0xA5, dtype=torch.uint8, device="cuda") if r in pat else full[r] for r in range(k + m)]
    gs.gs_reconstruct(code, work, list(pat), S)
    torch.cuda.synchronize()
    for r in pat:
        assert torch.equal(work[r], full[r])
    gs.gs_pipe_destroy(pipe)


def test_recovery_stress_full_size_through_the_paged_pipelines(gs):
    """The recovery-stress stripe (k=8, m=3, shards of 512 MiB) living in a paged pool of 64 planes
    with 32 KiB pages (16-token blocks): shards 0-3 are uniform random bytes in consecutive pages,
    shards 4-7 bf16 N(0,1) KV pages behind a seeded permutation.  gs_checkpoint_paged ships the
    parity to pinned host memory; for 20 seeded erasure triples the lost shards' pages are flushed
    and gs_restore_paged rebuilds them in place with parity coming back from the host."""
    c = inputs.CONFIGS["recovery_stress"]
    k, m, S = c["k"], c["m"], c["shard_bytes"]
    seed = inputs.config_seed("recovery_stress")
    n_planes, page = 64, 32768
    pps = S // (n_planes * page)                    # 256 slots per shard and plane
    ppp = k * pps                                   # 2048 pages = 64 MiB per plane
    half = 4 * pps * page                           # bytes per plane that belong to shards 0-3
    pool = torch.empty(n_planes, ppp * page, dtype=torch.uint8, device="cuda")
    pool[:, :half] = inputs.uniform_bytes_device(seed, n_planes * half, "cuda").view(n_planes, half)
    pool[:, half:] = inputs.kv_bytes_device(seed + 7, n_planes * half, "bf16", 1.0, "cuda").view(n_planes, half)
    table_np = np.concatenate([np.arange(4 * pps, dtype=np.int32).reshape(4, pps),
                               4 * pps + inputs.block_table_np(seed, 4, pps, 4 * pps)])
    table = torch.from_numpy(np.ascontiguousarray(table_np)).cuda()
    base = torch.tensor([pool.data_ptr() + p * ppp * page for p in range(n_planes)], dtype=torch.int64, device="cuda")
    pages = pool.view(n_planes, ppp, page)

    def gathered(j):   # shard j's logical byte stream, [plane][slot][page]
        return pages[:, table[j].long()].reshape(-1).contiguous()

    P = oracle.generator(k, m)
    code = gs.gs_make_code(k, m)
    host = [torch.empty(S, dtype=torch.uint8, pin_memory=True) for _ in range(m)]
    pipe = gs.gs_pipe_create(code, 64 << 20, 2)     # 32 slots of every plane per chunk, 8 chunks
    gs.gs_checkpoint_paged(pipe, base, n_planes, page, ppp, table, pps, host)
    gs.gs_pipe_sync(pipe)
    data = [gathered(j) for j in range(k)]
    parity = [h.cuda() for h in host]
    check_windows(P, data, parity, S, seed + 3)
    check_folds(P, data, parity)
    # one gs_encode_paged call over the whole table gives the same parity
    whole = [torch.empty(S, dtype=torch.uint8, device="cuda") for _ in range(m)]
    gs.gs_encode_paged(code, base, n_planes, page, ppp, table, pps, whole)
    torch.cuda.synchronize()
    for i in range(m):
        assert torch.equal(whole[i], parity[i])
    del whole, data
    original = pool.clone()
    pats = inputs.random_erasure_patterns(seed, k + m, 3, c["patterns_full"])
    assert len(pats) == 20
    out = [torch.empty(S, dtype=torch.uint8, device="cuda") for _ in range(m)]
    for pat in pats:
        for r in pat:
            if r < k:
                pages[:, table[r].long()] = 0xA5    # the failed worker's buffers are flushed
            else:
                out[r - k].fill_(0xA5)
        gs.gs_restore_paged(pipe, base, n_planes, page, ppp, table, pps, host, list(pat), parity_out=out)
        gs.gs_pipe_sync(pipe)
        torch.cuda.synchronize()
        assert torch.equal(pool, original), pat
        for r in pat:
            if r >= k:
                assert torch.equal(out[r - k], parity[r - k]), (pat, r)
    gs.gs_pipe_destroy(pipe)


@pytest.mark.parametrize("kind", ["cauchy", "rdp"])
def test_paged_pool_with_a_plane_larger_than_4_gib(gs, kind):
    """Page ids whose byte offset inside the plane is beyond 2^32: one plane of 6 GiB in 32 KiB pages, the
    shards' pages drawn from all of it (most of them above 4 GiB), parity from gs_encode_paged and from
    the paged checkpoint pipeline, a lost shard rebuilt into fresh pages above 4 GiB.  The oracle sees
    only the pages the table names, copied to the host and renumbered."""
    free, _ = torch.cuda.mem_get_info()
    if free < (8 << 30):
        pytest.skip("needs 8 GiB of free device memory")
    k, m, page, pps = 4, 2, 32768, 64
    ppp = (6 << 30) // page
    pool = torch.empty(ppp * page, dtype=torch.uint8, device="cuda")
    for at in range(0, pool.numel(), 1 << 30):
        pool[at:at + (1 << 30)].random_(0, 256)
    pages = pool.view(ppp, page)
    rng = np.random.default_rng(inputs.SEED_BASE + 0x410)
    high = (1 << 32) // page
    low = rng.choice(high, size=pps // 2, replace=False)                             # below 4 GiB
    above = high + rng.choice(ppp - high, size=(k + 1) * pps - pps // 2, replace=False)
    ids = rng.permutation(np.concatenate([low, above[pps:]])).astype(np.int32)
    table_np = np.ascontiguousarray(ids.reshape(k, pps))
    spare_np = above[:pps].astype(np.int32)                                           # fresh pages, all above 4 GiB
    table = torch.from_numpy(table_np).cuda()
    base = torch.tensor([pool.data_ptr()], dtype=torch.int64, device="cuda")
    S = pps * page
    # the oracle's pool: the named pages only, numbered 0 .. k*pps-1 in table order
    small = pages[torch.from_numpy(table_np.reshape(-1).astype(np.int64)).cuda()].cpu().numpy().reshape(-1)
    small_table = np.arange(k * pps, dtype=np.int32).reshape(k, pps)
    if kind == "rdp":
        code = gs.gs_make_rdp_code(k, page)
        streams = [small.reshape(k, S)[j] for j in range(k)]
        want = oracle.rdp_encode([np.ascontiguousarray(s) for s in streams], page)
    else:
        code = gs.gs_make_code(k, m)
        want = oracle.encode_paged(oracle.generator(k, m), [small], page, small_table)
    par = [torch.full((S + 64,), 0xC7, dtype=torch.uint8, device="cuda") for _ in range(m)]
    gs.gs_encode_paged(code, base, 1, page, ppp, table, pps, par)
    torch.cuda.synchronize()
    for i in range(m):
        got = par[i].cpu().numpy()
        assert np.array_equal(got[:S], want[i]), (kind, i)
        assert (got[S:] == 0xC7).all()
    pipe = gs.gs_pipe_create(code, 16 * page, 2)
    host = [torch.full((S,), 0x5A, dtype=torch.uint8).pin_memory() for _ in range(m)]
    gs.gs_checkpoint_paged(pipe, base, 1, page, ppp, table, pps, host)
    gs.gs_pipe_sync(pipe)
    for i in range(m):
        assert np.array_equal(host[i].numpy(), want[i]), (kind, i)
    # shard 2 is lost and rebuilt into fresh pages above 4 GiB; shard 0 in place through the pipeline
    lost = 2
    new_table_np = table_np.copy()
    new_table_np[lost] = spare_np[:pps]
    assert (new_table_np[lost].astype(np.int64) * page >= (1 << 32)).all()
    new_table = torch.from_numpy(np.ascontiguousarray(new_table_np)).cuda()
    before = pages[torch.from_numpy(table_np[lost].astype(np.int64)).cuda()].clone()
    gs.gs_reconstruct_paged(code, base, 1, page, ppp, new_table, pps, [p[:S] for p in par], [lost])
    torch.cuda.synchronize()
    assert torch.equal(pages[torch.from_numpy(new_table_np[lost].astype(np.int64)).cuda()], before)
    idx0 = torch.from_numpy(table_np[0].astype(np.int64)).cuda()
    keep = pages[idx0].clone()
    pages[idx0] = 0xA5
    gs.gs_restore_paged(pipe, base, 1, page, ppp, table, pps, host, [0])
    gs.gs_pipe_sync(pipe)
    torch.cuda.synchronize()
    assert torch.equal(pages[idx0], keep)
    gs.gs_pipe_destroy(pipe)

