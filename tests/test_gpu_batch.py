"""GPU parity for the many-chunk entry points: the grouped launch (gs_batch)
and the one-stream-per-chunk pool (gs_pool).  Every chunk must equal what the
CPU oracle computes for that chunk alone."""
import numpy as np
import pytest

import oracle
from paper_2605_00831_amd import inputs

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

CANARY, PAD = 0xC7, 64


@pytest.fixture(scope="module")
def gs():
    from paper_2605_00831_amd import binding
    binding.lib()
    binding.gs_set_launch_shape()
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def out_buf(n):
    return torch.full((n + PAD,), CANARY, dtype=torch.uint8, device="cuda")


def check(buf, want):
    got = buf.cpu().numpy()
    assert np.array_equal(got[:want.size], want)
    assert (got[want.size:] == CANARY).all()


SIZES = [4096, 0, 1, 15, 4097, (1 << 20) + 5, 65536, 16 * 64 * 33, 2 << 20, 777, 8192, 8192, 3 << 16, 16, 17, 100000]


def make_chunks(k, seed, sizes):
    return [[inputs.uniform_bytes_np(seed + 131 * c + j, S) for j in range(k)] for c, S in enumerate(sizes)]


@pytest.mark.parametrize("k,m", [(4, 2), (8, 3), (4, 1), (16, 4), (1, 1)])
@pytest.mark.parametrize("form", ["batch", "streams"])
def test_encode_many_chunks(gs, k, m, form):
    P = oracle.generator(k, m)
    code = gs.gs_make_code(k, m)
    chunks = make_chunks(k, 1000 * k + m, SIZES)
    want = [oracle.encode(P, ch, nthreads=8) if ch[0].size else [np.zeros(0, np.uint8)] * m for ch in chunks]
    data = [[dev(x) if x.size else torch.zeros(16, dtype=torch.uint8, device="cuda") for x in ch] for ch in chunks]
    par = [[out_buf(S) for _ in range(m)] for S in SIZES]
    torch.cuda.synchronize()
    if form == "batch":
        b = gs.gs_batch_create(code, len(SIZES))
        gs.gs_encode_batch(b, data, par, SIZES)
    else:
        pool = gs.gs_pool_create(5)
        gs.gs_encode_streams(code, pool, data, par, SIZES)
    torch.cuda.synchronize()
    for c in range(len(SIZES)):
        for i in range(m):
            check(par[c][i], want[c][i])


@pytest.mark.parametrize("k,m,pat", [(4, 2, (1, 3)), (8, 3, (2, 5, 9)), (8, 3, (8, 9, 10)), (4, 2, (5,)), (8, 2, (0, 7))])
@pytest.mark.parametrize("form", ["batch", "streams"])
def test_reconstruct_many_chunks(gs, k, m, pat, form):
    P = oracle.generator(k, m)
    code = gs.gs_make_code(k, m)
    sizes = [s for s in SIZES if s]
    chunks = make_chunks(k, 77 * k + m, sizes)
    full = [ch + oracle.encode(P, ch, nthreads=8) for ch in chunks]
    shards = []
    for c, S in enumerate(sizes):
        row = []
        for r in range(k + m):
            if r in pat:
                t = out_buf(S)
                t[:S] = 0xA5
            else:
                t = dev(full[c][r])
            row.append(t)
        shards.append(row)
    torch.cuda.synchronize()
    if form == "batch":
        b = gs.gs_batch_create(code, len(sizes))
        gs.gs_reconstruct_batch(b, shards, list(pat), sizes)
    else:
        pool = gs.gs_pool_create(8)
        gs.gs_reconstruct_streams(code, pool, shards, list(pat), sizes)
    torch.cuda.synchronize()
    for c, S in enumerate(sizes):
        for r in range(k + m):
            if r in pat:
                check(shards[c][r], full[c][r])
            else:
                assert np.array_equal(shards[c][r].cpu().numpy(), full[c][r])
        work = [x.copy() for x in full[c]]
        for r in pat:
            work[r][:] = 0
        oracle.reconstruct(P, work, list(pat))
        for r in pat:
            assert np.array_equal(work[r], full[c][r])


def test_descriptor_ring_wraps_without_corruption(gs):
    """More back-to-back calls than descriptor slots, no synchronisation between them."""
    k, m, S, n = 4, 2, 4096 + 48, 6
    P = oracle.generator(k, m)
    code = gs.gs_make_code(k, m)
    b = gs.gs_batch_create(code, n)
    rounds = []
    for rnd in range(11):
        chunks = make_chunks(k, 5000 + rnd, [S] * n)
        data = [[dev(x) for x in ch] for ch in chunks]
        par = [[out_buf(S) for _ in range(m)] for _ in range(n)]
        rounds.append((chunks, data, par))
    torch.cuda.synchronize()
    for chunks, data, par in rounds:
        gs.gs_encode_batch(b, data, par, [S] * n)
    torch.cuda.synchronize()
    for chunks, data, par in rounds:
        for c in range(n):
            want = oracle.encode(P, chunks[c])
            for i in range(m):
                check(par[c][i], want[i])


def test_batch_argument_errors(gs):
    code = gs.gs_make_code(4, 2)
    with pytest.raises(gs.GsError):
        gs.gs_batch_create(gs.gs_make_code(20, 2), 4)      # wider than one launch covers
    with pytest.raises(gs.GsError):
        gs.gs_batch_create(code, 0)
    b = gs.gs_batch_create(code, 2)
    d = [[torch.zeros(64, dtype=torch.uint8, device="cuda") for _ in range(4)] for _ in range(3)]
    p = [[out_buf(64) for _ in range(2)] for _ in range(3)]
    with pytest.raises(gs.GsError) as e:
        gs.gs_encode_batch(b, d, p, [64, 64, 64])          # more chunks than the batch was made for
    assert e.value.status == gs.GS_EINVAL
    with pytest.raises(gs.GsError) as e:
        gs.gs_reconstruct_batch(b, [x + y for x, y in zip(d[:2], p[:2])], [0, 1, 2], [64, 64])
    assert e.value.status == gs.GS_ETOOMANY
    gs.gs_encode_batch(b, [], [], [])
    torch.cuda.synchronize()
    for row in p:
        for t in row:
            assert (t.cpu().numpy() == CANARY).all()
    with pytest.raises(gs.GsError):
        gs.gs_pool_create(0)


def test_streams_check_every_chunk_before_enqueueing(gs):
    """A misaligned pointer in the last chunk: the call fails and the earlier chunks were not run."""
    k, m, S, n = 4, 2, 4096, 3
    code = gs.gs_make_code(k, m)
    pool = gs.gs_pool_create(2)
    data = [[dev(inputs.uniform_bytes_np(900 + 10 * c + j, S + 16)) for j in range(k)] for c in range(n)]
    par = [[out_buf(S) for _ in range(m)] for _ in range(n)]
    bad = [row[:] for row in data]
    bad[2][1] = data[2][1][1:]                             # base no longer 16-byte aligned
    torch.cuda.synchronize()
    with pytest.raises(gs.GsError) as e:
        gs.gs_encode_streams(code, pool, bad, par, [S] * n)
    assert e.value.status == gs.GS_EINVAL
    shards = [d + p for d, p in zip(data, par)]
    shards[2][0] = data[2][0][1:]
    with pytest.raises(gs.GsError) as e:
        gs.gs_reconstruct_streams(code, pool, shards, [4, 5], [S] * n)
    assert e.value.status == gs.GS_EINVAL
    torch.cuda.synchronize()
    for row in par:
        for t in row:
            assert (t.cpu().numpy() == CANARY).all()


def test_grouped_launch_takes_address_arrays(gs):
    # the same call with the addresses and lengths in numpy arrays instead of lists of tensors
    k, m = 4, 2
    P = oracle.generator(k, m)
    code = gs.gs_make_code(k, m)
    sizes = [4096, 100, 0, (1 << 18) + 3]
    chunks = make_chunks(k, 4242, sizes)
    hold = torch.zeros(16, dtype=torch.uint8, device="cuda")
    data = [[dev(x) if x.size else hold for x in ch] for ch in chunks]
    par = [[out_buf(S) for _ in range(m)] for S in sizes]
    b = gs.gs_batch_create(code, len(sizes))
    a_in = np.array([[t.data_ptr() for t in row] for row in data], dtype=np.uint64)
    a_out = np.array([[t.data_ptr() for t in row] for row in par], dtype=np.uint64)
    gs.gs_encode_batch(b, a_in, a_out, np.array(sizes, dtype=np.uint64))
    torch.cuda.synchronize()
    for c, S in enumerate(sizes):
        want = oracle.encode(P, chunks[c]) if S else [np.zeros(0, np.uint8)] * m
        for i in range(m):
            check(par[c][i], want[i])
    with pytest.raises(ValueError):
        gs.gs_encode_batch(b, a_in[:, :3], a_out, sizes)                 # wrong width
    with pytest.raises(ValueError):
        gs.gs_encode_batch(b, a_in.astype(np.uint32), a_out, sizes)      # not addresses
    with pytest.raises(ValueError):
        gs.gs_encode_batch(b, np.asfortranarray(a_in), a_out, sizes)     # not chunk-major
    gs.gs_batch_destroy(b)


def test_grouped_launch_at_its_largest_chunk_count(gs):
    # 65535 chunks (the grid's y limit) of 48 bytes each, addresses handed over as arrays; chunks are
    # independent, so the oracle encodes shard position j of all chunks as one long stream
    k, m, S, n = 2, 2, 48, 65535
    P = oracle.generator(k, m)
    code = gs.gs_make_code(k, m)
    src_np = inputs.uniform_bytes_np(777, n * k * S)
    src = dev(src_np)
    out = torch.full((n * m * S + PAD,), CANARY, dtype=torch.uint8, device="cuda")
    c = np.arange(n, dtype=np.uint64)
    a_in = np.ascontiguousarray(np.stack([src.data_ptr() + (c * k + j) * S for j in range(k)], axis=1).astype(np.uint64))
    a_out = np.ascontiguousarray(np.stack([out.data_ptr() + (c * m + i) * S for i in range(m)], axis=1).astype(np.uint64))
    b = gs.gs_batch_create(code, n)
    gs.gs_encode_batch(b, a_in, a_out, np.full(n, S, dtype=np.uint64))
    torch.cuda.synchronize()
    want = oracle.encode(P, [np.ascontiguousarray(src_np.reshape(n, k, S)[:, j, :]).reshape(-1) for j in range(k)], nthreads=8)
    got = out.cpu().numpy()
    assert (got[n * m * S:] == CANARY).all()
    got = got[: n * m * S].reshape(n, m, S)
    for i in range(m):
        assert np.array_equal(got[:, i, :].reshape(-1), want[i])
    gs.gs_batch_destroy(b)
    with pytest.raises(gs.GsError):
        gs.gs_batch_create(code, n + 1)


SMALL_GROUP = [4096, 1, 15, 4097, 65536, 16 * 64 * 33, 777, 8192, 100000, 16]


@pytest.mark.parametrize("k,m,pat", [(4, 2, (1, 3)), (8, 3, (2, 5, 9)), (4, 1, (2,)), (6, 4, (0, 1, 2, 3)), (16, 2, (16,))])
def test_grouped_launch_that_does_not_fill_the_chip(gs, k, m, pat):
    """All chunks together are a few hundred workgroups: the grouped launch then runs the kernel form of
    small launches.  Encode and rebuild against the oracle, every kernel variant."""
    P = oracle.generator(k, m)
    code = gs.gs_make_code(k, m)
    chunks = make_chunks(k, 31 * k + m, SMALL_GROUP)
    full = [ch + oracle.encode(P, ch, nthreads=8) for ch in chunks]
    b = gs.gs_batch_create(code, len(SMALL_GROUP))
    data = [[dev(x) for x in ch] for ch in chunks]
    par = [[out_buf(S) for _ in range(m)] for S in SMALL_GROUP]
    gs.gs_encode_batch(b, data, par, SMALL_GROUP)
    torch.cuda.synchronize()
    for c in range(len(SMALL_GROUP)):
        for i in range(m):
            check(par[c][i], full[c][k + i])
    shards = []
    for c, S in enumerate(SMALL_GROUP):
        row = []
        for r in range(k + m):
            if r in pat:
                t = out_buf(S)
                t[:S] = 0xA5
            else:
                t = dev(full[c][r])
            row.append(t)
        shards.append(row)
    gs.gs_reconstruct_batch(b, shards, list(pat), SMALL_GROUP)
    torch.cuda.synchronize()
    for c in range(len(SMALL_GROUP)):
        for r in pat:
            check(shards[c][r], full[c][r])
    gs.gs_batch_destroy(b)
