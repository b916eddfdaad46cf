"""The grouped encode that allocates nothing (gs_encode_batch_static) against
the grouped encode it is a variant of (gs_encode_batch), through the C ABI:
same bytes, on two calls in a row that share the library's fixed descriptor
array, the second with fewer and smaller chunks.  The oracle is the referee
for both."""
import numpy as np
import pytest

import oracle
from paper_2605_00831_amd import inputs

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def gs():
    from paper_2605_00831_amd import binding
    binding.lib()
    binding.gs_set_launch_shape()
    return binding


def run_both(gs, code, batch, P, sizes, seed):
    k, m = P.shape[1], P.shape[0]
    data_np = [[inputs.uniform_bytes_np(seed + 31 * c + j, S) for j in range(k)] for c, S in enumerate(sizes)]
    data = [[torch.from_numpy(x).cuda() if x.size else torch.empty(16, dtype=torch.uint8, device="cuda") for x in row]
            for row in data_np]
    out_a = [[torch.full((S + 64,), 0xEE, dtype=torch.uint8, device="cuda") for _ in range(m)] for S in sizes]
    out_b = [[torch.full((S + 64,), 0xEE, dtype=torch.uint8, device="cuda") for _ in range(m)] for S in sizes]
    torch.cuda.synchronize()
    gs.gs_encode_batch(batch, data, out_a, sizes)
    gs.gs_encode_batch_static(code, data, out_b, sizes)
    torch.cuda.synchronize()
    for c, S in enumerate(sizes):
        want = oracle.encode(P, data_np[c]) if S else [np.zeros(0, np.uint8)] * m
        for i in range(m):
            a, b = out_a[c][i].cpu().numpy(), out_b[c][i].cpu().numpy()
            assert np.array_equal(b, a), "chunk %d parity %d: static differs from gs_encode_batch" % (c, i)
            assert np.array_equal(b[:S], want[i]), "chunk %d parity %d differs from the oracle" % (c, i)
            assert (b[S:] == 0xEE).all(), "chunk %d parity %d: bytes past the end were written" % (c, i)


@pytest.mark.parametrize("k,m", [(8, 2), (4, 1), (16, 4)])
def test_static_grouped_encode_equals_grouped_encode_on_two_calls_in_a_row(gs, k, m):
    P = oracle.generator(k, m)
    code = gs.gs_make_code(k, m)
    batch = gs.gs_batch_create(code, 64)
    # first call: more chunks than one fill launch carries, ragged sizes across several tiles, an empty chunk
    first = [(256 << 10) + 16 * c + (c % 5) for c in range(40)]
    first[7] = 0
    first[11] = 5
    run_both(gs, code, batch, P, first, 1000 * k)
    # second call right after it: fewer and smaller chunks; nothing of the first call's descriptors may leak in
    second = [4096 + 3 * c for c in range(9)]
    run_both(gs, code, batch, P, second, 2000 * k)
    gs.gs_batch_destroy(batch)


@pytest.mark.parametrize("k,m", [(1, 1), (2, 1), (2, 2)])
def test_static_grouped_encode_of_narrow_codes_with_many_chunks(gs, k, m):
    # a narrow code's chunks take few argument words each: a fill launch is then bounded by its
    # thread count, not by the argument block
    P = oracle.generator(k, m)
    code = gs.gs_make_code(k, m)
    batch = gs.gs_batch_create(code, 200)
    run_both(gs, code, batch, P, [2048 + 16 * c + (c % 3) for c in range(200)], 3000 * k + m)
    run_both(gs, code, batch, P, [1024 + c for c in range(70)], 4000 * k + m)
    gs.gs_batch_destroy(batch)


def test_static_grouped_encode_limits(gs):
    code = gs.gs_make_code(4, 2)
    t = torch.zeros(64, dtype=torch.uint8, device="cuda")
    n = gs.GS_STATIC_MAX_CHUNKS + 1
    with pytest.raises(gs.GsError) as e:
        gs.gs_encode_batch_static(code, [[t] * 4] * n, [[t, t]] * n, [0] * n)
    assert e.value.status == gs.GS_ELIMIT
    wide = gs.gs_make_code(17, 2)
    with pytest.raises(gs.GsError) as e:
        gs.gs_encode_batch_static(wide, [[t] * 17], [[t, t]], [16])
    assert e.value.status == gs.GS_EINVAL
    gs.gs_encode_batch_static(code, [], [], [])           # no chunks: nothing to do
    # the full capacity in one call, tiny chunks
    k, m, S = 4, 2, 64
    P = oracle.generator(k, m)
    n = gs.GS_STATIC_MAX_CHUNKS
    buf_np = inputs.uniform_bytes_np(5, n * k * S)
    buf = torch.from_numpy(buf_np).cuda()
    out = torch.full((n * m * S,), 0xEE, dtype=torch.uint8, device="cuda")
    data = [[buf[(c * k + j) * S:(c * k + j + 1) * S] for j in range(k)] for c in range(n)]
    par = [[out[(c * m + i) * S:(c * m + i + 1) * S] for i in range(m)] for c in range(n)]
    gs.gs_encode_batch_static(code, data, par, [S] * n)
    torch.cuda.synchronize()
    got = out.cpu().numpy().reshape(n, m, S)
    src = buf_np.reshape(n, k, S)
    # chunks are independent: encode all of them as one long stream per shard position
    want = oracle.encode(P, [np.ascontiguousarray(src[:, j, :]).reshape(-1) for j in range(k)])
    for i in range(m):
        assert np.array_equal(got[:, i, :].reshape(-1), want[i])


def test_static_grouped_encode_replays_from_a_graph(gs):
    """The call enqueues kernel launches only, so it can be captured; the graph (two descriptor-fill
    launches and the grouped kernel) is replayed several times on changing data, with eager work and
    synchronisation between the replays, and every replay is checked against the oracle."""
    k, m, n = 8, 2, 60
    P = oracle.generator(k, m)
    code = gs.gs_make_code(k, m)
    sizes = [8192 + 16 * c + (c % 7) for c in range(n)]
    data = [[torch.zeros(S, dtype=torch.uint8, device="cuda") for _ in range(k)] for S in sizes]
    par = [[torch.zeros(S + 64, dtype=torch.uint8, device="cuda") for _ in range(m)] for S in sizes]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        gs.gs_encode_batch_static(code, data, par, sizes)     # first use on this device: outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        gs.gs_encode_batch_static(code, data, par, sizes)
    for rep in range(4):
        data_np = [[inputs.uniform_bytes_np(7000 + 1000 * rep + 10 * c + j, S) for j in range(k)] for c, S in enumerate(sizes)]
        for c in range(n):
            for j in range(k):
                data[c][j].copy_(torch.from_numpy(data_np[c][j]))     # eager work between replays
            for t in par[c]:
                t.fill_(0xEE)
        # another eager call in between overwrites the shared descriptor array: the replay must rewrite it
        gs.gs_encode_batch_static(code, data[:3], par[:3], sizes[:3])
        for t in par[0] + par[1] + par[2]:
            t.fill_(0xEE)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for c, S in enumerate(sizes):
            want = oracle.encode(P, data_np[c])
            for i in range(m):
                got = par[c][i].cpu().numpy()
                assert np.array_equal(got[:S], want[i]), (rep, c, i)
                assert (got[S:] == 0xEE).all(), (rep, c, i)
