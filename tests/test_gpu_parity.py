"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle,
byte for byte, on the same seeded inputs.  Integer/byte work, so the bar is
bit-exact everywhere."""
import itertools

import numpy as np
import pytest

import oracle
from paper_2605_00831_amd import inputs

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

CANARY = 0xC7
PAD = 256  # canary bytes after every output buffer


@pytest.fixture(scope="module")
def gs():
    from paper_2605_00831_amd import binding
    binding.lib()
    yield binding
    binding.gs_set_launch_shape()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def out_buf(nbytes):
    """device buffer of nbytes + PAD canary bytes (whole thing pre-filled)"""
    return torch.full((nbytes + PAD,), CANARY, dtype=torch.uint8, device="cuda")


def check_out(buf, want):
    got = buf.cpu().numpy()
    n = want.size
    assert np.array_equal(got[:n], want), "payload differs (first at %d)" % int(np.nonzero(got[:n] != want)[0][0])
    assert (got[n:] == CANARY).all(), "wrote past shard_bytes"


def rand_shards(seed, k, S):
    return [inputs.uniform_bytes_np(seed * 1009 + j, S) for j in range(k)]


def gpu_encode(gs, code, data_np, S, stream=None):
    d = [dev(x) for x in data_np]
    p = [out_buf(S) for _ in range(code.m)]
    gs.gs_encode(code, d, p, S, stream)
    torch.cuda.synchronize()
    return d, p


# ---------------------------------------------------------------- encode

SIZES = [1, 15, 16, 17, 4095, 4096, 4097, 8192 + 16, 65536 + 5, 3 * 8192 + 4080, 1 << 20, (1 << 21) + 3]


@pytest.mark.parametrize("k,m", [(4, 2), (4, 1), (8, 2), (8, 3), (1, 1), (2, 4), (3, 3), (5, 3), (7, 2), (16, 4)])
def test_encode_matches_oracle_over_ragged_sizes(gs, k, m):
    code = gs.gs_make_code(k, m)
    P = oracle.generator(k, m)
    assert np.array_equal(gs.gs_code_matrix(code), P)
    for S in SIZES:
        if k * S > (24 << 20):
            continue
        data = rand_shards(S + k, k, S)
        want = oracle.encode(P, data, nthreads=8)
        d, p = gpu_encode(gs, code, data, S)
        for i in range(m):
            check_out(p[i], want[i])
        for j in range(k):
            assert np.array_equal(d[j].cpu().numpy(), data[j])  # inputs untouched


@pytest.mark.parametrize("unroll,tiles_per_wg,nt,ilv", [
    (1, 1, 1, 5), (2, 1, 0, 5), (4, 1, 1, 5), (1, 3, 0, 3), (2, 5, 1, 0), (4, 2, 0, 1), (2, 64, 1, 5), (2, 1, 1, 10),
    (1, 7, 1, 6), (2, 1, 1, 0)])
def test_every_launch_shape_gives_the_same_bytes(gs, unroll, tiles_per_wg, nt, ilv):
    gs.gs_set_launch_shape(unroll, tiles_per_wg, nt, ilv)
    try:
        sizes = [16 * 256 * 11 + 48 + 7, 777, (1 << 20) + 16 * 64 * 3 + 9, 256 * 1024, 256 * 1024 - 16]
        for (k, m), S in itertools.product([(4, 2), (8, 3), (6, 1)], sizes):
            code = gs.gs_make_code(k, m)
            data = rand_shards(S + k + unroll, k, S)
            want = oracle.encode(oracle.generator(k, m), data, nthreads=8)
            _, p = gpu_encode(gs, code, data, S)
            for i in range(m):
                check_out(p[i], want[i])
    finally:
        gs.gs_set_launch_shape()


def test_wide_code_runs_as_accumulating_launches(gs):
    """k > 16 or m > 4 is split into several launches that XOR-accumulate."""
    for k, m, S in [(20, 6, 70001), (33, 2, 4096 + 9), (17, 5, 123)]:
        code = gs.gs_make_code(k, m)
        data = rand_shards(k * 7 + m, k, S)
        want = oracle.encode(oracle.generator(k, m), data, nthreads=8)
        _, p = gpu_encode(gs, code, data, S)
        for i in range(m):
            check_out(p[i], want[i])


def test_encode_on_a_side_stream(gs):
    k, m, S = 4, 2, (1 << 20) + 100
    code = gs.gs_make_code(k, m)
    data = rand_shards(91, k, S)
    want = oracle.encode(oracle.generator(k, m), data, nthreads=8)
    s = torch.cuda.Stream()
    d = [dev(x) for x in data]
    p = [out_buf(S) for _ in range(m)]
    torch.cuda.synchronize()
    gs.gs_encode(code, d, p, S, s)
    s.synchronize()
    for i in range(m):
        check_out(p[i], want[i])


def test_config1_tiny_encode_then_lose_1_and_3(gs):
    """fp16 KV of a 2-layer model, 1024 tokens, 8 MiB, k=4, m=2; erase {1,3}."""
    c = inputs.CONFIGS["tiny"]
    buf = inputs.kv_bytes_np(inputs.config_seed("tiny"), inputs.config_total_bytes("tiny"), c["dtype"], c["sigma"])
    inputs.plant_specials(buf, "fp16", 1)
    data = [np.ascontiguousarray(s) for s in inputs.split_shards(buf, 4)]
    S = data[0].size
    assert S == 2 << 20
    P = oracle.generator(4, 2)
    want = oracle.encode(P, data, nthreads=8)
    code = gs.gs_make_code(4, 2)
    d, p = gpu_encode(gs, code, data, S)
    for i in range(2):
        check_out(p[i], want[i])
    # failure = flushed buffers: poison the lost shards, rebuild in place
    shards = d + [x[:S] for x in p]
    for r in c["erased"]:
        shards[r].fill_(0xA5)
    gs.gs_reconstruct(code, shards, list(c["erased"]), S)
    torch.cuda.synchronize()
    full = data + want
    for r in range(6):
        got = shards[r].cpu().numpy()
        assert np.array_equal(got, full[r])
        assert np.array_equal(got.view(np.int16), full[r].view(np.int16))
    # and the oracle agrees on the same erasure
    work = [x.copy() for x in full]
    for r in c["erased"]:
        work[r][:] = 0xA5
    oracle.reconstruct(P, work, list(c["erased"]))
    assert all(np.array_equal(a, b) for a, b in zip(work, full))


# ---------------------------------------------------------------- reconstruct

def _stripe_on_gpu(gs, k, m, S, seed, kv=False):
    if kv:
        buf = inputs.kv_bytes_np(seed, k * S, "bf16", 1.0)
        inputs.plant_specials(buf, "bf16", seed)
        data = [np.ascontiguousarray(x) for x in inputs.split_shards(buf, k)]
    else:
        data = rand_shards(seed, k, S)
    P = oracle.generator(k, m)
    full = data + oracle.encode(P, data, nthreads=8)
    return P, full


def _reconstruct_and_check(gs, code, P, full, pat, S):
    n = len(full)
    bufs = []
    for r in range(n):
        if r in pat:
            b = out_buf(S)
            b[:S] = 0xA5
        else:
            b = torch.cat([dev(full[r]), torch.full((PAD,), CANARY, dtype=torch.uint8, device="cuda")])
        bufs.append(b)
    gs.gs_reconstruct(code, bufs, list(pat), S)
    torch.cuda.synchronize()
    for r in range(n):
        check_out(bufs[r], full[r])
    # the oracle rebuilds the same bytes from the same survivors
    work = [x.copy() for x in full]
    for r in pat:
        work[r][:] = 0xA5
    oracle.reconstruct(P, work, list(pat))
    for r in pat:
        assert np.array_equal(work[r], full[r])


@pytest.mark.parametrize("k,m", [(4, 2), (3, 3), (2, 4), (5, 1), (1, 2)])
def test_reconstruct_every_erasure_subset_small_codes(gs, k, m):
    S = 4096 + 16 + 5
    P, full = _stripe_on_gpu(gs, k, m, S, 300 + k * 8 + m)
    code = gs.gs_make_code(k, m)
    for pat in inputs.all_erasure_patterns(k + m, m, 1):
        _reconstruct_and_check(gs, code, P, full, pat, S)


def test_config5_small_all_165_triples(gs):
    """k=8, m=3, S = 64 KiB + 5: shards 0-3 uniform bytes, 4-7 bf16 N(0,1) KV."""
    c = inputs.CONFIGS["recovery_stress"]
    S = c["small_shard_bytes"]
    seed = inputs.config_seed("recovery_stress")
    data = [inputs.uniform_bytes_np(seed + j, S) for j in range(4)]
    data += [inputs.kv_bytes_np(seed + j, S, "bf16", 1.0) for j in range(4, 8)]
    P = oracle.generator(8, 3)
    full = data + oracle.encode(P, data, nthreads=8)
    code = gs.gs_make_code(8, 3)
    pats = list(itertools.combinations(range(11), 3))
    assert len(pats) == 165
    for pat in pats:
        _reconstruct_and_check(gs, code, P, full, pat, S)


def test_reconstruct_wide_code_and_order_of_erased_list(gs):
    k, m, S = 20, 6, 9001
    P, full = _stripe_on_gpu(gs, k, m, S, 17)
    code = gs.gs_make_code(k, m)
    for pat in [(0, 19, 20, 25, 7, 3), (25, 24, 23, 22, 21, 20), (5,), (19, 18, 17, 16, 15, 14)]:
        _reconstruct_and_check(gs, code, P, full, pat, S)


def test_reconstruct_is_lossless_for_float_bit_patterns(gs):
    k, m, S = 4, 2, 1 << 16
    P, full = _stripe_on_gpu(gs, k, m, S, 5, kv=True)
    code = gs.gs_make_code(k, m)
    _reconstruct_and_check(gs, code, P, full, (0, 2), S)
    allv = np.concatenate([s.view(np.uint16) for s in full[:k]])
    for pat in inputs.special_bits("bf16"):
        assert (allv == pat).any()


def test_reconstruct_errors_write_nothing(gs):
    k, m, S = 4, 2, 1024
    P, full = _stripe_on_gpu(gs, k, m, S, 6)
    code = gs.gs_make_code(k, m)
    bufs = [dev(x) for x in full]
    for bad, status in [([0, 1, 2], gs.GS_ETOOMANY), ([1, 1], gs.GS_EINVAL), ([9], gs.GS_EINVAL)]:
        with pytest.raises(gs.GsError) as e:
            gs.gs_reconstruct(code, bufs, bad, S)
        assert e.value.status == status
    gs.gs_reconstruct(code, bufs, [], S)
    torch.cuda.synchronize()
    for r in range(k + m):
        assert np.array_equal(bufs[r].cpu().numpy(), full[r])


# ---------------------------------------------------------------- paged

def _paged_case(gs, k, m, n_planes, pps, page_bytes, extra_pages=9, seed=1):
    num_pages = k * pps + extra_pages
    planes_np = [inputs.kv_bytes_np(seed * 100 + p, num_pages * page_bytes, "bf16", 1.0) for p in range(n_planes)]
    table_np = inputs.block_table_np(seed, k, pps, num_pages)
    P = oracle.generator(k, m)
    want = oracle.encode_paged(P, planes_np, page_bytes, table_np)
    planes = [dev(x) for x in planes_np]
    base = torch.tensor([x.data_ptr() for x in planes], dtype=torch.int64, device="cuda")
    table = dev(table_np)
    out_bytes = n_planes * pps * page_bytes
    par = [out_buf(out_bytes) for _ in range(m)]
    code = gs.gs_make_code(k, m)
    gs.gs_encode_paged(code, base, n_planes, page_bytes, num_pages, table, pps, par)
    torch.cuda.synchronize()
    for i in range(m):
        check_out(par[i], want[i])
    for p in range(n_planes):
        assert np.array_equal(planes[p].cpu().numpy(), planes_np[p])
    return planes_np, table_np, want


@pytest.mark.parametrize("k,m,n_planes,pps,page_bytes", [
    (4, 1, 64, 16, 2048),    # the decode-step geometry: 64 planes, 16 token slots of 2 KiB
    (4, 2, 3, 5, 32768),     # whole 16-token blocks
    (8, 2, 16, 7, 512),      # KV-head-group segments
    (3, 3, 2, 11, 48),       # page size not a power of two
    (5, 2, 1, 1, 16),        # one vector
    (20, 5, 2, 9, 1040),     # wide code through the paged path
])
def test_paged_encode_matches_oracle(gs, k, m, n_planes, pps, page_bytes):
    for shape in [(1, 1, 1), (2, 1, 1), (4, 2, 0)]:
        gs.gs_set_launch_shape(*shape)
        try:
            _paged_case(gs, k, m, n_planes, pps, page_bytes)
        finally:
            gs.gs_set_launch_shape()


def test_paged_out_of_range_page_ids_read_as_zero(gs):
    k, m, n_planes, pps, page_bytes = 4, 2, 2, 6, 256
    num_pages = k * pps
    planes_np = [inputs.uniform_bytes_np(40 + p, num_pages * page_bytes) for p in range(n_planes)]
    table_np = inputs.block_table_np(3, k, pps, num_pages)
    table_bad = table_np.copy()
    table_bad[1, 2] = -1
    table_bad[3, 0] = num_pages
    table_bad[2, 5] = 2 ** 31 - 1
    # oracle view: those pages are zero pages appended to the pool
    planes_z = [np.concatenate([pl, np.zeros(page_bytes, np.uint8)]) for pl in planes_np]
    table_z = table_bad.copy()
    table_z[(table_bad < 0) | (table_bad >= num_pages)] = num_pages
    P = oracle.generator(k, m)
    want = oracle.encode_paged(P, planes_z, page_bytes, table_z)
    planes = [dev(x) for x in planes_np]
    base = torch.tensor([x.data_ptr() for x in planes], dtype=torch.int64, device="cuda")
    par = [out_buf(n_planes * pps * page_bytes) for _ in range(m)]
    code = gs.gs_make_code(k, m)
    gs.gs_encode_paged(code, base, n_planes, page_bytes, num_pages, dev(table_bad), pps, par)
    torch.cuda.synchronize()
    for i in range(m):
        check_out(par[i], want[i])


def test_paged_identity_table_equals_contiguous_encode(gs):
    k, m, pps, page_bytes = 4, 2, 8, 4096
    plane_np = inputs.uniform_bytes_np(4, k * pps * page_bytes)
    table_np = np.arange(k * pps, dtype=np.int32).reshape(k, pps)
    plane = dev(plane_np)
    base = torch.tensor([plane.data_ptr()], dtype=torch.int64, device="cuda")
    code = gs.gs_make_code(k, m)
    S = pps * page_bytes
    par_p = [out_buf(S) for _ in range(m)]
    par_c = [out_buf(S) for _ in range(m)]
    gs.gs_encode_paged(code, base, 1, page_bytes, k * pps, dev(table_np), pps, par_p)
    gs.gs_encode(code, [plane[j * S:(j + 1) * S] for j in range(k)], par_c, S)
    torch.cuda.synchronize()
    for i in range(m):
        assert torch.equal(par_p[i], par_c[i])


# ---------------------------------------------------------------- extremes

def test_widest_code_the_field_allows(gs):
    """k + m = 256 is the limit (distinct evaluation points in GF(2^8))."""
    for k, m in [(250, 6), (1, 255), (128, 128)]:
        S = 1111 if k * m > 4000 else 4099
        code = gs.gs_make_code(k, m)
        data = rand_shards(k + m, k, S)
        want = oracle.encode(oracle.generator(k, m), data, nthreads=8)
        _, p = gpu_encode(gs, code, data, S)
        for i in range(m):
            check_out(p[i], want[i])
    # lose the maximum number of shards of the (250, 6) code
    k, m, S = 250, 6, 515
    P, full = _stripe_on_gpu(gs, k, m, S, 99)
    code = gs.gs_make_code(k, m)
    _reconstruct_and_check(gs, code, P, full, (0, 17, 100, 249, 250, 255), S)


def test_empty_inputs_are_no_ops_on_the_gpu(gs):
    code = gs.gs_make_code(4, 2)
    d = [torch.zeros(16, dtype=torch.uint8, device="cuda") for _ in range(4)]
    p = [out_buf(0) for _ in range(2)]
    gs.gs_encode(code, d, p, 0)
    gs.gs_reconstruct(code, d + p, [1], 0)
    gs.gs_reconstruct(code, d + p, [], 16)
    base = torch.tensor([d[0].data_ptr()], dtype=torch.int64, device="cuda")
    table = torch.zeros((4, 1), dtype=torch.int32, device="cuda")
    gs.gs_encode_paged(code, base, 0, 16, 1, table, 1, p)
    gs.gs_encode_paged(code, base, 1, 16, 1, table, 0, p)
    torch.cuda.synchronize()
    for b in p:
        assert (b.cpu().numpy() == CANARY).all()


def test_misaligned_or_null_pointers_are_rejected(gs):
    code = gs.gs_make_code(4, 2)
    big = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    good = [big[i * 256:(i + 1) * 256] for i in range(4)]
    par = [out_buf(256) for _ in range(2)]
    bad = list(good)
    bad[2] = big[1001:1257]
    with pytest.raises(gs.GsError) as e:
        gs.gs_encode(code, bad, par, 256)
    assert e.value.status == gs.GS_EINVAL
    with pytest.raises(gs.GsError) as e:
        gs.gs_encode(code, good, [par[0], None], 256)
    assert e.value.status == gs.GS_EINVAL
    # a survivor that the decode needs must be present
    shards = good + [p[:256] for p in par]
    gs.gs_encode(code, good, par, 256)
    with pytest.raises(gs.GsError) as e:
        gs.gs_reconstruct(code, [good[0], None, good[2], good[3], par[0], par[1]], [0], 256)
    assert e.value.status == gs.GS_EINVAL
    # ... but a survivor beyond the first k may be missing
    gs.gs_reconstruct(code, [good[0], good[1], good[2], good[3], par[0], None], [0], 256)
    torch.cuda.synchronize()
    for b in par:
        assert (b.cpu().numpy()[256:] == CANARY).all()


# ---------------------------------------------------------------- paged reconstruct

@pytest.mark.parametrize("k,m,n_planes,pps,page_bytes,pats", [
    (4, 1, 8, 16, 2048, [(2,), (4,)]),
    (4, 2, 3, 5, 32768, [(1, 3), (0, 5), (4, 5), (2,)]),
    (8, 3, 2, 7, 512, [(2, 5, 9), (0, 1, 2), (8, 9, 10), (7, 8)]),
    (3, 2, 2, 11, 48, [(0, 2), (1, 4)]),
    (20, 5, 2, 3, 1040, [(0, 19, 20, 24, 7)]),
    (4, 2, 8, 288, 2048, [(1, 3), (0, 4)]),   # more than 1024 workgroups: the bulk form of the kernel
])
def test_paged_reconstruct_rebuilds_into_fresh_pages(gs, k, m, n_planes, pps, page_bytes, pats):
    spare = 3 * pps + 5
    num_pages = k * pps + spare
    planes_np = [inputs.kv_bytes_np(700 + p, num_pages * page_bytes, "bf16", 1.0) for p in range(n_planes)]
    perm = np.random.default_rng(77).permutation(num_pages).astype(np.int32)
    table_np = np.ascontiguousarray(perm[: k * pps].reshape(k, pps))
    free_pages = perm[k * pps:]
    P = oracle.generator(k, m)
    gathered = [np.ascontiguousarray(np.concatenate([pl.reshape(num_pages, page_bytes)[table_np[j]].reshape(-1)
                                                     for pl in planes_np])) for j in range(k)]
    par_np = oracle.encode(P, gathered, nthreads=8)
    code = gs.gs_make_code(k, m)
    out_bytes = n_planes * pps * page_bytes
    for pat in pats:
        lost_data = [r for r in pat if r < k]
        assert len(lost_data) * pps <= free_pages.size
        # the restarted engine gives every lost data shard fresh pages; everything it lost is poison
        new_table = table_np.copy()
        pool_np = [pl.copy() for pl in planes_np]
        for n, r in enumerate(lost_data):
            new_table[r] = free_pages[n * pps:(n + 1) * pps]
            for pl in pool_np:
                v = pl.reshape(num_pages, page_bytes)
                v[table_np[r]] = 0xA5          # old pages are gone
                v[new_table[r]] = 0x5A         # new pages hold garbage
        planes = [dev(x) for x in pool_np]
        base = torch.tensor([x.data_ptr() for x in planes], dtype=torch.int64, device="cuda")
        parity = []
        for i in range(m):
            if k + i in pat:
                t = out_buf(out_bytes)
                t[:out_bytes] = 0xA5
            else:
                t = torch.cat([dev(par_np[i]), torch.full((PAD,), CANARY, dtype=torch.uint8, device="cuda")])
            parity.append(t)
        gs.gs_reconstruct_paged(code, base, n_planes, page_bytes, num_pages, dev(new_table), pps, parity, list(pat))
        torch.cuda.synchronize()
        for p in range(n_planes):
            got = planes[p].cpu().numpy().reshape(num_pages, page_bytes)
            want = pool_np[p].reshape(num_pages, page_bytes).copy()
            for r in lost_data:
                want[new_table[r]] = planes_np[p].reshape(num_pages, page_bytes)[table_np[r]]
            assert np.array_equal(got, want), (pat, p)      # rebuilt pages right, every other page untouched
        for i in range(m):
            check_out(parity[i], par_np[i])
        # oracle on the gathered stripe gives the same bytes
        work = [x.copy() for x in gathered + par_np]
        for r in pat:
            work[r][:] = 0
        oracle.reconstruct(P, work, list(pat))
        for r in pat:
            assert np.array_equal(work[r], (gathered + par_np)[r])


def test_paged_reconstruct_errors_and_noop(gs):
    code = gs.gs_make_code(4, 2)
    plane = torch.zeros(64 * 256, dtype=torch.uint8, device="cuda")
    base = torch.tensor([plane.data_ptr()], dtype=torch.int64, device="cuda")
    table = torch.arange(32, dtype=torch.int32, device="cuda").reshape(4, 8).contiguous()
    par = [out_buf(8 * 256) for _ in range(2)]
    with pytest.raises(gs.GsError) as e:
        gs.gs_reconstruct_paged(code, base, 1, 256, 64, table, 8, par, [0, 1, 2])
    assert e.value.status == gs.GS_ETOOMANY
    with pytest.raises(gs.GsError) as e:
        gs.gs_reconstruct_paged(code, base, 1, 256, 64, table, 8, [None, par[1]], [0])   # parity 0 is needed
    assert e.value.status == gs.GS_EINVAL
    gs.gs_reconstruct_paged(code, base, 1, 256, 64, table, 8, par, [])
    torch.cuda.synchronize()
    assert not plane.cpu().numpy().any()
    for b in par:
        assert (b.cpu().numpy() == CANARY).all()


def test_one_code_shared_by_host_threads(gs):
    """A gs_code is immutable: four host threads encode and rebuild through the same handle,
    each on a stream of its own (ctypes drops the interpreter lock during the calls)."""
    import threading
    k, m, S, rounds = 8, 3, (1 << 18) + 4096 + 21, 6
    P = oracle.generator(k, m)
    code = gs.gs_make_code(k, m)
    errors = []

    def worker(tid):
        try:
            stream = torch.cuda.Stream()
            for rnd in range(rounds):
                data_np = [inputs.uniform_bytes_np(40000 + 1000 * tid + 10 * rnd + j, S) for j in range(k)]
                with torch.cuda.stream(stream):
                    data = [torch.from_numpy(x).cuda() for x in data_np]
                    par = [torch.zeros(S, dtype=torch.uint8, device="cuda") for _ in range(m)]
                    gs.gs_encode(code, data, par, S, stream=stream)
                    pat = [(tid + rnd) % k, k + (rnd % m), (tid + rnd + 3) % k]
                    pat = sorted(set(pat))
                    for r in pat:
                        (data + par)[r].fill_(0x5A)
                    gs.gs_reconstruct(code, data + par, pat, S, stream=stream)
                    stream.synchronize()
                    want = oracle.encode(P, data_np)
                    full = data_np + want
                    for r in range(k + m):
                        if not np.array_equal((data + par)[r].cpu().numpy(), full[r]):
                            errors.append((tid, rnd, r))
        except Exception as e:  # noqa: BLE001 - reported below
            errors.append((tid, repr(e)))

    threads = [threading.Thread(target=worker, args=(t,)) for t in range(4)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors


def test_paged_encode_at_the_largest_plane_count(gs):
    # 65535 planes (the grid's y limit), 3 slots of 48 bytes per shard and plane, planes cut from one pool
    k, m, n_planes, pps, page = 3, 2, 65535, 3, 48
    num_pages = k * pps + 2
    pool_np = inputs.uniform_bytes_np(4321, n_planes * num_pages * page)
    planes_np = [pool_np[p * num_pages * page:(p + 1) * num_pages * page] for p in range(n_planes)]
    table_np = inputs.block_table_np(9, k, pps, num_pages)
    want = oracle.encode_paged(oracle.generator(k, m), planes_np, page, table_np)
    pool = dev(pool_np)
    base = dev(pool.data_ptr() + np.arange(n_planes, dtype=np.int64) * (num_pages * page))
    out_bytes = n_planes * pps * page
    par = [out_buf(out_bytes) for _ in range(m)]
    code = gs.gs_make_code(k, m)
    gs.gs_encode_paged(code, base, n_planes, page, num_pages, dev(table_np), pps, par)
    torch.cuda.synchronize()
    for i in range(m):
        check_out(par[i], want[i])
    with pytest.raises(gs.GsError):
        gs.gs_encode_paged(code, base, n_planes + 1, page, num_pages, dev(table_np), pps, par)


def test_occupancy_reservation_changes_no_byte(gs):
    # bulk launches with and without the LDS reservation that limits the workgroups per CU: the same bytes,
    # and the oracle's on sampled windows (GF(2^8), Horner and RDP kernels, the grouped launch)
    S = 320 << 20
    rng = np.random.default_rng(99)
    cases = [("cauchy", 4, 2), ("cauchy", 8, 1), ("power", 8, 3), ("rdp", 8, 2)]
    try:
        for kind, k, m in cases:
            if kind == "rdp":
                code = gs.gs_make_rdp_code(k, 32768)
                unit = (gs.gs_rdp_prime(code) - 1) * 32768
            else:
                code = gs.gs_make_code(k, m, gs.GS_POWER if kind == "power" else gs.GS_CAUCHY)
                P = oracle.power_generator(k, m) if kind == "power" else oracle.generator(k, m)
                unit = 1
            Sk = S // unit * unit
            data = [torch.empty(Sk, dtype=torch.uint8, device="cuda").random_(0, 256) for _ in range(k)]
            outs = []
            for on in (1, 0):
                gs.gs_set_occupancy_cap(on)
                par = [torch.full((Sk + PAD,), CANARY, dtype=torch.uint8, device="cuda") for _ in range(m)]
                gs.gs_encode(code, data, par, Sk)
                torch.cuda.synchronize()
                outs.append(par)
            for i in range(m):
                assert torch.equal(outs[0][i], outs[1][i]), (kind, k, m, i)
                assert (outs[0][i][Sk:] == CANARY).all()
            for _ in range(3):
                off = int(rng.integers(0, Sk // unit - 1)) * unit
                n = unit if kind == "rdp" else int(rng.integers(1, 100000))
                n = min(n, Sk - off)
                host = [np.ascontiguousarray(d[off:off + n].cpu().numpy()) for d in data]
                want = oracle.rdp_encode(host, 32768) if kind == "rdp" else oracle.encode(P, host, nthreads=8)
                for i in range(m):
                    assert np.array_equal(outs[0][i][off:off + n].cpu().numpy(), want[i]), (kind, k, m, off, i)
            # rebuild of a lost data shard under both settings
            lost = [1] if m == 1 else [1, k]
            for on in (1, 0):
                gs.gs_set_occupancy_cap(on)
                shards = data + [p[:Sk] for p in outs[0]]
                keep = [shards[r].clone() for r in lost]
                for r in lost:
                    shards[r].fill_(0xA5)
                gs.gs_reconstruct(code, shards, lost, Sk)
                torch.cuda.synchronize()
                for r, orig in zip(lost, keep):
                    assert torch.equal(shards[r], orig), (kind, k, m, on, r)
            del data, outs, shards, keep
    finally:
        gs.gs_set_occupancy_cap(1)


# the library runs launches of at most 1024 workgroups (8 KiB per stream and workgroup for contiguous
# shards, 4 KiB for the paged gather) in a kernel form of their own; sizes on both sides of that line
SMALL_FORM_SIZES = [1024 * 8192 - 16, 1024 * 8192, 1024 * 8192 + 16 + 5, 1100 * 8192 + 4080]


@pytest.mark.parametrize("k,m", [(2, 1), (5, 2), (8, 3), (3, 4), (16, 2), (20, 5)])   # (20, 5): accumulating launches
def test_encode_on_both_sides_of_the_small_launch_threshold(gs, k, m):
    P = oracle.generator(k, m)
    code = gs.gs_make_code(k, m)
    for S in SMALL_FORM_SIZES:
        data = rand_shards(S % 1000 + k, k, S)
        want = oracle.encode(P, data, nthreads=8)
        _, p = gpu_encode(gs, code, data, S)
        for i in range(m):
            check_out(p[i], want[i])


@pytest.mark.parametrize("k,m,pat", [(4, 2, (1,)), (4, 2, (0, 3)), (8, 3, (2, 5, 9)), (6, 4, (0, 1, 2, 3)), (9, 2, (9, 10))])
def test_reconstruct_on_both_sides_of_the_small_launch_threshold(gs, k, m, pat):
    # rebuild matrices without an all-ones row: the kernel variants an encode never runs
    code = gs.gs_make_code(k, m)
    for S in (SMALL_FORM_SIZES[1], SMALL_FORM_SIZES[2]):
        P, full = _stripe_on_gpu(gs, k, m, S, seed=S % 997 + k)
        _reconstruct_and_check(gs, code, P, full, pat, S)


@pytest.mark.parametrize("k,m", [(4, 2), (7, 3)])
def test_horner_encode_on_both_sides_of_the_small_launch_threshold(gs, k, m):
    P = oracle.power_generator(k, m)
    code = gs.gs_make_code(k, m, gs.GS_POWER)
    for S in SMALL_FORM_SIZES[1:3]:
        data = rand_shards(S % 1000 + 3 * k, k, S)
        want = oracle.encode(P, data, nthreads=8)
        _, p = gpu_encode(gs, code, data, S)
        for i in range(m):
            check_out(p[i], want[i])


@pytest.mark.parametrize("k,m,n_planes,pps,page_bytes", [
    (4, 1, 8, 256, 2048),     # 8 planes x 128 workgroups = 1024: the small form
    (4, 1, 8, 258, 2048),     # one super-tile more per plane: the bulk form
    (8, 3, 4, 16, 65536),     # 4 x 256 = 1024
    (8, 3, 4, 17, 65536),
    (5, 2, 2, 1000, 1040),    # lane-indexed pages, 254 tiles rounded up to 256 per plane: 512
    (5, 2, 2, 4100, 1040),
    (18, 5, 2, 2100, 1040),   # accumulating launches in the bulk form
])
def test_paged_encode_on_both_sides_of_the_small_launch_threshold(gs, k, m, n_planes, pps, page_bytes):
    _paged_case(gs, k, m, n_planes, pps, page_bytes, seed=k + pps)


@pytest.mark.parametrize("k,m,sizes", [(8, 3, (3,)), (6, 4, (3, 4)), (16, 3, (3,)), (4, 4, (3, 4))])
def test_bulk_rebuild_of_three_and_four_shards_every_pattern(gs, k, m, sizes):
    """Launches above the small-launch threshold rebuild three and four shards with one row of the matrix
    turned into an XOR row where the matrix allows it (the all-ones parity among the survivors).  Every
    loss pattern (a seeded sample of 120 for 16+3), ragged length: a partial last tile and trailing bytes.
    The stripe is the oracle's; a rebuilt shard must equal the oracle's shard."""
    S = 1056 * 8192 + 3 * 16 + 5
    P, full = _stripe_on_gpu(gs, k, m, S, seed=17 * k + m)
    code = gs.gs_make_code(k, m)
    good = [torch.cat([dev(x), torch.full((PAD,), CANARY, dtype=torch.uint8, device="cuda")]) for x in full]
    work = [g.clone() for g in good]
    pats = [p for e in sizes for p in itertools.combinations(range(k + m), e)]
    if len(pats) > 400:
        rng = np.random.default_rng(5)
        pats = [pats[i] for i in sorted(rng.choice(len(pats), 120, replace=False))]
    for pat in pats:
        for r in pat:
            work[r][:S] = 0xA5
        gs.gs_reconstruct(code, work, list(pat), S)
        for r in range(k + m):
            assert torch.equal(work[r], good[r]), (pat, r)


def test_kernel_forms_by_size_change_no_byte(gs):
    """gs_set_size_forms(0) sends small launches and rebuilds of three and four shards through the general
    bulk form, gs_set_size_forms(2) every contiguous launch through the form of small launches: the same
    bytes as the default, and the oracle's."""
    cases = [(8, 3, (2, 5, 9), 1056 * 8192 + 16 + 7), (6, 4, (0, 1, 3, 7), 1030 * 8192 + 5), (8, 2, (1, 3), 300000),
             (16, 2, (0, 17), 65536 + 3), (5, 1, (2,), 4097)]
    try:
        for k, m, pat, S in cases:
            code = gs.gs_make_code(k, m)
            P, full = _stripe_on_gpu(gs, k, m, S, seed=S % 991 + k)
            outs = []
            for on in (1, 0, 2):
                gs.gs_set_size_forms(on)
                d = [dev(x) for x in full[:k]]
                p = [out_buf(S) for _ in range(m)]
                gs.gs_encode(code, d, p, S)
                shards = []
                for r in range(k + m):
                    if r in pat:
                        t = out_buf(S)
                        t[:S] = 0xA5
                    else:
                        t = torch.cat([dev(full[r]), torch.full((PAD,), CANARY, dtype=torch.uint8, device="cuda")])
                    shards.append(t)
                gs.gs_reconstruct(code, shards, list(pat), S)
                torch.cuda.synchronize()
                for i in range(m):
                    check_out(p[i], full[k + i])
                for r in pat:
                    check_out(shards[r], full[r])
                outs.append([x.clone() for x in p] + [shards[r].clone() for r in pat])
            for other in outs[1:]:
                for a, b in zip(outs[0], other):
                    assert torch.equal(a, b)
        with pytest.raises(gs.GsError):
            gs.gs_set_size_forms(3)
    finally:
        gs.gs_set_size_forms(1)
