"""Seeded random sweep on the GPU: code kind, (k, m), shard length, launch
shape and erasure pattern drawn at random; every case is compared with the
CPU oracle byte for byte."""
import numpy as np
import pytest

import oracle
from paper_2605_00831_amd import inputs

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def test_random_cases_against_the_oracle():
    from paper_2605_00831_amd import binding as gs
    gs.lib()
    rng = np.random.default_rng(inputs.SEED_BASE + 0x300)
    try:
        for case in range(60):
            kind = ["cauchy", "power", "rdp"][int(rng.integers(0, 3))]
            if kind == "rdp":
                k, m = int(rng.integers(1, 17)), 2
                cell = int(2 ** rng.integers(4, 9))
                code = gs.gs_make_rdp_code(k, cell)
                S = (gs.gs_rdp_prime(code) - 1) * cell * int(rng.integers(1, 40))
            else:
                k = int(rng.integers(1, 25))
                m = int(rng.integers(1, 4 if kind == "power" else 6))
                code = gs.gs_make_code(k, m, gs.GS_POWER if kind == "power" else gs.GS_CAUCHY)
                S = int(rng.integers(1, 300000))
                P = oracle.power_generator(k, m) if kind == "power" else oracle.generator(k, m)
            gs.gs_set_launch_shape(int(rng.choice([1, 2, 4])), int(rng.integers(1, 4)), int(rng.integers(0, 2)),
                                   int(rng.integers(0, 8)))
            data_np = [inputs.uniform_bytes_np(case * 100 + j, S) for j in range(k)]
            want = oracle.rdp_encode(data_np, cell) if kind == "rdp" else oracle.encode(P, data_np, nthreads=8)
            data = [torch.from_numpy(x).cuda() for x in data_np]
            par = [torch.full((S + 32,), 0xC7, dtype=torch.uint8, device="cuda") for _ in range(m)]
            gs.gs_encode(code, data, par, S)
            torch.cuda.synchronize()
            for i in range(m):
                got = par[i].cpu().numpy()
                assert np.array_equal(got[:S], want[i]), (case, kind, k, m, S, i)
                assert (got[S:] == 0xC7).all()
            e = int(rng.integers(1, m + 1))
            pat = sorted(int(x) for x in rng.choice(k + m, size=e, replace=False))
            full = data_np + want
            shards = []
            for r in range(k + m):
                t = torch.full((S + 32,), 0xC7, dtype=torch.uint8, device="cuda")
                t[:S] = torch.from_numpy(full[r]).cuda() if r not in pat else 0xA5
                shards.append(t)
            gs.gs_reconstruct(code, shards, pat, S)
            torch.cuda.synchronize()
            for r in range(k + m):
                got = shards[r].cpu().numpy()
                assert np.array_equal(got[:S], full[r]), (case, kind, k, m, S, pat, r)
                assert (got[S:] == 0xC7).all()
    finally:
        gs.gs_set_launch_shape()


def test_random_pipeline_and_paged_cases_against_the_oracle():
    """Seeded random sweep of the chunked checkpoint / restore pipelines (chunk size, depth, shard
    length, erasure pattern) and of the paged encode / rebuild (planes, pages per shard, page sizes
    that are and are not powers of two, random tables)."""
    from paper_2605_00831_amd import binding as gs
    gs.lib()
    gs.gs_set_launch_shape()
    rng = np.random.default_rng(inputs.SEED_BASE + 0x301)
    for case in range(25):
        k, m = int(rng.integers(1, 13)), int(rng.integers(1, 5))
        code = gs.gs_make_code(k, m)
        P = oracle.generator(k, m)
        chunk = 16 * int(rng.integers(1, 3000))
        depth = int(rng.integers(2, 6))
        S = int(rng.integers(1, 12 * chunk))
        data_np = [inputs.uniform_bytes_np(70000 + case * 50 + j, S) for j in range(k)]
        want = oracle.encode(P, data_np, nthreads=8)
        data = [torch.from_numpy(x).cuda() for x in data_np]
        host = [torch.full((S + 16,), 0x5A, dtype=torch.uint8).pin_memory() for _ in range(m)]
        pipe = gs.gs_pipe_create(code, chunk, depth)
        gs.gs_checkpoint(pipe, data, S, host)
        gs.gs_pipe_sync(pipe)
        for i in range(m):
            assert np.array_equal(host[i].numpy()[:S], want[i]), (case, k, m, S, chunk, depth, i)
            assert (host[i].numpy()[S:] == 0x5A).all()
        e = int(rng.integers(1, m + 1))
        pat = sorted(int(x) for x in rng.choice(k + m, size=e, replace=False))
        shards = [d if r not in pat else torch.full((S + 16,), 0xA5, dtype=torch.uint8, device="cuda")
                  for r, d in enumerate(data)]
        shards += [torch.full((S + 16,), 0xA5, dtype=torch.uint8, device="cuda") if k + i in pat else None for i in range(m)]
        gs.gs_restore(pipe, shards, host, pat, S)
        gs.gs_pipe_sync(pipe)
        full = data_np + want
        for r in pat:
            got = shards[r].cpu().numpy()
            assert np.array_equal(got[:S], full[r]), (case, k, m, S, chunk, depth, pat, r)
            assert (got[S:] == 0xA5).all()
        gs.gs_pipe_destroy(pipe)

    for case in range(25):
        k, m = int(rng.integers(1, 10)), int(rng.integers(1, 4))
        code = gs.gs_make_code(k, m)
        P = oracle.generator(k, m)
        n_planes, pps = int(rng.integers(1, 6)), int(rng.integers(1, 20))
        page = 16 * int(rng.choice([1, 3, 4, 64, 65, 128, 200, 1024]))
        n_pages = (k + m) * pps + int(rng.integers(0, 10))
        planes_np = [inputs.uniform_bytes_np(90000 + case * 20 + p, n_pages * page) for p in range(n_planes)]
        planes = [torch.from_numpy(x).cuda() for x in planes_np]
        base = torch.tensor([x.data_ptr() for x in planes], dtype=torch.int64, device="cuda")
        ids = rng.permutation(n_pages).astype(np.int32)
        table_np = ids[: k * pps].reshape(k, pps)
        spare_np = ids[k * pps: (k + m) * pps].reshape(m, pps)       # fresh pages for rebuilt shards
        table = torch.from_numpy(np.ascontiguousarray(table_np)).cuda()
        out_bytes = n_planes * pps * page
        par = [torch.full((out_bytes + 16,), 0xC7, dtype=torch.uint8, device="cuda") for _ in range(m)]
        gs.gs_encode_paged(code, base, n_planes, page, n_pages, table, pps, par)
        torch.cuda.synchronize()
        want = oracle.encode_paged(P, planes_np, page, table_np)
        for i in range(m):
            got = par[i].cpu().numpy()
            assert np.array_equal(got[:out_bytes], want[i]), (case, k, m, n_planes, pps, page, i)
            assert (got[out_bytes:] == 0xC7).all()
        # lose one data shard: it is rebuilt into fresh pages named by a new table row
        lost = int(rng.integers(0, k))
        new_table_np = table_np.copy()
        new_table_np[lost] = spare_np[0]
        new_table = torch.from_numpy(np.ascontiguousarray(new_table_np)).cuda()
        gs.gs_reconstruct_paged(code, base, n_planes, page, n_pages, new_table, pps, par, [lost])
        torch.cuda.synchronize()
        for p in range(n_planes):
            got = planes[p].cpu().numpy().reshape(n_pages, page)
            orig = planes_np[p].reshape(n_pages, page)
            assert np.array_equal(got[new_table_np[lost]], orig[table_np[lost]]), (case, k, m, p, page, lost)
            untouched = np.setdiff1d(np.arange(n_pages), new_table_np[lost])
            assert np.array_equal(got[untouched], orig[untouched])


def test_random_grouped_and_rdp_paged_cases_against_the_oracle():
    """Seeded random sweep of the grouped launches (gs_batch, the allocation-free encode; GF(2^8), power and
    RDP codes; chunk counts, ragged and empty chunks, launch shapes, erasure patterns) and of RDP over a
    paged pool (planes, page = cell sizes, stripes per plane, random tables, encode and restore)."""
    from paper_2605_00831_amd import binding as gs
    gs.lib()
    rng = np.random.default_rng(inputs.SEED_BASE + 0x302)
    hold = torch.zeros(16, dtype=torch.uint8, device="cuda")

    def out_buf(n, fill=0xC7):
        return torch.full((n + 48,), fill, dtype=torch.uint8, device="cuda")

    def same(buf, want, fill, ctx):
        got = buf.cpu().numpy()
        assert np.array_equal(got[:want.size], want), ctx
        assert (got[want.size:] == fill).all(), ctx

    try:
        for case in range(45):
            kind = ["cauchy", "power", "rdp"][case % 3]
            k = int(rng.integers(1, 17))
            if kind == "rdp":
                m, cell = 2, int(2 ** rng.integers(4, 12))
                code = gs.gs_make_rdp_code(k, cell)
                unit = (gs.gs_rdp_prime(code) - 1) * cell
            else:
                m = int(rng.integers(1, 4 if kind == "power" else 5))
                code = gs.gs_make_code(k, m, gs.GS_POWER if kind == "power" else gs.GS_CAUCHY)
                P = oracle.power_generator(k, m) if kind == "power" else oracle.generator(k, m)
            n = int(rng.integers(1, 30))
            sizes = []
            for c in range(n):
                r = rng.random()
                if kind == "rdp":
                    sizes.append(0 if r < 0.1 else unit * int(rng.integers(1, max(2, min(100, (1 << 19) // unit)))))
                else:
                    sizes.append(0 if r < 0.1 else int(rng.integers(1, 100000 if r < 0.9 else 1500000)))
            gs.gs_set_launch_shape(int(rng.choice([1, 2, 4])), int(rng.integers(1, 4)), int(rng.integers(0, 2)),
                                   int(rng.integers(0, 8)))
            chunks = [[inputs.uniform_bytes_np(300000 + case * 1000 + c * 20 + j, S) for j in range(k)]
                      for c, S in enumerate(sizes)]
            want = [([np.zeros(0, np.uint8)] * m if S == 0 else
                     oracle.rdp_encode(ch, cell) if kind == "rdp" else oracle.encode(P, ch, nthreads=8))
                    for ch, S in zip(chunks, sizes)]
            data = [[torch.from_numpy(x).cuda() if x.size else hold for x in ch] for ch in chunks]
            par = [[out_buf(S) for _ in range(m)] for S in sizes]
            batch = gs.gs_batch_create(code, n + int(rng.integers(0, 3)))
            static = kind != "rdp" and case % 2 == 0
            if static:
                gs.gs_encode_batch_static(code, data, par, sizes)
            else:
                gs.gs_encode_batch(batch, data, par, sizes)
            torch.cuda.synchronize()
            for c in range(n):
                for i in range(m):
                    same(par[c][i], want[c][i], 0xC7, (case, kind, k, m, sizes, c, i, static))
            pat = sorted(int(x) for x in rng.choice(k + m, size=int(rng.integers(1, m + 1)), replace=False))
            shards = []
            for c, S in enumerate(sizes):
                full = chunks[c] + want[c]
                row = []
                for r in range(k + m):
                    if r in pat:
                        t = out_buf(S)
                        t[:S] = 0xA5
                    else:
                        t = torch.from_numpy(full[r]).cuda() if S else hold
                    row.append(t)
                shards.append(row)
            gs.gs_reconstruct_batch(batch, shards, pat, sizes)
            torch.cuda.synchronize()
            for c in range(n):
                for r in pat:
                    same(shards[c][r], (chunks[c] + want[c])[r], 0xC7, (case, kind, k, m, sizes, pat, c, r))
            gs.gs_batch_destroy(batch)

        for case in range(20):
            k, n_planes = int(rng.integers(1, 17)), int(rng.integers(1, 6))
            page = int(2 ** rng.integers(10, 14))
            code = gs.gs_make_rdp_code(k, page)
            rows = gs.gs_rdp_prime(code) - 1
            pps = rows * int(rng.integers(1, 5))
            n_pages = (k + 2) * pps + int(rng.integers(0, 10))
            planes_np = [inputs.uniform_bytes_np(400000 + case * 20 + p, n_pages * page) for p in range(n_planes)]
            pool = torch.from_numpy(np.concatenate(planes_np)).cuda()
            base = torch.tensor([pool.data_ptr() + p * n_pages * page for p in range(n_planes)], dtype=torch.int64,
                                device="cuda")
            table_np = np.ascontiguousarray(rng.permutation(n_pages).astype(np.int32)[: k * pps].reshape(k, pps))
            table = torch.from_numpy(table_np).cuda()
            S = n_planes * pps * page
            # a shard's byte stream: plane by plane, slot by slot; stripes never cross a plane
            streams = [np.concatenate([pl.reshape(n_pages, page)[table_np[j]].reshape(-1) for pl in planes_np])
                       for j in range(k)]
            want = oracle.rdp_encode(streams, page)
            gs.gs_set_launch_shape(int(rng.choice([1, 2])), 1, int(rng.integers(0, 2)), int(rng.integers(0, 8)))
            par = [out_buf(S) for _ in range(2)]
            gs.gs_encode_paged(code, base, n_planes, page, n_pages, table, pps, par)
            torch.cuda.synchronize()
            for i in range(2):
                same(par[i], want[i], 0xC7, (case, k, n_planes, page, pps, i))
            spc = max(rows, int(rng.integers(1, pps + 3)) // rows * rows)
            pipe = gs.gs_pipe_create(code, n_planes * page * spc, int(rng.integers(2, 4)))
            host = [torch.full((S + 16,), 0x5A, dtype=torch.uint8).pin_memory() for _ in range(2)]
            gs.gs_checkpoint_paged(pipe, base, n_planes, page, n_pages, table, pps, host)
            gs.gs_pipe_sync(pipe)
            for i in range(2):
                assert np.array_equal(host[i].numpy()[:S], want[i]), (case, k, n_planes, page, pps, spc, i)
                assert (host[i].numpy()[S:] == 0x5A).all()
            pat = sorted(int(x) for x in rng.choice(k + 2, size=int(rng.integers(1, 3)), replace=False))
            view = pool.view(n_planes, n_pages, page)
            for r in pat:
                if r < k:
                    view[:, torch.from_numpy(table_np[r].astype(np.int64)).cuda(), :] = 0xA5
                else:
                    host[r - k].fill_(0xA5)      # a lost parity shard must not be read
            out = [out_buf(S, 0xC3) for _ in range(2)]
            gs.gs_restore_paged(pipe, base, n_planes, page, n_pages, table, pps, host, pat, parity_out=out)
            gs.gs_pipe_sync(pipe)
            torch.cuda.synchronize()
            assert np.array_equal(pool.cpu().numpy(), np.concatenate(planes_np)), (case, k, n_planes, page, pps, spc, pat)
            for i in range(2):
                if k + i in pat:
                    same(out[i], want[i], 0xC3, (case, k, pat, i))
            gs.gs_pipe_destroy(pipe)
    finally:
        gs.gs_set_launch_shape()


def test_random_bulk_size_cases_against_the_oracle():
    """The kernel forms of launches that fill the chip (one stream at a time, LDS reservation from 48 MiB
    shards on, rebuilds of three and four shards with a folded XOR row): random code, length between
    9 and 70 MiB with a ragged end, default launch shape, random loss pattern; encode against the oracle,
    the rebuilt shards against the stripe."""
    from paper_2605_00831_amd import binding as gs
    gs.lib()
    gs.gs_set_launch_shape()
    rng = np.random.default_rng(inputs.SEED_BASE + 0x340)
    for case in range(12):
        kind = ["cauchy", "power", "rdp"][int(rng.integers(0, 3))]
        if kind == "rdp":
            k, m = int(rng.integers(2, 13)), 2
            cell = 4096
            code = gs.gs_make_rdp_code(k, cell)
            unit = (gs.gs_rdp_prime(code) - 1) * cell
            S = unit * int(rng.integers((9 << 20) // unit + 1, (70 << 20) // unit))
        else:
            k = int(rng.integers(2, 13))
            m = int(rng.integers(1, 4 if kind == "power" else 5))
            code = gs.gs_make_code(k, m, gs.GS_POWER if kind == "power" else gs.GS_CAUCHY)
            S = int(rng.integers(9 << 20, 70 << 20)) | 1
            P = oracle.power_generator(k, m) if kind == "power" else oracle.generator(k, m)
        data_np = [inputs.uniform_bytes_np(7000 + case * 100 + j, S) for j in range(k)]
        want = oracle.rdp_encode(data_np, cell) if kind == "rdp" else oracle.encode(P, data_np, nthreads=8)
        good = [torch.cat([torch.from_numpy(x).cuda(), torch.full((32,), 0xC7, dtype=torch.uint8, device="cuda")])
                for x in data_np + want]
        par = [torch.full((S + 32,), 0xC7, dtype=torch.uint8, device="cuda") for _ in range(m)]
        gs.gs_encode(code, good[:k], par, S)
        for i in range(m):
            assert torch.equal(par[i], good[k + i]), (case, kind, k, m, S, i)
        for _ in range(3):
            e = int(rng.integers(1, m + 1))
            pat = sorted(int(x) for x in rng.choice(k + m, size=e, replace=False))
            shards = [g.clone() for g in good]
            for r in pat:
                shards[r][:S] = 0xA5
            gs.gs_reconstruct(code, shards, pat, S)
            for r in range(k + m):
                assert torch.equal(shards[r], good[r]), (case, kind, k, m, S, pat, r)
