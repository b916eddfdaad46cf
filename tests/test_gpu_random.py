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
