"""The power code (P[i][j] = 2^(i*j)): oracle matrix pinned by repeated
multiplication with the independent multiply and by exhaustive MDS checks;
the library must build the same matrix, and refuse m > 3 where the matrix
stops being MDS."""
import itertools

import numpy as np
import pytest

import oracle
from paper_2605_00831_amd import binding as gs
from paper_2605_00831_amd import inputs
from tests import _gfref


def power_by_repeated_multiplication(k, m):
    P = np.zeros((m, k), np.uint8)
    for i in range(m):
        g = 1
        for _ in range(i):
            g = _gfref.clmul_reduce(g, 2)
        v = 1
        for j in range(k):
            P[i, j] = v
            v = _gfref.clmul_reduce(v, g)
    return P


@pytest.mark.parametrize("k,m", [(1, 1), (4, 2), (8, 3), (100, 3), (253, 3), (255, 1)])
def test_matrix(k, m):
    want = power_by_repeated_multiplication(k, m)
    assert np.array_equal(oracle.power_generator(k, m), want)
    assert np.array_equal(gs.gs_code_matrix(gs.gs_make_code(k, m, gs.GS_POWER)), want)
    assert (want[0] == 1).all() and (want[:, 0] == 1).all()


def test_mds_exhaustive_small_and_sampled_wide():
    for n in range(2, 11):
        for m in range(1, min(3, n - 1) + 1):
            k = n - m
            G = np.vstack([np.eye(k, dtype=np.uint8), oracle.power_generator(k, m)])
            for rows in itertools.combinations(range(n), k):
                assert _gfref.mat_rank(G[list(rows)]) == k
    # wide code: every 3x3 minor that involves the far columns is non-zero (sampled)
    P = oracle.power_generator(255, 3)
    rng = np.random.default_rng(2)
    for _ in range(300):
        cols = sorted(rng.choice(255, size=3, replace=False))
        assert _gfref.mat_rank(P[:, cols]) == 3
    # with a fourth row the matrix is singular on columns {0, 85}: why m stops at 3
    four = power_by_repeated_multiplication(86, 4)
    assert _gfref.mat_rank(four[[0, 3]][:, [0, 85]]) == 1


def test_limits():
    for k, m in [(4, 4), (256, 1), (0, 2)]:
        with pytest.raises(gs.GsError):
            gs.gs_make_code(k, m, gs.GS_POWER)
        with pytest.raises(ValueError):
            oracle.power_generator(k, m)


def test_decode_matrix_matches_oracle():
    for k, m in [(4, 2), (8, 3)]:
        code = gs.gs_make_code(k, m, gs.GS_POWER)
        P = oracle.power_generator(k, m)
        for pat in inputs.all_erasure_patterns(k + m, m, 1):
            R, surv = gs.gs_decode_matrix(code, list(pat))
            Ro, so = oracle.decode_matrix(P, list(pat))
            assert surv == so and np.array_equal(R, Ro)


@pytest.mark.gpu
def test_power_code_on_the_gpu():
    torch = pytest.importorskip("torch")
    for k, m, S in [(4, 2, 70001), (8, 3, (1 << 20) + 48), (40, 3, 5000)]:
        code = gs.gs_make_code(k, m, gs.GS_POWER)
        P = oracle.power_generator(k, m)
        data_np = [inputs.uniform_bytes_np(3 * k + j, S) for j in range(k)]
        want = oracle.encode(P, data_np, nthreads=8)
        data = [torch.from_numpy(x).cuda() for x in data_np]
        par = [torch.zeros(S, dtype=torch.uint8, device="cuda") for _ in range(m)]
        gs.gs_encode(code, data, par, S)
        torch.cuda.synchronize()
        for i in range(m):
            assert np.array_equal(par[i].cpu().numpy(), want[i])
        lost = list(range(m))                       # lose the first m data shards
        for r in lost:
            data[r].fill_(0xA5)
        gs.gs_reconstruct(code, data + par, lost, S)
        torch.cuda.synchronize()
        for r in lost:
            assert np.array_equal(data[r].cpu().numpy(), data_np[r])
        work = data_np + want
        work = [x.copy() for x in work]
        for r in lost:
            work[r][:] = 0
        oracle.reconstruct(P, work, lost)
        for r in lost:
            assert np.array_equal(work[r], data_np[r])


HORNER_SIZES = [1, 15, 16, 17, 4095, 8192, 70001, 256 * 32 * 32 * 2 + 48 + 7, (3 << 20) + 5]


@pytest.mark.gpu
@pytest.mark.parametrize("k,m", [(1, 2), (2, 2), (4, 2), (5, 3), (8, 3), (13, 2), (16, 3)])
def test_horner_encode_equals_oracle_and_matrix_kernel(k, m):
    """The Horner kernel (default for power codes with m >= 2, k <= 16) against the oracle's
    matrix encode, at sizes from one byte to several interleaved super-tiles with ragged ends,
    for one and two vectors per lane; canaries after every parity buffer; and the same bytes
    from the general matrix kernel with the Horner path switched off."""
    torch = pytest.importorskip("torch")
    code = gs.gs_make_code(k, m, gs.GS_POWER)
    P = oracle.power_generator(k, m)
    pad, canary = 64, 0x3C
    try:
        for S in HORNER_SIZES:
            data_np = [inputs.uniform_bytes_np(7000 + 17 * k + j, S) for j in range(k)]
            want = oracle.encode(P, data_np, nthreads=8)
            data = [torch.from_numpy(np.concatenate([x, np.zeros((-S) % 16, np.uint8)])).cuda() for x in data_np]
            for unroll in (1, 2):
                gs.gs_set_launch_shape(unroll=unroll)
                for horner in (True, False):
                    gs.gs_set_power_horner(horner)
                    par = [torch.full((S + pad,), canary, dtype=torch.uint8, device="cuda") for _ in range(m)]
                    gs.gs_encode(code, data, par, S)
                    torch.cuda.synchronize()
                    for i in range(m):
                        got = par[i].cpu().numpy()
                        assert np.array_equal(got[:S], want[i]), (k, m, S, unroll, horner, i)
                        assert (got[S:] == canary).all(), (k, m, S, unroll, horner, i)
    finally:
        gs.gs_set_power_horner(True)
        gs.gs_set_launch_shape()


@pytest.mark.gpu
def test_horner_in_the_checkpoint_pipeline():
    """gs_checkpoint encodes through gs_encode, so a power code takes the Horner kernel there too."""
    torch = pytest.importorskip("torch")
    k, m, S, chunk = 8, 2, (5 << 16) + 4096 + 80, 1 << 16
    code = gs.gs_make_code(k, m, gs.GS_POWER)
    P = oracle.power_generator(k, m)
    data_np = [inputs.uniform_bytes_np(8100 + j, S) for j in range(k)]
    want = oracle.encode(P, data_np, nthreads=8)
    data = [torch.from_numpy(x).cuda() for x in data_np]
    host = [torch.zeros(S, dtype=torch.uint8, pin_memory=True) for _ in range(m)]
    pipe = gs.gs_pipe_create(code, chunk, 2)
    gs.gs_checkpoint(pipe, data, S, host)
    gs.gs_pipe_sync(pipe)
    for i in range(m):
        assert np.array_equal(host[i].numpy(), want[i])
    gs.gs_pipe_destroy(pipe)
