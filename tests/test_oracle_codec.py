"""Pins for the oracle's encode, paged encode, decode matrix and reconstruct.

Expected values come from definitions the paper fixes (XOR parity for one
parity shard, Section 2; recovery from up to K losses and lossless
reinterpretation of FP16, Section 4.1; bounds on the partial last chunk,
Section 4.2 "Overall Workflow") or from an independent numpy encode built on
the carry-less multiply in tests/_gfref.py.
"""
import itertools

import numpy as np
import pytest

import oracle
from paper_2605_00831_amd import inputs
from tests import _gfref


def _rand_shards(seed, k, S):
    return [inputs.uniform_bytes_np(seed * 131 + j, S) for j in range(k)]


@pytest.mark.parametrize("k", [1, 2, 4, 8, 13])
def test_single_parity_is_byte_xor(k):
    data = _rand_shards(3, k, 4099)
    (par,) = oracle.encode(oracle.generator(k, 1), data)
    assert np.array_equal(par, np.bitwise_xor.reduce(np.stack(data), axis=0))


@pytest.mark.parametrize("k,m", [(4, 2), (8, 2), (8, 3), (5, 3), (3, 4)])
def test_row0_is_xor_and_encode_matches_independent_table_encode(k, m):
    data = _rand_shards(5, k, 10007)
    P = oracle.generator(k, m)
    par = oracle.encode(P, data)
    assert np.array_equal(par[0], np.bitwise_xor.reduce(np.stack(data), axis=0))
    want = _gfref.encode_np(_gfref.cauchy_normalised(k, m), data)
    for i in range(m):
        assert np.array_equal(par[i], want[i])


def test_worked_example_k4_m2():
    # data byte d_j[t] = (17 j + 29 t + 1) mod 256, t < 8
    data = [np.array([(17 * j + 29 * t + 1) % 256 for t in range(8)], np.uint8) for j in range(4)]
    assert [bytes(d).hex() for d in data] == ["011e3b587592afcc", "122f4c6986a3c0dd",
                                              "23405d7a97b4d1ee", "34516e8ba8c5e2ff"]
    par = oracle.encode(oracle.generator(4, 2), data)
    # par0 is the XOR of the four rows; par1 uses the row 01 d9 5c ac
    assert bytes(par[0]).hex() == "042044c0cc405c00"
    want1 = bytes(
        d0 ^ _gfref.clmul_reduce(0xD9, d1) ^ _gfref.clmul_reduce(0x5C, d2) ^ _gfref.clmul_reduce(0xAC, d3)
        for d0, d1, d2, d3 in zip(*[d.tolist() for d in data]))
    assert bytes(par[1]) == want1
    assert want1.hex() == "a8e7cc0bad1a9076"


def test_linearity_zero_and_impulse():
    k, m, S = 6, 3, 513
    P = oracle.generator(k, m)
    a, b = _rand_shards(11, k, S), _rand_shards(12, k, S)
    pa, pb = oracle.encode(P, a), oracle.encode(P, b)
    pab = oracle.encode(P, [x ^ y for x, y in zip(a, b)])
    for i in range(m):
        assert np.array_equal(pab[i], pa[i] ^ pb[i])
    assert not any(p.any() for p in oracle.encode(P, [np.zeros(S, np.uint8)] * k))
    # a single 0x01 in shard j at offset t reads out column j of P at offset t
    for j in range(k):
        data = [np.zeros(S, np.uint8) for _ in range(k)]
        data[j][j * 7 + 3] = 1
        par = oracle.encode(P, data)
        for i in range(m):
            want = np.zeros(S, np.uint8)
            want[j * 7 + 3] = P[i, j]
            assert np.array_equal(par[i], want)


def test_xor_fold_commutes_with_encode():
    k, m, S, F = 4, 2, 8 * 256, 256
    P = oracle.generator(k, m)
    data = _rand_shards(21, k, S)
    par = oracle.encode(P, data)
    fold = lambda x: np.bitwise_xor.reduce(x.reshape(-1, F), axis=0)
    pf = oracle.encode(P, [np.ascontiguousarray(fold(d)) for d in data])
    for i in range(m):
        assert np.array_equal(fold(par[i]), pf[i])


def test_encode_touches_nothing_past_shard_bytes():
    # parity arrays are allocated by the wrapper with exactly S bytes; run the C
    # entry directly on padded buffers and check the canaries
    import ctypes
    k, m, S = 3, 2, 37
    P = oracle.generator(k, m)
    data = _rand_shards(31, k, S + 16)
    bufs = [np.full(S + 16, 0xEE, np.uint8) for _ in range(m)]
    L = oracle.lib()
    u8p = ctypes.POINTER(ctypes.c_uint8)
    dp = (u8p * k)(*[d.ctypes.data_as(u8p) for d in data])
    pp = (u8p * m)(*[b.ctypes.data_as(u8p) for b in bufs])
    L.gso_encode(k, m, P.ctypes.data_as(u8p), dp, pp, S)
    want = oracle.encode(P, [np.ascontiguousarray(d[:S]) for d in data])
    for i in range(m):
        assert np.array_equal(bufs[i][:S], want[i])
        assert (bufs[i][S:] == 0xEE).all()


def test_multithreaded_encode_equals_single_thread():
    k, m, S = 4, 2, 100003
    P = oracle.generator(k, m)
    data = _rand_shards(41, k, S)
    one = oracle.encode(P, data)
    for nt in (2, 3, 8):
        many = oracle.encode(P, data, nthreads=nt)
        for i in range(m):
            assert np.array_equal(one[i], many[i])


# ------------------------------------------------------------------ reconstruct

def _stripe(seed, k, m, S, dtype=None):
    if dtype:
        buf = inputs.kv_bytes_np(seed, k * S, dtype, 1.0)
        inputs.plant_specials(buf, dtype, seed)
        data = [np.ascontiguousarray(x) for x in inputs.split_shards(buf, k)]
    else:
        data = _rand_shards(seed, k, S)
    P = oracle.generator(k, m)
    # parity from the independent encoder, so the round trip is not self-referential
    par = _gfref.encode_np(_gfref.cauchy_normalised(k, m), data)
    return P, data + par


def test_round_trip_every_erasure_subset_small_codes():
    """Encode, erase every subset of <= m shards (data and parity alike),
    reconstruct, compare -- for every code with k+m <= 9."""
    for n in range(2, 10):
        for m in range(1, n):
            k = n - m
            P, full = _stripe(100 + n * 16 + m, k, m, 61)
            for pat in inputs.all_erasure_patterns(n, m):
                work = [s.copy() for s in full]
                for r in pat:
                    work[r][:] = 0xA5
                oracle.reconstruct(P, work, list(pat))
                for r in range(n):
                    assert np.array_equal(work[r], full[r]), (k, m, pat, r)


def test_round_trip_all_165_triples_of_the_8_3_code():
    P, full = _stripe(5, 8, 3, 1029)
    for pat in itertools.combinations(range(11), 3):
        work = [s.copy() for s in full]
        for r in pat:
            work[r][:] = 0xA5
        oracle.reconstruct(P, work, list(pat))
        for r in range(11):
            assert np.array_equal(work[r], full[r]), (pat, r)


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
def test_reconstruction_is_lossless_for_float_bit_patterns(dtype):
    """Section 4.1: the integer reinterpretation is reversible -- NaN payloads,
    infinities, signed zeros and denormals come back bit for bit."""
    P, full = _stripe(77, 4, 2, 2048, dtype)
    work = [s.copy() for s in full]
    for r in (1, 3):
        work[r][:] = 0xA5
    oracle.reconstruct(P, work, [1, 3])
    for r in range(6):
        assert np.array_equal(work[r].view(np.int16), full[r].view(np.int16))
    # the planted patterns really are in the stripe
    allv = np.concatenate([s.view(np.uint16) for s in full[:4]])
    for pat in inputs.special_bits(dtype):
        assert (allv == pat).any()


def test_decode_matrix_definition():
    """R must map the k lowest-indexed survivors to the lost shards:
    check R against G algebraically with the independent matmul."""
    for k, m in [(4, 2), (8, 3), (5, 3), (2, 4)]:
        P = oracle.generator(k, m)
        G = np.vstack([np.eye(k, dtype=np.uint8), P])
        for pat in inputs.all_erasure_patterns(k + m, m, 1):
            R, surv = oracle.decode_matrix(P, list(pat))
            assert surv == [r for r in range(k + m) if r not in pat][:k]
            # R * G[surv] must equal G[lost]   (both sides applied to any data vector)
            assert np.array_equal(_gfref.matmul(R, G[surv]), G[list(pat)]), (k, m, pat)


def test_known_rebuild_matrices():
    R, surv = oracle.decode_matrix(oracle.generator(4, 2), [1, 3])
    assert surv == [0, 2, 4, 5]
    assert [bytes(r).hex() for r in R] == ["f5690efb", "f4680ffb"]
    R, surv = oracle.decode_matrix(oracle.generator(8, 3), [2, 5, 9])
    assert surv == [0, 1, 3, 4, 6, 7, 8, 10]
    assert [bytes(r).hex() for r in R] == ["d2f0c7f8697963b1", "d3f1c6f9687862b1", "cd75b0f2e60bda16"]


def test_survivor_choice_does_not_change_the_bytes():
    """With fewer than m losses more than k shards survive; any k of them give
    the same rebuilt bytes.  Drop an extra (intact) shard from the survivor set
    by declaring it erased too, and compare."""
    P, full = _stripe(9, 5, 3, 257)
    base = [s.copy() for s in full]
    base[2][:] = 0
    oracle.reconstruct(P, base, [2])
    for extra in (0, 4, 5, 7):
        work = [s.copy() for s in full]
        work[2][:] = 0
        work[extra][:] = 0
        oracle.reconstruct(P, work, [2, extra])
        assert np.array_equal(work[2], base[2]) and np.array_equal(work[2], full[2])
        assert np.array_equal(work[extra], full[extra])


def test_erasure_list_errors_and_noop():
    P, full = _stripe(13, 4, 2, 33)
    work = [s.copy() for s in full]
    oracle.reconstruct(P, work, [])
    assert all(np.array_equal(a, b) for a, b in zip(work, full))
    with pytest.raises(OverflowError):
        oracle.reconstruct(P, work, [0, 1, 2])
    for bad in ([0, 0], [6], [-1]):
        with pytest.raises(ValueError):
            oracle.reconstruct(P, work, bad)
    assert all(np.array_equal(a, b) for a, b in zip(work, full))


def test_survivors_are_never_written():
    P, full = _stripe(17, 8, 3, 130)
    work = [s.copy() for s in full]
    for r in (0, 9):
        work[r][:] = 0xA5
    oracle.reconstruct(P, work, [0, 9])
    for r in range(11):
        assert np.array_equal(work[r], full[r])


# ------------------------------------------------------------------ paged

@pytest.mark.parametrize("k,m,n_planes,pps,page_bytes", [(4, 1, 3, 5, 64), (4, 2, 2, 16, 2048),
                                                         (3, 3, 1, 7, 48), (8, 2, 4, 3, 512)])
def test_paged_encode_equals_encode_of_explicit_gather(k, m, n_planes, pps, page_bytes):
    num_pages = k * pps + 9
    planes = [inputs.kv_bytes_np(900 + p, num_pages * page_bytes, "bf16", 1.0) for p in range(n_planes)]
    table = inputs.block_table_np(55, k, pps, num_pages)
    P = oracle.generator(k, m)
    got = oracle.encode_paged(P, planes, page_bytes, table)
    # gather with numpy fancy indexing: shard j = for each plane, its pages in table order
    gathered = []
    for j in range(k):
        parts = [pl.reshape(num_pages, page_bytes)[table[j]].reshape(-1) for pl in planes]
        gathered.append(np.ascontiguousarray(np.concatenate(parts)))
    want = _gfref.encode_np(_gfref.cauchy_normalised(k, m), gathered)
    for i in range(m):
        assert np.array_equal(got[i], want[i])


def test_paged_identity_table_reduces_to_contiguous():
    k, m, pps, page_bytes = 4, 2, 8, 128
    plane = inputs.uniform_bytes_np(4, k * pps * page_bytes)
    table = np.arange(k * pps, dtype=np.int32).reshape(k, pps)
    P = oracle.generator(k, m)
    got = oracle.encode_paged(P, [plane], page_bytes, table)
    want = oracle.encode(P, [np.ascontiguousarray(s) for s in inputs.split_shards(plane, k)])
    for i in range(m):
        assert np.array_equal(got[i], want[i])
