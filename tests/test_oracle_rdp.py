"""Pins for the RDP oracle (row-diagonal parity; the paper's Section 2 cites
it as the XOR-only code that survives any two simultaneous shard failures).

What fixes the expected values here: row parity is the plain XOR of the data;
the code must be MDS for two erasures -- checked (a) by reading the code's
generator out with impulses and testing, with an independent GF(2)
elimination, that the surviving symbols determine the data under every pair of
lost disks, and (b) by exhaustive search for completions on small stripes --
and reconstruction must return the original bytes for every pair of disks."""
import itertools

import numpy as np
import pytest

import oracle
from paper_2605_00831_amd import inputs


def gf2_rank(M):
    M = (np.array(M, dtype=np.uint8) & 1).copy()
    rank = 0
    rows, cols = M.shape
    for c in range(cols):
        piv = None
        for r in range(rank, rows):
            if M[r, c]:
                piv = r
                break
        if piv is None:
            continue
        M[[rank, piv]] = M[[piv, rank]]
        for r in range(rows):
            if r != rank and M[r, c]:
                M[r] ^= M[rank]
        rank += 1
    return rank


def test_prime_choice():
    assert [oracle.rdp_prime(k) for k in (1, 2, 3, 4, 5, 6, 7, 8, 10, 11, 12, 16)] == \
        [3, 3, 5, 5, 7, 7, 11, 11, 11, 13, 13, 17]


@pytest.mark.parametrize("k", [1, 2, 4, 6, 8, 10, 16])
def test_row_parity_is_xor_and_length_must_divide(k):
    p = oracle.rdp_prime(k)
    S = (p - 1) * 37
    data = [inputs.uniform_bytes_np(3 * k + j, S) for j in range(k)]
    par = oracle.rdp_encode(data)
    assert np.array_equal(par[0], np.bitwise_xor.reduce(np.stack(data), axis=0))
    with pytest.raises(ValueError):
        oracle.rdp_encode([d[:S - 1].copy() for d in data])


@pytest.mark.parametrize("k", [2, 3, 4, 6, 8, 10])
def test_generator_read_out_by_impulses_is_mds_for_two_erasures(k):
    """One bit per block: encode unit vectors to get the (k+2)(p-1) x k(p-1)
    generator over GF(2); losing any two disks must leave full column rank."""
    p = oracle.rdp_prime(k)
    rows = p - 1
    n_in = k * rows
    G = np.zeros(((k + 2) * rows, n_in), np.uint8)
    for j in range(k):
        for i in range(rows):
            data = [np.zeros(rows, np.uint8) for _ in range(k)]
            data[j][i] = 1
            par = oracle.rdp_encode(data)
            col = np.concatenate(data + par)
            G[:, j * rows + i] = col
    # systematic part is the identity
    assert np.array_equal(G[:n_in], np.eye(n_in, dtype=np.uint8))
    # linear: a random bit vector encodes to G @ x over GF(2)
    rng = np.random.default_rng(k)
    x = rng.integers(0, 2, n_in, dtype=np.uint8)
    data = [np.ascontiguousarray(x[j * rows:(j + 1) * rows]) for j in range(k)]
    par = oracle.rdp_encode(data)
    assert np.array_equal(np.concatenate(data + par), (G.astype(np.int64) @ x) % 2)
    for a, b in itertools.combinations(range(k + 2), 2):
        keep = [r for d in range(k + 2) if d not in (a, b) for r in range(d * rows, (d + 1) * rows)]
        assert gf2_rank(G[keep]) == n_in, (k, a, b)
    # and it is not 3-erasure tolerant (it has only two parity disks)
    keep = [r for d in range(3, k + 2) for r in range(d * rows, (d + 1) * rows)]
    if k >= 3:
        assert gf2_rank(G[keep]) < n_in


@pytest.mark.parametrize("k", [2, 4])
def test_exhaustive_search_finds_exactly_one_completion(k):
    """Smallest stripes, one bit per block: with two data disks gone, try every
    assignment of their bits; exactly one is consistent with both parities."""
    p = oracle.rdp_prime(k)
    rows = p - 1
    rng = np.random.default_rng(40 + k)
    for trial in range(3):
        data = [rng.integers(0, 2, rows, dtype=np.uint8) for _ in range(k)]
        par = oracle.rdp_encode(data)
        for a, b in itertools.combinations(range(k), 2):
            hits = []
            for bits in itertools.product((0, 1), repeat=2 * rows):
                cand = [d.copy() for d in data]
                cand[a] = np.array(bits[:rows], np.uint8)
                cand[b] = np.array(bits[rows:], np.uint8)
                cp = oracle.rdp_encode(cand)
                if np.array_equal(cp[0], par[0]) and np.array_equal(cp[1], par[1]):
                    hits.append(bits)
            assert len(hits) == 1
            assert hits[0] == tuple(data[a]) + tuple(data[b])


@pytest.mark.parametrize("k", list(range(1, 17)))
def test_round_trip_every_single_and_double_erasure(k):
    p = oracle.rdp_prime(k)
    S = (p - 1) * 16 + 0
    data = [inputs.kv_bytes_np(50 * k + j, S, "bf16", 1.0) for j in range(k)]
    full = [d.copy() for d in data] + oracle.rdp_encode(data)
    pats = [()] + list(itertools.combinations(range(k + 2), 1)) + list(itertools.combinations(range(k + 2), 2))
    for pat in pats:
        for order in (pat, pat[::-1]):
            work = [x.copy() for x in full]
            for r in order:
                work[r][:] = 0xA5
            oracle.rdp_reconstruct(work, list(order))
            for r in range(k + 2):
                assert np.array_equal(work[r], full[r]), (k, order, r)


@pytest.mark.parametrize("k,cell", [(4, 16), (8, 8), (3, 1), (10, 32)])
def test_stripes_are_independent_and_laid_out_one_after_the_other(k, cell):
    """A shard of T stripes encodes to the concatenation of the T one-stripe
    encodings, and reconstructs stripe by stripe."""
    p = oracle.rdp_prime(k)
    T, stripe = 5, (p - 1) * cell
    data = [inputs.uniform_bytes_np(7 * k + j, T * stripe) for j in range(k)]
    par = oracle.rdp_encode(data, cell)
    for t in range(T):
        one = oracle.rdp_encode([np.ascontiguousarray(d[t * stripe:(t + 1) * stripe]) for d in data])
        assert np.array_equal(par[0][t * stripe:(t + 1) * stripe], one[0])
        assert np.array_equal(par[1][t * stripe:(t + 1) * stripe], one[1])
    full = data + par
    for pat in [(0, 1), (k - 1, k), (0, k + 1), (k, k + 1), (k - 1,)]:
        work = [x.copy() for x in full]
        for r in pat:
            work[r][:] = 0xA5
        oracle.rdp_reconstruct(work, list(pat), cell)
        for r in range(k + 2):
            assert np.array_equal(work[r], full[r]), (pat, r)
    with pytest.raises(ValueError):
        oracle.rdp_encode([d[:-1].copy() for d in data], cell)


def test_reconstruct_errors():
    data = [inputs.uniform_bytes_np(j, 64) for j in range(4)]
    full = data + oracle.rdp_encode(data)
    with pytest.raises(OverflowError):
        oracle.rdp_reconstruct([x.copy() for x in full], [0, 1, 2])
    for bad in ([0, 0], [6], [-1]):
        with pytest.raises(ValueError):
            oracle.rdp_reconstruct([x.copy() for x in full], bad)


# ---------------------------------------------------------------------------
# Pins of the diagonal-parity CONVENTION.  The tests above hold for any
# consistent 2-erasure-MDS array code; the ones below fix which one this is,
# from the published RDP construction written out cell by cell (Section 2 and
# Section 4.1 of the paper name RDP; the construction is the cited
# publication's, which is not available here to read against -- these values
# follow from its definition as restated in the oracle's header: disks 0..p-2
# data, disk p-1 row parity, cell (i, j) of those p disks on diagonal
# (i+j) mod p, diagonal p-1 not stored, Q[d] = XOR of diagonal d).
# None of the expected values below comes from the oracle.

def test_hand_worked_stripe_p3():
    """k = 2, p = 3: two rows; disks 0, 1 data, disk 2 row parity R.
         row 0:  a=01  c=04 | R0 = a^c = 05
         row 1:  b=02  d=08 | R1 = b^d = 0a
       diagonal of (i, j) is (i+j) mod 3:
         diagonal 0 = {(0,0), (1,2)}         -> Q0 = a ^ R1 = 01 ^ 0a = 0b
         diagonal 1 = {(0,1), (1,0)}         -> Q1 = c ^ b  = 04 ^ 02 = 06
         diagonal 2 = {(0,2), (1,1)}         not stored
    """
    d0 = np.array([0x01, 0x02], np.uint8)
    d1 = np.array([0x04, 0x08], np.uint8)
    R, Q = oracle.rdp_encode([d0, d1])
    assert R.tolist() == [0x05, 0x0A]
    assert Q.tolist() == [0x0B, 0x06]


def test_hand_worked_stripe_p5():
    """k = 4, p = 5: four rows, cells of two bytes; data cell (row i, disk j)
    holds the 16-bit word with only bit 4j+i set (little-endian), so every
    parity word lists the data cells it covers.
      row parity  R[i] = bits {i, 4+i, 8+i, 12+i} = 0x1111 << i
      diagonal d  = cells (i, j), i <= 3, j <= 4 (j = 4 is the row-parity disk), i+j = d mod 5:
        d=0: (0,0) (2,3) (3,2) + R[1]:  0001 ^ 4000 ^ 0800 ^ 2222 = 6a23
        d=1: (0,1) (1,0) (3,3) + R[2]:  0010 ^ 0002 ^ 8000 ^ 4444 = c456
        d=2: (0,2) (1,1) (2,0) + R[3]:  0100 ^ 0020 ^ 0004 ^ 8888 = 89ac
        d=3: (0,3) (1,2) (2,1) (3,0) :  1000 ^ 0200 ^ 0040 ^ 0008 = 1248   (row 4 of disk 4 does not exist)
        d=4: (0,4) (1,3) (2,2) (3,1)    not stored
    """
    data = [np.array([1 << (4 * j + i) for i in range(4)], dtype="<u2").view(np.uint8).copy() for j in range(4)]
    R, Q = oracle.rdp_encode(data)
    assert R.view("<u2").tolist() == [0x1111, 0x2222, 0x4444, 0x8888]
    assert Q.view("<u2").tolist() == [0x6A23, 0xC456, 0x89AC, 0x1248]


def rdp_by_definition(data, cell, direction=+1, with_row_parity_disk=True, unstored=None):
    """Row and diagonal parity written straight from the definition with numpy,
    stripe by stripe; never calls the oracle.  The keyword arguments exist only
    to build WRONG variants (flipped diagonal direction, row-parity disk left
    out of the diagonals, another diagonal left unstored) that the pins must
    tell apart from the real convention."""
    k = len(data)
    p = next(q for q in range(max(3, k + 1), 300) if all(q % f for f in range(2, q)))
    rows = p - 1
    unstored = p - 1 if unstored is None else unstored
    stored = [d for d in range(p) if d != unstored]      # diagonal stored in cell stored.index(d)
    stripes = data[0].size // (rows * cell)
    D = np.zeros((stripes, rows, p, cell), np.uint8)     # [stripe][row][disk 0..p-1][byte]
    for j in range(k):
        D[:, :, j, :] = data[j].reshape(stripes, rows, cell)
    D[:, :, p - 1, :] = np.bitwise_xor.reduce(D[:, :, :p - 1, :], axis=2)
    Q = np.zeros((stripes, rows, cell), np.uint8)
    for i in range(rows):
        for j in range(p if with_row_parity_disk else p - 1):
            d = (i + direction * j) % p
            if d != unstored:
                Q[:, stored.index(d), :] ^= D[:, i, j, :]
    return D[:, :, p - 1, :].reshape(-1).copy(), Q.reshape(-1)


@pytest.mark.parametrize("k", list(range(1, 17)))
def test_diagonal_parity_equals_definition_direct_construction(k):
    p = oracle.rdp_prime(k)
    for cell, stripes in ((1, 1), (3, 4), (16, 2)):
        S = stripes * (p - 1) * cell
        data = [inputs.uniform_bytes_np(900 + 17 * k + j, S) for j in range(k)]
        R, Q = oracle.rdp_encode(data, cell)
        wantR, wantQ = rdp_by_definition(data, cell)
        assert np.array_equal(R, wantR), (k, cell)
        assert np.array_equal(Q, wantQ), (k, cell)


def test_the_pins_tell_wrong_conventions_apart():
    """Each plausible wrong convention is still a two-erasure code, so the
    property tests cannot see it; the hand-worked stripes can: the wrong
    variants of the definition-direct construction miss the hand-worked Q."""
    d3 = [np.array([0x01, 0x02], np.uint8), np.array([0x04, 0x08], np.uint8)]
    d5 = [np.array([1 << (4 * j + i) for i in range(4)], dtype="<u2").view(np.uint8).copy() for j in range(4)]
    assert rdp_by_definition(d3, 1)[1].tolist() == [0x0B, 0x06]
    assert rdp_by_definition(d5, 2)[1].view("<u2").tolist() == [0x6A23, 0xC456, 0x89AC, 0x1248]
    for wrong in (dict(direction=-1), dict(with_row_parity_disk=False), dict(unstored=0), dict(unstored=1)):
        assert rdp_by_definition(d3, 1, **wrong)[1].tolist() != [0x0B, 0x06], wrong
        assert rdp_by_definition(d5, 2, **wrong)[1].view("<u2").tolist() != [0x6A23, 0xC456, 0x89AC, 0x1248], wrong
