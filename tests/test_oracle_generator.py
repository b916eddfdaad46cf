"""Pins for the oracle's generator matrix and matrix inverse.

The paper (Section 2, Section 4.1) fixes only the properties: N data shards,
K parity shards, any K losses are recoverable (MDS), XOR is the one-parity
code.  The oracle builds P by the Vandermonde + Gauss-Jordan route; these
tests check it against the Cauchy closed form written with an independent
multiply, and check the MDS property exhaustively on small codes.
"""
import itertools

import numpy as np
import pytest

import oracle
from tests import _gfref


@pytest.mark.parametrize("k,m", [(1, 1), (2, 1), (4, 1), (4, 2), (8, 2), (8, 3), (3, 2), (5, 3),
                                 (10, 4), (16, 4), (20, 6), (7, 5), (250, 6), (128, 128), (1, 255)])
def test_vandermonde_route_equals_cauchy_closed_form(k, m):
    assert np.array_equal(oracle.generator(k, m), _gfref.cauchy_normalised(k, m))


def test_first_row_and_first_column_are_ones():
    for k in range(1, 13):
        for m in range(1, 7):
            P = oracle.generator(k, m)
            assert (P[0] == 1).all() and (P[:, 0] == 1).all()


def test_bad_parameters_rejected():
    for k, m in [(0, 1), (1, 0), (-1, 2), (200, 57), (256, 1)]:
        with pytest.raises(ValueError):
            oracle.generator(k, m)
    oracle.generator(255, 1)
    oracle.generator(200, 56)


def test_known_matrices():
    # computed once with two independent multipliers (see tests/_gfref.py for one)
    want = {
        (4, 2): ["01010101", "01d95cac"],
        (8, 2): ["0101010101010101", "0137274954b5e1d9"],
        (8, 3): ["0101010101010101", "0137274954b5e1d9", "0127d9a15c3cac5a"],
        (3, 2): ["010101", "01c453"],
        (5, 3): ["0101010101", "019c7ba6f4", "0197d47bc5"],
    }
    for (k, m), rows in want.items():
        P = oracle.generator(k, m)
        assert [bytes(r).hex() for r in P] == rows
        assert np.array_equal(_gfref.cauchy_normalised(k, m), P)


def test_every_k_row_submatrix_of_G_is_invertible_exhaustive():
    """MDS: any k of the k+m shards determine the data (Section 4.1: up to K
    simultaneous failures).  Exhaustive for every code with k+m <= 10, checked
    with the independent rank routine, not with the oracle's inverse."""
    for n in range(2, 11):
        for m in range(1, n):
            k = n - m
            P = oracle.generator(k, m)
            G = np.vstack([np.eye(k, dtype=np.uint8), P])
            for rows in itertools.combinations(range(n), k):
                assert _gfref.mat_rank(G[list(rows)]) == k, (k, m, rows)


def test_config5_code_all_165_erasure_triples_leave_full_rank():
    P = oracle.generator(8, 3)
    G = np.vstack([np.eye(8, dtype=np.uint8), P])
    for lost in itertools.combinations(range(11), 3):
        rows = [r for r in range(11) if r not in lost]
        assert _gfref.mat_rank(G[rows]) == 8


def test_inverse_times_matrix_is_identity():
    rng = np.random.default_rng(7)
    done = 0
    while done < 40:
        n = int(rng.integers(1, 12))
        A = rng.integers(0, 256, size=(n, n), dtype=np.uint8)
        if _gfref.mat_rank(A) < n:
            with pytest.raises(ArithmeticError):
                oracle.invert(A)
            continue
        Ai = oracle.invert(A)
        assert np.array_equal(_gfref.matmul(A, Ai), np.eye(n, dtype=np.uint8))
        assert np.array_equal(_gfref.matmul(Ai, A), np.eye(n, dtype=np.uint8))
        done += 1
    with pytest.raises(ArithmeticError):
        oracle.invert(np.array([[1, 2], [1, 2]], np.uint8))
    # needs a row swap: zero pivot in the corner
    A = np.array([[0, 1], [1, 0]], np.uint8)
    assert np.array_equal(oracle.invert(A), A)


def test_known_inverse_rows():
    # k=4, m=2, shards 1 and 3 lost: survivors are rows {0, 2, 4, 5} of G
    P = oracle.generator(4, 2)
    G = np.vstack([np.eye(4, dtype=np.uint8), P])
    A = G[[0, 2, 4, 5]]
    Ai = oracle.invert(A)
    assert [bytes(r).hex() for r in Ai] == ["01000000", "f5690efb", "00010000", "f4680ffb"]
    assert np.array_equal(_gfref.matmul(A, Ai), np.eye(4, dtype=np.uint8))
