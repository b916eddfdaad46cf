"""Pins for the oracle's field arithmetic (Section 2: Reed-Solomon works "over
Galois fields"; the field itself -- 0x11D, generator 2 -- is this build's reading).

Expected values come from the field axioms, from an independently written
carry-less multiply (tests/_gfref.py) and from constants fixed by the
polynomial; none comes from the oracle itself.
"""
import hashlib

import numpy as np

import oracle
from tests import _gfref


def test_product_table_matches_independent_multiply_on_all_pairs():
    assert np.array_equal(oracle.mul_table(), _gfref.T())


def test_scalar_multiply_matches_polynomial_long_division():
    rng = np.random.default_rng(1)
    for a, b in rng.integers(0, 256, size=(2000, 2)):
        assert oracle.gf_mul(int(a), int(b)) == _gfref.clmul_reduce(int(a), int(b))
    for a in range(256):
        assert oracle.gf_mul(a, 0) == 0 and oracle.gf_mul(0, a) == 0
        assert oracle.gf_mul(a, 1) == a and oracle.gf_mul(1, a) == a


def test_field_axioms_brute_force():
    t = oracle.mul_table()
    idx = np.arange(256)
    # commutative
    assert np.array_equal(t, t.T)
    # identity and zero
    assert np.array_equal(t[1], idx) and not t[0].any()
    # associative over all 2^24 triples: (a*b)*c == a*(b*c)
    ab = t  # [a,b]
    left = t[ab[:, :, None], idx[None, None, :]]
    right = t[idx[:, None, None], t[None, :, :]]
    assert np.array_equal(left, right)
    # distributive over XOR for all triples: a*(b^c) == a*b ^ a*c
    bc = idx[:, None] ^ idx[None, :]
    lhs = t[idx[:, None, None], bc[None, :, :]]
    rhs = t[:, :, None] ^ t[:, None, :]
    assert np.array_equal(lhs, rhs)
    # no zero divisors; every non-zero row is a permutation of 0..255
    for a in range(1, 256):
        assert sorted(t[a]) == list(range(256))


def test_inverse_and_order():
    t = oracle.mul_table()
    for a in range(1, 256):
        ia = oracle.gf_inv(a)
        assert t[a, ia] == 1
        assert ia == _gfref.inv_by_search(a)
        # a^255 == 1
        p = 1
        for _ in range(255):
            p = int(t[p, a])
        assert p == 1
    # 2 is primitive: its powers visit every non-zero element
    seen, p = set(), 1
    for _ in range(255):
        seen.add(p)
        p = int(t[p, 2])
    assert len(seen) == 255 and p == 1


def test_constants_fixed_by_the_polynomial():
    e, lg = oracle.tables()
    # 2^8 = x^8 = x^4+x^3+x^2+1 = 0x1D under 0x11D, then keep doubling
    assert list(e[:17]) == [0x01, 0x02, 0x04, 0x08, 0x10, 0x20, 0x40, 0x80, 0x1D,
                            0x3A, 0x74, 0xE8, 0xCD, 0x87, 0x13, 0x26, 0x4C]
    for i in range(255):
        assert lg[e[i]] == i
    assert oracle.gf_inv(2) == 0x8E and oracle.gf_inv(3) == 0xF4
    assert lg[3] == 25 and lg[0xFF] == 175
    assert oracle.gf_mul(0x53, 0xCA) == 0x8F
    assert oracle.gf_mul(0xFF, 0xFF) == 0xE2
    # each of these is also what the independent multiply says
    assert _gfref.clmul_reduce(0x53, 0xCA) == 0x8F
    assert _gfref.clmul_reduce(0xFF, 0xFF) == 0xE2
    assert _gfref.clmul_reduce(2, 0x8E) == 1 and _gfref.clmul_reduce(3, 0xF4) == 1


def test_table_digests():
    # digests of the independent table; the oracle must reproduce both
    ind = _gfref.T()
    assert hashlib.sha256(oracle.mul_table().tobytes()).hexdigest() == \
        hashlib.sha256(ind.tobytes()).hexdigest() == \
        "003d1a609783d2740b9b3f00b0cd9e43e42c4f3eedc5ff54ec1709996d52e1e0"
    pw, p = [], 1
    for _ in range(255):
        pw.append(p)
        p = _gfref.clmul_reduce(p, 2)
    e, _ = oracle.tables()
    assert bytes(pw) == e.tobytes()
    assert hashlib.sha256(bytes(pw)).hexdigest() == \
        "bdc336e3f040e4deac02d4ee345234a3aeecd636b8c944c229dd29b0a1852987"
