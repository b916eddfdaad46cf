"""Independent GF(2^8) helpers for pinning the oracle.

Nothing here calls the oracle or the HIP library.  Multiplication is the
schoolbook carry-less product of two degree-<8 polynomials over GF(2),
followed by long division by x^8+x^4+x^3+x^2+1 -- no log/exp tables, so a
mistake in the oracle's table construction cannot hide here.
"""
import numpy as np

POLY = 0x11D


def clmul_reduce(a, b):
    """a*b in GF(2)[x] mod POLY, plain integers."""
    prod = 0
    for bit in range(8):
        if (b >> bit) & 1:
            prod ^= a << bit
    for deg in range(14, 7, -1):
        if (prod >> deg) & 1:
            prod ^= POLY << (deg - 8)
    return prod


def full_table():
    """256x256 product table built with vectorised shift-and-reduce (xtime)."""
    a = np.arange(256, dtype=np.uint16).reshape(256, 1).repeat(256, 1)
    b = np.arange(256, dtype=np.uint16).reshape(1, 256).repeat(256, 0)
    acc = np.zeros((256, 256), np.uint16)
    cur = a.copy()
    for bit in range(8):
        acc ^= np.where((b >> bit) & 1, cur, 0).astype(np.uint16)
        cur = cur << 1
        cur = np.where(cur & 0x100, cur ^ POLY, cur).astype(np.uint16)
    return acc.astype(np.uint8)


_T = None


def T():
    global _T
    if _T is None:
        _T = full_table()
    return _T


def inv_by_search(a):
    row = T()[a]
    hits = np.nonzero(row == 1)[0]
    assert len(hits) == 1
    return int(hits[0])


def mat_rank(A):
    """Rank over the field by row reduction (python ints, table lookups)."""
    t = T()
    A = [list(map(int, r)) for r in A]
    rows, cols = len(A), len(A[0])
    rank = 0
    for c in range(cols):
        piv = None
        for r in range(rank, rows):
            if A[r][c]:
                piv = r
                break
        if piv is None:
            continue
        A[rank], A[piv] = A[piv], A[rank]
        iv = inv_by_search(A[rank][c])
        A[rank] = [int(t[iv, x]) for x in A[rank]]
        for r in range(rows):
            if r != rank and A[r][c]:
                f = A[r][c]
                A[r] = [x ^ int(t[f, y]) for x, y in zip(A[r], A[rank])]
        rank += 1
        if rank == rows:
            break
    return rank


def matmul(A, B):
    t = T()
    A = np.asarray(A, np.uint8)
    B = np.asarray(B, np.uint8)
    out = np.zeros((A.shape[0], B.shape[1]), np.uint8)
    for i in range(A.shape[0]):
        for j in range(B.shape[1]):
            out[i, j] = np.bitwise_xor.reduce(t[A[i, :], B[:, j]]) if A.shape[1] else 0
    return out


def cauchy_normalised(k, m):
    """Closed form: 1/(x_i+y_j) with x_i=k+i, y_j=j, columns scaled so row 0
    is all ones, rows scaled so column 0 is all ones."""
    t = T()

    def div(a, b):
        return int(t[a, inv_by_search(b)])

    P = np.zeros((m, k), np.uint8)
    for i in range(m):
        for j in range(k):
            xi, x0, yj, y0 = k + i, k, j, 0
            num = int(t[x0 ^ yj, xi ^ y0])
            den = int(t[xi ^ yj, x0 ^ y0])
            P[i, j] = div(num, den)
    return P


def encode_np(P, data):
    """Vectorised encode with the independent table: list of k arrays -> m arrays."""
    t = T()
    P = np.asarray(P, np.uint8)
    out = []
    for i in range(P.shape[0]):
        acc = np.zeros_like(data[0])
        for j in range(P.shape[1]):
            acc ^= t[P[i, j]][data[j]]
        out.append(acc)
    return out
