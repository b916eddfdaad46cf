"""ctypes front end of the plain CPU oracle (oracle/gs_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The HIP library and its Python binding never
import this package, and this package never imports them.

All functions take and return numpy uint8 arrays; nothing here does field
arithmetic in Python -- every result comes from the C file.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gs_oracle.c")
_SRC_RDP = os.path.join(_HERE, "gs_rdp_oracle.c")
_LIB = os.path.join(_HERE, "libgs_oracle.so")

_u8p = ctypes.POINTER(ctypes.c_uint8)
_u8pp = ctypes.POINTER(_u8p)
_i32p = ctypes.POINTER(ctypes.c_int32)
_intp = ctypes.POINTER(ctypes.c_int)


def build(force=False):
    """Compile the oracle with gcc -O2 (no SIMD flags) if missing or stale."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < max(os.path.getmtime(_SRC),
                                                                       os.path.getmtime(_SRC_RDP))
    if force or stale:
        tmp = _LIB + ".%d.tmp" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", tmp, _SRC, _SRC_RDP, "-lpthread"])
        os.replace(tmp, _LIB)
    return _LIB


class _Costs(ctypes.Structure):
    _fields_ = [(n, ctypes.c_double) for n in ("base", "growth", "gather", "h2d", "reconstruct", "startup")]


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        L.gso_mul.restype = ctypes.c_uint8
        L.gso_mul.argtypes = [ctypes.c_uint8, ctypes.c_uint8]
        L.gso_inv.restype = ctypes.c_uint8
        L.gso_inv.argtypes = [ctypes.c_uint8]
        L.gso_tables.argtypes = [_u8p, _u8p]
        L.gso_mul_table.argtypes = [_u8p]
        L.gso_invert.argtypes = [ctypes.c_int, _u8p, _u8p]
        L.gso_generator.argtypes = [ctypes.c_int, ctypes.c_int, _u8p]
        L.gso_encode.argtypes = [ctypes.c_int, ctypes.c_int, _u8p, _u8pp, _u8pp, ctypes.c_size_t]
        L.gso_encode.restype = None
        L.gso_encode_mt.argtypes = [ctypes.c_int, ctypes.c_int, _u8p, _u8pp, _u8pp,
                                    ctypes.c_size_t, ctypes.c_int]
        L.gso_encode_paged.argtypes = [ctypes.c_int, ctypes.c_int, _u8p, _u8pp, ctypes.c_int,
                                       ctypes.c_size_t, _i32p, ctypes.c_int, _u8pp]
        L.gso_encode_paged.restype = None
        L.gso_decode_matrix.argtypes = [ctypes.c_int, ctypes.c_int, _u8p, _intp, ctypes.c_int,
                                        _u8p, _intp]
        L.gso_reconstruct.argtypes = [ctypes.c_int, ctypes.c_int, _u8p, _u8pp, _intp,
                                      ctypes.c_int, ctypes.c_size_t]
        L.gso_recompute_units.argtypes = [ctypes.c_int, ctypes.POINTER(_Costs), ctypes.POINTER(ctypes.c_double)]
        L.gso_power_generator.argtypes = [ctypes.c_int, ctypes.c_int, _u8p]
        L.gso_rdp_prime.argtypes = [ctypes.c_int]
        L.gso_rdp_encode.argtypes = [ctypes.c_int, _u8pp, ctypes.c_size_t, ctypes.c_size_t]
        L.gso_rdp_reconstruct.argtypes = [ctypes.c_int, _u8pp, _intp, ctypes.c_int, ctypes.c_size_t,
                                          ctypes.c_size_t]
        L.gso_init()
        _lib = L
    return _lib


def _p(a):
    return a.ctypes.data_as(_u8p)


def _ptr_array(arrs):
    return (_u8p * len(arrs))(*[_p(a) for a in arrs])


def _check_u8(a, name):
    if not (isinstance(a, np.ndarray) and a.dtype == np.uint8 and a.flags["C_CONTIGUOUS"]):
        raise TypeError("%s must be a C-contiguous numpy uint8 array" % name)


def gf_mul(a, b):
    return int(lib().gso_mul(a, b))


def gf_inv(a):
    return int(lib().gso_inv(a))


def tables():
    """(exp[0..254], log[0..255]) of the field."""
    e = np.zeros(255, np.uint8)
    lg = np.zeros(256, np.uint8)
    lib().gso_tables(_p(e), _p(lg))
    return e, lg


def mul_table():
    t = np.zeros((256, 256), np.uint8)
    lib().gso_mul_table(_p(t))
    return t


def invert(A):
    A = np.ascontiguousarray(A, np.uint8)
    n = A.shape[0]
    assert A.shape == (n, n)
    out = np.zeros((n, n), np.uint8)
    rc = lib().gso_invert(n, _p(A), _p(out))
    if rc:
        raise ArithmeticError("singular matrix")
    return out


def generator(k, m):
    """Canonical parity block P (m x k) of the systematic code [I; P]."""
    P = np.zeros((m, k), np.uint8)
    rc = lib().gso_generator(k, m, _p(P))
    if rc:
        raise ValueError("bad code parameters k=%d m=%d" % (k, m))
    return P


def power_generator(k, m):
    """Parity block of the power code, P[i][j] = 2^(i*j), m <= 3."""
    P = np.zeros((m, k), np.uint8)
    if lib().gso_power_generator(k, m, _p(P)):
        raise ValueError("bad power-code parameters k=%d m=%d" % (k, m))
    return P


def encode(P, data, nthreads=1):
    """data: list of k equal-length uint8 arrays -> list of m parity arrays."""
    P = np.ascontiguousarray(P, np.uint8)
    m, k = P.shape
    assert len(data) == k
    S = data[0].size
    for d in data:
        _check_u8(d, "data shard")
        assert d.size == S
    parity = [np.zeros(S, np.uint8) for _ in range(m)]
    if nthreads <= 1:
        lib().gso_encode(k, m, _p(P), _ptr_array(data), _ptr_array(parity), S)
    else:
        lib().gso_encode_mt(k, m, _p(P), _ptr_array(data), _ptr_array(parity), S, nthreads)
    return parity


def encode_paged(P, planes, page_bytes, table):
    """planes: list of uint8 arrays (one per pool plane); table: int32 [k][pages_per_shard]."""
    P = np.ascontiguousarray(P, np.uint8)
    m, k = P.shape
    table = np.ascontiguousarray(table, np.int32)
    assert table.ndim == 2 and table.shape[0] == k
    pps = table.shape[1]
    for pl in planes:
        _check_u8(pl, "plane")
        if pps:
            assert (int(table.max()) + 1) * page_bytes <= pl.size and int(table.min()) >= 0
    out_bytes = len(planes) * pps * page_bytes
    parity = [np.zeros(out_bytes, np.uint8) for _ in range(m)]
    lib().gso_encode_paged(k, m, _p(P), _ptr_array(planes), len(planes), page_bytes,
                           table.ctypes.data_as(_i32p), pps, _ptr_array(parity))
    return parity


def decode_matrix(P, erased):
    """(R, survivors): R is len(erased) x k, survivors the k lowest surviving shard ids."""
    P = np.ascontiguousarray(P, np.uint8)
    m, k = P.shape
    e = len(erased)
    er = (ctypes.c_int * max(e, 1))(*erased)
    R = np.zeros((e, k), np.uint8)
    surv = (ctypes.c_int * k)()
    rc = lib().gso_decode_matrix(k, m, _p(P), er, e, _p(R), surv)
    if rc == -3:
        raise OverflowError("more erasures than parity shards")
    if rc == -4:
        raise ArithmeticError("singular survivor matrix")
    if rc:
        raise ValueError("bad erasure list")
    return R, list(surv)


def reconstruct(P, shards, erased):
    """shards: list of k+m equal-length uint8 arrays; those named in `erased`
    are overwritten in place with the rebuilt bytes."""
    P = np.ascontiguousarray(P, np.uint8)
    m, k = P.shape
    assert len(shards) == k + m
    S = shards[0].size
    for s in shards:
        _check_u8(s, "shard")
        assert s.size == S
    e = len(erased)
    er = (ctypes.c_int * max(e, 1))(*erased)
    rc = lib().gso_reconstruct(k, m, _p(P), _ptr_array(shards), er, e, S)
    if rc == -3:
        raise OverflowError("more erasures than parity shards")
    if rc == -4:
        raise ArithmeticError("singular survivor matrix")
    if rc:
        raise ValueError("bad erasure list")
    return shards


def recompute_units(n_chunks, base, growth, gather, h2d, reconstruct, startup=0.0):
    """(r, makespan): brute force over every r in [0, n]."""
    c = _Costs(base, growth, gather, h2d, reconstruct, startup)
    t = ctypes.c_double()
    r = lib().gso_recompute_units(n_chunks, ctypes.byref(c), ctypes.byref(t))
    return r, t.value


def rdp_prime(k):
    return lib().gso_rdp_prime(k)


def rdp_encode(data, cell_bytes=None):
    """data: list of k equal-length uint8 arrays holding whole stripes of p-1
    cells of cell_bytes (default: one stripe, cell = length / (p-1))
    -> [row parity, diagonal parity]."""
    k, S = len(data), data[0].size
    if cell_bytes is None:
        cell_bytes = S // (rdp_prime(k) - 1)
        if cell_bytes * (rdp_prime(k) - 1) != S:
            raise ValueError("bad RDP geometry: k=%d S=%d" % (k, S))
    for d in data:
        _check_u8(d, "data shard")
        assert d.size == S
    par = [np.zeros(S, np.uint8), np.zeros(S, np.uint8)]
    if cell_bytes < 1 or lib().gso_rdp_encode(k, _ptr_array(list(data) + par), S, cell_bytes):
        raise ValueError("bad RDP geometry: k=%d S=%d" % (k, S))
    return par


def rdp_reconstruct(shards, erased, cell_bytes=None):
    """shards: k data + row parity + diagonal parity; erased ones are rebuilt in place."""
    k, S = len(shards) - 2, shards[0].size
    if cell_bytes is None:
        cell_bytes = max(1, S // (rdp_prime(k) - 1))
    for s in shards:
        _check_u8(s, "shard")
        assert s.size == S
    e = len(erased)
    er = (ctypes.c_int * max(e, 1))(*erased)
    rc = lib().gso_rdp_reconstruct(k, _ptr_array(shards), er, e, S, cell_bytes)
    if rc == -3:
        raise OverflowError("RDP tolerates two erasures")
    if rc:
        raise ValueError("bad RDP arguments")
    return shards
