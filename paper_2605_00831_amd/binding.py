"""Thin ctypes binding of the C-ABI HIP library (include/ghostserve_ec.h).

Same names as the C entry points; this layer only marshals arguments (device
pointers out of torch tensors, host pointer arrays, stream handles).  Every
step of the path runs in the library's HIP kernels.  There is no CPU
fallback: if the built library is missing, loading raises.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libghostserve_ec.so")

GS_OK, GS_EINVAL, GS_ENOMEM, GS_ETOOMANY, GS_ESINGULAR, GS_EHIP, GS_ELIMIT = 0, -1, -2, -3, -4, -5, -6
GS_STATIC_MAX_CHUNKS = 1024
GS_CAUCHY, GS_VANDERMONDE, GS_RDP, GS_POWER = 0, 1, 2, 3

EXPORTS = [
    "gs_make_code", "gs_free_code", "gs_code_params", "gs_code_matrix", "gs_decode_matrix", "gs_make_rdp_code", "gs_rdp_prime", "gs_rdp_cell_bytes", "gs_rdp_plan",
    "gs_encode", "gs_encode_paged", "gs_reconstruct", "gs_reconstruct_paged",
    "gs_pipe_create", "gs_pipe_destroy", "gs_checkpoint", "gs_restore", "gs_checkpoint_paged", "gs_restore_paged", "gs_pipe_sync",
    "gs_pipe_done_event", "gs_pipe_set_timing", "gs_pipe_chunk_times",
    "gs_step_graph_create", "gs_step_graph_launch", "gs_step_graph_destroy",
    "gs_batch_create", "gs_batch_destroy", "gs_encode_batch", "gs_reconstruct_batch", "gs_encode_batch_static",
    "gs_pool_create", "gs_pool_destroy", "gs_encode_streams", "gs_reconstruct_streams",
    "gs_recompute_units",
    "gs_strerror", "gs_last_hip_error", "gs_coef_words", "gs_set_launch_shape", "gs_set_power_horner",
    "gs_set_occupancy_cap",
    "gs_set_size_forms",
]

_vp = ctypes.c_void_p
_vpp = ctypes.POINTER(ctypes.c_void_p)
_u8p = ctypes.POINTER(ctypes.c_uint8)
_intp = ctypes.POINTER(ctypes.c_int)

class RecoveryCosts(ctypes.Structure):
    """seconds per chunk; see gs_recovery_costs in the header"""
    _fields_ = [("recompute_base_s", ctypes.c_double), ("recompute_growth_s", ctypes.c_double),
                ("gather_s", ctypes.c_double), ("h2d_s", ctypes.c_double),
                ("reconstruct_s", ctypes.c_double), ("restore_startup_s", ctypes.c_double)]


_lib = None


class GsError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = lib().gs_strerror(status).decode()
        if status == GS_EHIP:
            msg += " (hipError %d)" % lib().gs_last_hip_error()
        super().__init__("%s: %s [%d]" % (where, msg, status))


def lib():
    """Load the HIP library (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            "HIP library %s is missing: run `python -m paper_2605_00831_amd.build` "
            "(there is no CPU fallback)" % LIB_PATH)
    # torch ships its own HIP runtime; import it first so that the library
    # binds to the runtime that owns torch's device memory and streams
    import torch  # noqa: F401
    L = ctypes.CDLL(LIB_PATH)
    L.gs_make_code.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.POINTER(_vp)]
    L.gs_free_code.argtypes = [_vp]
    L.gs_free_code.restype = None
    L.gs_code_params.argtypes = [_vp, _intp, _intp]
    L.gs_code_matrix.argtypes = [_vp, _u8p]
    L.gs_decode_matrix.argtypes = [_vp, _intp, ctypes.c_int, _u8p, _intp]
    L.gs_rdp_prime.argtypes = [_vp, _intp]
    L.gs_make_rdp_code.argtypes = [ctypes.c_int, ctypes.c_size_t, ctypes.POINTER(_vp)]
    L.gs_rdp_cell_bytes.argtypes = [_vp, ctypes.POINTER(ctypes.c_size_t)]
    L.gs_rdp_plan.argtypes = [_vp, _intp, ctypes.c_int, _intp, _intp, ctypes.POINTER(ctypes.c_uint32)]
    L.gs_encode.argtypes = [_vp, _vpp, _vpp, ctypes.c_size_t, _vp]
    L.gs_encode_paged.argtypes = [_vp, _vp, ctypes.c_int, ctypes.c_size_t, ctypes.c_int64, _vp,
                                  ctypes.c_int, _vpp, _vp]
    L.gs_reconstruct.argtypes = [_vp, _vpp, _intp, ctypes.c_int, ctypes.c_size_t, _vp]
    L.gs_reconstruct_paged.argtypes = [_vp, _vp, ctypes.c_int, ctypes.c_size_t, ctypes.c_int64, _vp,
                                       ctypes.c_int, _vpp, _intp, ctypes.c_int, _vp]
    L.gs_pipe_create.argtypes = [_vp, ctypes.c_size_t, ctypes.c_int, ctypes.POINTER(_vp)]
    L.gs_pipe_destroy.argtypes = [_vp]
    L.gs_pipe_destroy.restype = None
    L.gs_checkpoint.argtypes = [_vp, _vpp, ctypes.c_size_t, _vpp, _vp]
    L.gs_restore.argtypes = [_vp, _vpp, _vpp, _intp, ctypes.c_int, ctypes.c_size_t, _vp]
    L.gs_checkpoint_paged.argtypes = [_vp, _vp, ctypes.c_int, ctypes.c_size_t, ctypes.c_int64, _vp, ctypes.c_int, _vpp, _vp]
    L.gs_restore_paged.argtypes = [_vp, _vp, ctypes.c_int, ctypes.c_size_t, ctypes.c_int64, _vp, ctypes.c_int, _vpp, _vpp,
                                   _intp, ctypes.c_int, _vp]
    L.gs_pipe_sync.argtypes = [_vp]
    L.gs_pipe_done_event.argtypes = [_vp]
    L.gs_pipe_done_event.restype = _vp
    _fp = ctypes.POINTER(ctypes.c_float)
    L.gs_pipe_set_timing.argtypes = [_vp, ctypes.c_int]
    L.gs_pipe_chunk_times.argtypes = [_vp, ctypes.c_int, _fp, _fp, _fp, _intp]
    L.gs_step_graph_create.argtypes = [_vp, _vp, ctypes.c_int, ctypes.c_size_t, ctypes.c_int64, _vp,
                                       ctypes.c_int, _vpp, _vpp, ctypes.POINTER(_vp)]
    L.gs_step_graph_launch.argtypes = [_vp, _vp]
    L.gs_step_graph_destroy.argtypes = [_vp]
    L.gs_step_graph_destroy.restype = None
    _szp = ctypes.POINTER(ctypes.c_size_t)
    L.gs_batch_create.argtypes = [_vp, ctypes.c_int, ctypes.POINTER(_vp)]
    L.gs_batch_destroy.argtypes = [_vp]
    L.gs_batch_destroy.restype = None
    L.gs_encode_batch.argtypes = [_vp, ctypes.c_int, _vpp, _vpp, _szp, _vp]
    L.gs_reconstruct_batch.argtypes = [_vp, ctypes.c_int, _vpp, _intp, ctypes.c_int, _szp, _vp]
    L.gs_encode_batch_static.argtypes = [_vp, ctypes.c_int, _vpp, _vpp, _szp, _vp]
    L.gs_pool_create.argtypes = [ctypes.c_int, ctypes.POINTER(_vp)]
    L.gs_pool_destroy.argtypes = [_vp]
    L.gs_pool_destroy.restype = None
    L.gs_encode_streams.argtypes = [_vp, _vp, ctypes.c_int, _vpp, _vpp, _szp, _vp]
    L.gs_reconstruct_streams.argtypes = [_vp, _vp, ctypes.c_int, _vpp, _intp, ctypes.c_int, _szp, _vp]
    L.gs_recompute_units.argtypes = [ctypes.c_int, ctypes.POINTER(RecoveryCosts), _intp,
                                     ctypes.POINTER(ctypes.c_double)]
    L.gs_strerror.argtypes = [ctypes.c_int]
    L.gs_strerror.restype = ctypes.c_char_p
    L.gs_last_hip_error.argtypes = []
    L.gs_coef_words.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_uint32)]
    L.gs_set_launch_shape.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int]
    L.gs_set_power_horner.argtypes = [ctypes.c_int]
    L.gs_set_occupancy_cap.argtypes = [ctypes.c_int]
    L.gs_set_size_forms.argtypes = [ctypes.c_int]
    _lib = L
    return L


def _check(status, where):
    if status != GS_OK:
        raise GsError(status, where)


def _ptr(x):
    """Device or host address of a tensor / array / int / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    if isinstance(x, np.ndarray):
        return x.ctypes.data
    raise TypeError("cannot take the address of %r" % type(x))


def _ptr_array(seq):
    return (ctypes.c_void_p * len(seq))(*[_ptr(x) for x in seq])


def _int_array(seq):
    seq = list(seq)
    return (ctypes.c_int * max(len(seq), 1))(*seq), len(seq)


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


class Code:
    """Owner of a gs_code handle."""

    def __init__(self, handle, k, m):
        self.handle, self.k, self.m = handle, k, m

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.gs_free_code(self.handle)
            self.handle = None


class Pipe:
    def __init__(self, handle, code):
        self.handle, self.code = handle, code

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.gs_pipe_destroy(self.handle)
            self.handle = None


class StepGraph:
    def __init__(self, handle, keep):
        self.handle, self._keep = handle, keep

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.gs_step_graph_destroy(self.handle)
            self.handle = None


def gs_make_code(k, m, kind=GS_CAUCHY):
    h = _vp()
    _check(lib().gs_make_code(k, m, kind, ctypes.byref(h)), "gs_make_code")
    return Code(h, k, m)


def gs_code_matrix(code):
    P = np.zeros((code.m, code.k), np.uint8)
    _check(lib().gs_code_matrix(code.handle, P.ctypes.data_as(_u8p)), "gs_code_matrix")
    return P


def gs_make_rdp_code(k, cell_bytes):
    h = _vp()
    _check(lib().gs_make_rdp_code(k, cell_bytes, ctypes.byref(h)), "gs_make_rdp_code")
    return Code(h, k, 2)


def gs_rdp_cell_bytes(code):
    c = ctypes.c_size_t()
    _check(lib().gs_rdp_cell_bytes(code.handle, ctypes.byref(c)), "gs_rdp_cell_bytes")
    return c.value


def gs_rdp_prime(code):
    p = ctypes.c_int()
    _check(lib().gs_rdp_prime(code.handle, ctypes.byref(p)), "gs_rdp_prime")
    return p.value


def gs_rdp_plan(code, missing=()):
    """(shards read, syndrome masks [len(missing) or 2][p-1]) of the encode plan
    (nothing missing = both parity shards are produced) or of a rebuild plan"""
    er, n = _int_array(missing)
    read = (ctypes.c_int * 18)()
    nr = ctypes.c_int()
    mask = (ctypes.c_uint32 * 32)()
    _check(lib().gs_rdp_plan(code.handle, er, n, read, ctypes.byref(nr), mask), "gs_rdp_plan")
    rows = gs_rdp_prime(code) - 1
    n_out = n if n else 2
    return list(read[: nr.value]), np.array(list(mask[: n_out * rows]), dtype=np.uint32).reshape(n_out, rows)


def gs_decode_matrix(code, erased):
    er, n = _int_array(erased)
    R = np.zeros((n, code.k), np.uint8)
    surv = (ctypes.c_int * code.k)()
    _check(lib().gs_decode_matrix(code.handle, er, n, R.ctypes.data_as(_u8p), surv), "gs_decode_matrix")
    return R, list(surv)


def gs_encode(code, data, parity, shard_bytes, stream=None):
    if len(data) != code.k or len(parity) != code.m:
        raise ValueError("need k data and m parity pointers")
    _check(lib().gs_encode(code.handle, _ptr_array(data), _ptr_array(parity), shard_bytes,
                           _stream(stream)), "gs_encode")


def gs_encode_paged(code, plane_base, n_planes, page_bytes, pages_per_plane, table, pages_per_shard,
                    parity, stream=None):
    if len(parity) != code.m:
        raise ValueError("need m parity pointers")
    _check(lib().gs_encode_paged(code.handle, _ptr(plane_base), n_planes, page_bytes, pages_per_plane,
                                 _ptr(table), pages_per_shard, _ptr_array(parity), _stream(stream)),
           "gs_encode_paged")


def gs_reconstruct_paged(code, plane_base, n_planes, page_bytes, pages_per_plane, table, pages_per_shard,
                         parity, erased, stream=None):
    if len(parity) != code.m:
        raise ValueError("need m parity pointers")
    er, n = _int_array(erased)
    _check(lib().gs_reconstruct_paged(code.handle, _ptr(plane_base), n_planes, page_bytes, pages_per_plane,
                                      _ptr(table), pages_per_shard, _ptr_array(parity), er, n, _stream(stream)),
           "gs_reconstruct_paged")


def gs_reconstruct(code, shards, erased, shard_bytes, stream=None):
    if len(shards) != code.k + code.m:
        raise ValueError("need k+m shard pointers")
    er, n = _int_array(erased)
    _check(lib().gs_reconstruct(code.handle, _ptr_array(shards), er, n, shard_bytes, _stream(stream)),
           "gs_reconstruct")


def gs_pipe_create(code, chunk_bytes, depth=2):
    h = _vp()
    _check(lib().gs_pipe_create(code.handle, chunk_bytes, depth, ctypes.byref(h)), "gs_pipe_create")
    return Pipe(h, code)


def gs_checkpoint(pipe, data, shard_bytes, host_parity, stream=None):
    if len(data) != pipe.code.k or len(host_parity) != pipe.code.m:
        raise ValueError("need k data and m host parity pointers")
    _check(lib().gs_checkpoint(pipe.handle, _ptr_array(data), shard_bytes, _ptr_array(host_parity),
                               _stream(stream)), "gs_checkpoint")


def gs_restore(pipe, shards, host_parity, erased, shard_bytes, stream=None):
    if len(shards) != pipe.code.k + pipe.code.m or len(host_parity) != pipe.code.m:
        raise ValueError("need k+m shard pointers and m host parity pointers")
    er, n = _int_array(erased)
    _check(lib().gs_restore(pipe.handle, _ptr_array(shards), _ptr_array(host_parity), er, n, shard_bytes,
                            _stream(stream)), "gs_restore")


def gs_checkpoint_paged(pipe, plane_base, n_planes, page_bytes, pages_per_plane, table, pages_per_shard,
                        host_parity, stream=None):
    if len(host_parity) != pipe.code.m:
        raise ValueError("need m host parity pointers")
    _check(lib().gs_checkpoint_paged(pipe.handle, _ptr(plane_base), n_planes, page_bytes, pages_per_plane, _ptr(table),
                                     pages_per_shard, _ptr_array(host_parity), _stream(stream)), "gs_checkpoint_paged")


def gs_restore_paged(pipe, plane_base, n_planes, page_bytes, pages_per_plane, table, pages_per_shard,
                     host_parity, erased, parity_out=None, stream=None):
    if len(host_parity) != pipe.code.m or (parity_out is not None and len(parity_out) != pipe.code.m):
        raise ValueError("need m host parity pointers (and m device parity pointers, if any)")
    er, n = _int_array(erased)
    po = _ptr_array(parity_out) if parity_out is not None else None
    _check(lib().gs_restore_paged(pipe.handle, _ptr(plane_base), n_planes, page_bytes, pages_per_plane, _ptr(table),
                                  pages_per_shard, _ptr_array(host_parity), po, er, n, _stream(stream)), "gs_restore_paged")


def gs_pipe_sync(pipe):
    _check(lib().gs_pipe_sync(pipe.handle), "gs_pipe_sync")


def gs_pipe_done_event(pipe):
    return lib().gs_pipe_done_event(pipe.handle)


def gs_pipe_set_timing(pipe, enable=True):
    _check(lib().gs_pipe_set_timing(pipe.handle, 1 if enable else 0), "gs_pipe_set_timing")


def gs_pipe_chunk_times(pipe, max_chunks=4096):
    """[(kernel_begin_ms, kernel_end_ms, copy_end_ms)] per chunk of the last timed call"""
    a = (ctypes.c_float * max_chunks)()
    b = (ctypes.c_float * max_chunks)()
    c = (ctypes.c_float * max_chunks)()
    n = ctypes.c_int()
    _check(lib().gs_pipe_chunk_times(pipe.handle, max_chunks, a, b, c, ctypes.byref(n)), "gs_pipe_chunk_times")
    return [(a[i], b[i], c[i]) for i in range(min(n.value, max_chunks))]


def gs_pipe_destroy(pipe):
    if pipe.handle:
        lib().gs_pipe_destroy(pipe.handle)
        pipe.handle = None


def gs_step_graph_create(code, plane_base, n_planes, page_bytes, pages_per_plane, table, pages_per_shard,
                         parity, host_parity=None):
    h = _vp()
    hp = _ptr_array(host_parity) if host_parity is not None else None
    _check(lib().gs_step_graph_create(code.handle, _ptr(plane_base), n_planes, page_bytes, pages_per_plane,
                                      _ptr(table), pages_per_shard, _ptr_array(parity), hp,
                                      ctypes.byref(h)), "gs_step_graph_create")
    return StepGraph(h, (code, plane_base, table, parity, host_parity))


def gs_step_graph_launch(graph, stream=None):
    _check(lib().gs_step_graph_launch(graph.handle, _stream(stream)), "gs_step_graph_launch")


def gs_step_graph_destroy(graph):
    if graph.handle:
        lib().gs_step_graph_destroy(graph.handle)
        graph.handle = None


class Batch:
    def __init__(self, handle, code):
        self.handle, self.code = handle, code

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.gs_batch_destroy(self.handle)
            self.handle = None


class Pool:
    def __init__(self, handle):
        self.handle = handle

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.gs_pool_destroy(self.handle)
            self.handle = None


def _flat_ptrs(chunks, width):
    """list (per chunk) of lists of `width` pointers -> one flat pointer array.
    A C-contiguous numpy array of addresses, shape (n_chunks, width), 64-bit integers, is passed
    as it is: an engine that keeps its addresses in such an array pays no per-pointer work."""
    if isinstance(chunks, np.ndarray):
        if chunks.dtype not in (np.uint64, np.int64) or chunks.ndim != 2 or chunks.shape[1] != width \
                or not chunks.flags["C_CONTIGUOUS"]:
            raise ValueError("an address array must be C-contiguous 64-bit integers of shape (n_chunks, %d)" % width)
        return chunks.ctypes.data_as(ctypes.POINTER(ctypes.c_void_p))
    flat = []
    for c in chunks:
        if len(c) != width:
            raise ValueError("every chunk needs %d pointers" % width)
        flat.extend(c)
    return _ptr_array(flat)


def _size_array(sizes):
    if isinstance(sizes, np.ndarray) and sizes.dtype == np.uint64 and sizes.ndim == 1 and sizes.flags["C_CONTIGUOUS"] \
            and ctypes.sizeof(ctypes.c_size_t) == 8:
        return sizes.ctypes.data_as(ctypes.POINTER(ctypes.c_size_t))
    sizes = list(sizes)
    return (ctypes.c_size_t * max(len(sizes), 1))(*sizes)


def gs_batch_create(code, max_chunks):
    h = _vp()
    _check(lib().gs_batch_create(code.handle, max_chunks, ctypes.byref(h)), "gs_batch_create")
    return Batch(h, code)


def gs_batch_destroy(batch):
    if batch.handle:
        lib().gs_batch_destroy(batch.handle)
        batch.handle = None


def gs_encode_batch(batch, data, parity, shard_bytes, stream=None):
    """data / parity: per chunk, a list of k resp. m tensors or addresses."""
    n = len(data)
    _check(lib().gs_encode_batch(batch.handle, n, _flat_ptrs(data, batch.code.k), _flat_ptrs(parity, batch.code.m),
                                 _size_array(shard_bytes), _stream(stream)), "gs_encode_batch")


def gs_encode_batch_static(code, data, parity, shard_bytes, stream=None):
    """gs_encode_batch without a gs_batch object and without any allocation (at most GS_STATIC_MAX_CHUNKS chunks)."""
    n = len(data)
    _check(lib().gs_encode_batch_static(code.handle, n, _flat_ptrs(data, code.k), _flat_ptrs(parity, code.m),
                                        _size_array(shard_bytes), _stream(stream)), "gs_encode_batch_static")


def gs_reconstruct_batch(batch, shards, erased, shard_bytes, stream=None):
    n = len(shards)
    er, ne = _int_array(erased)
    _check(lib().gs_reconstruct_batch(batch.handle, n, _flat_ptrs(shards, batch.code.k + batch.code.m), er, ne,
                                      _size_array(shard_bytes), _stream(stream)), "gs_reconstruct_batch")


def gs_pool_create(n_streams):
    h = _vp()
    _check(lib().gs_pool_create(n_streams, ctypes.byref(h)), "gs_pool_create")
    return Pool(h)


def gs_pool_destroy(pool):
    if pool.handle:
        lib().gs_pool_destroy(pool.handle)
        pool.handle = None


def gs_encode_streams(code, pool, data, parity, shard_bytes, stream=None):
    n = len(data)
    _check(lib().gs_encode_streams(code.handle, pool.handle, n, _flat_ptrs(data, code.k), _flat_ptrs(parity, code.m),
                                   _size_array(shard_bytes), _stream(stream)), "gs_encode_streams")


def gs_reconstruct_streams(code, pool, shards, erased, shard_bytes, stream=None):
    n = len(shards)
    er, ne = _int_array(erased)
    _check(lib().gs_reconstruct_streams(code.handle, pool.handle, n, _flat_ptrs(shards, code.k + code.m), er, ne,
                                        _size_array(shard_bytes), _stream(stream)), "gs_reconstruct_streams")


def gs_recompute_units(n_chunks, recompute_base_s, recompute_growth_s, gather_s, h2d_s, reconstruct_s,
                       restore_startup_s=0.0):
    """(r, makespan_s): chunks to recompute, and the modelled recovery time"""
    costs = RecoveryCosts(recompute_base_s, recompute_growth_s, gather_s, h2d_s, reconstruct_s, restore_startup_s)
    r = ctypes.c_int()
    t = ctypes.c_double()
    _check(lib().gs_recompute_units(n_chunks, ctypes.byref(costs), ctypes.byref(r), ctypes.byref(t)),
           "gs_recompute_units")
    return r.value, t.value


def gs_coef_words(c):
    w = (ctypes.c_uint32 * 5)()
    _check(lib().gs_coef_words(c, w), "gs_coef_words")
    return list(w)


def gs_set_power_horner(enable=True):
    _check(lib().gs_set_power_horner(1 if enable else 0), "gs_set_power_horner")


def gs_set_occupancy_cap(enable=True):
    _check(lib().gs_set_occupancy_cap(1 if enable else 0), "gs_set_occupancy_cap")


def gs_set_size_forms(mode=1):
    _check(lib().gs_set_size_forms(int(mode)), "gs_set_size_forms")


def gs_set_launch_shape(unroll=0, tiles_per_wg=0, nontemporal=-1, interleave_shift=-1):
    _check(lib().gs_set_launch_shape(unroll, tiles_per_wg, nontemporal, interleave_shift),
           "gs_set_launch_shape")
