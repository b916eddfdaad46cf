"""CPU-only checks of the HIP library's host side: it loads, exports what the
header declares, builds the same generator and rebuild matrices as the oracle
(two independent implementations: closed-form Cauchy + shift-and-reduce
multiply in the library, Vandermonde + elimination + log/exp in the oracle),
builds correct lookup words, and rejects bad arguments.  No kernel is
launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from paper_2605_00831_amd import binding as gs
from paper_2605_00831_amd import inputs
from tests import _gfref

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    with open(os.path.join(ROOT, "include", "ghostserve_ec.h")) as f:
        text = f.read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(gs_[a-z_0-9]+)\s*\(", text))
    assert declared == set(gs.EXPORTS)
    L = gs.lib()
    for name in declared:
        assert hasattr(L, name), name


@pytest.mark.parametrize("k,m", [(1, 1), (4, 1), (4, 2), (8, 2), (8, 3), (5, 3), (16, 4), (20, 6),
                                 (17, 5), (250, 6), (1, 255), (128, 128)])
def test_generator_matches_oracle_for_both_kinds(k, m):
    want = oracle.generator(k, m)
    for kind in (gs.GS_CAUCHY, gs.GS_VANDERMONDE):
        code = gs.gs_make_code(k, m, kind)
        assert np.array_equal(gs.gs_code_matrix(code), want)


def test_make_code_rejects_bad_parameters():
    for k, m, kind in [(0, 1, 0), (1, 0, 0), (-3, 2, 0), (200, 57, 0), (4, 2, 4), (4, 2, -1)]:
        with pytest.raises(gs.GsError) as e:
            gs.gs_make_code(k, m, kind)
        assert e.value.status == gs.GS_EINVAL
    gs.gs_make_code(200, 56)


@pytest.mark.parametrize("k,m", [(4, 2), (8, 3), (5, 3), (2, 4), (3, 1)])
def test_decode_matrix_matches_oracle_for_every_pattern(k, m):
    code = gs.gs_make_code(k, m)
    P = oracle.generator(k, m)
    for pat in inputs.all_erasure_patterns(k + m, m, 0):
        for order in (list(pat), list(reversed(pat))):
            R, surv = gs.gs_decode_matrix(code, order)
            Ro, so = oracle.decode_matrix(P, order)
            assert surv == so and np.array_equal(R, Ro), (k, m, order)


def test_decode_matrix_errors():
    code = gs.gs_make_code(4, 2)
    for bad, status in [([0, 0], gs.GS_EINVAL), ([6], gs.GS_EINVAL), ([-1], gs.GS_EINVAL),
                        ([0, 1, 2], gs.GS_ETOOMANY)]:
        with pytest.raises(gs.GsError) as e:
            gs.gs_decode_matrix(code, bad)
        assert e.value.status == status


def _perm_b32(hi, lo, sel):
    """v_perm_b32 for selector bytes 0..7: byte s of the 64-bit value {hi:lo}."""
    pool = [(lo >> (8 * i)) & 0xFF for i in range(4)] + [(hi >> (8 * i)) & 0xFF for i in range(4)]
    out = 0
    for b in range(4):
        s = (sel >> (8 * b)) & 0xFF
        assert s < 8
        out |= pool[s] << (8 * b)
    return out


def test_lookup_words_multiply_every_byte_by_every_constant():
    t = _gfref.T()
    rng = np.random.default_rng(3)
    for c in range(256):
        w = gs.gs_coef_words(c)
        # all 256 byte values, four at a time, the way the kernel does it
        for base in range(0, 256, 4):
            d = base | (base + 1) << 8 | (base + 2) << 16 | (base + 3) << 24
            s0, s1, s2 = d & 0x07070707, (d >> 3) & 0x07070707, (d >> 6) & 0x03030303
            got = _perm_b32(w[1], w[0], s0) ^ _perm_b32(w[3], w[2], s1) ^ _perm_b32(w[4], w[4], s2)
            want = sum(int(t[c, base + i]) << (8 * i) for i in range(4))
            assert got == want, (c, base)
        d = int(rng.integers(0, 1 << 32))
        s0, s1, s2 = d & 0x07070707, (d >> 3) & 0x07070707, (d >> 6) & 0x03030303
        got = _perm_b32(w[1], w[0], s0) ^ _perm_b32(w[3], w[2], s1) ^ _perm_b32(w[4], w[4], s2)
        want = sum(int(t[c, (d >> (8 * i)) & 0xFF]) << (8 * i) for i in range(4))
        assert got == want


def test_entry_points_validate_before_touching_the_gpu():
    """Every check below fails in argument validation, so no HIP call is made."""
    L = gs.lib()
    code = gs.gs_make_code(4, 2)
    vp = ctypes.c_void_p
    good = (vp * 4)(0x1000, 0x2000, 0x3000, 0x4000)
    par = (vp * 2)(0x5000, 0x6000)
    odd = (vp * 4)(0x1000, 0x2001, 0x3000, 0x4000)
    null = (vp * 4)(0x1000, None, 0x3000, 0x4000)
    assert L.gs_encode(None, good, par, 64, None) == gs.GS_EINVAL
    assert L.gs_encode(code.handle, odd, par, 64, None) == gs.GS_EINVAL
    assert L.gs_encode(code.handle, null, par, 64, None) == gs.GS_EINVAL
    assert L.gs_encode(code.handle, good, None, 64, None) == gs.GS_EINVAL
    assert L.gs_encode(code.handle, good, par, 0, None) == gs.GS_OK          # empty shard: no-op
    six = (vp * 6)(0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000)
    er = (ctypes.c_int * 3)(0, 1, 2)
    assert L.gs_reconstruct(code.handle, six, er, 3, 64, None) == gs.GS_ETOOMANY
    er = (ctypes.c_int * 2)(1, 1)
    assert L.gs_reconstruct(code.handle, six, er, 2, 64, None) == gs.GS_EINVAL
    er = (ctypes.c_int * 1)(7)
    assert L.gs_reconstruct(code.handle, six, er, 1, 64, None) == gs.GS_EINVAL
    assert L.gs_reconstruct(code.handle, six, er, 0, 64, None) == gs.GS_OK   # nothing erased: no-op
    er = (ctypes.c_int * 1)(2)
    assert L.gs_reconstruct(code.handle, six, er, 1, 0, None) == gs.GS_OK    # empty shards: no-op
    # paged: page size must be a positive multiple of 16; sizes must be in range
    for page_bytes, n_planes, ppp, pps in [(0, 1, 8, 4), (24, 1, 8, 4), (64, -1, 8, 4), (64, 70000, 8, 4),
                                           (64, 1, 8, -2), (64, 1, 0, 4), (1 << 40, 1, 8, 4)]:
        assert L.gs_encode_paged(code.handle, 0x1000, n_planes, page_bytes, ppp, 0x2000, pps, par,
                                 None) == gs.GS_EINVAL
    assert L.gs_encode_paged(code.handle, 0x1000, 0, 64, 8, 0x2000, 4, par, None) == gs.GS_OK
    assert L.gs_encode_paged(code.handle, 0x1000, 3, 64, 8, 0x2000, 0, par, None) == gs.GS_OK
    out = vp()
    assert L.gs_pipe_create(code.handle, 100, 2, ctypes.byref(out)) == gs.GS_EINVAL   # not a multiple of 16
    assert L.gs_pipe_create(code.handle, 1024, 1, ctypes.byref(out)) == gs.GS_EINVAL  # depth < 2
    assert L.gs_set_launch_shape(3, 1, 1, -1) == gs.GS_EINVAL
    assert L.gs_set_launch_shape(2, 1, 1, 11) == gs.GS_EINVAL
    assert L.gs_set_launch_shape(0, 0, -1, -1) == gs.GS_OK
    assert L.gs_strerror(gs.GS_ETOOMANY).decode() == "more erasures than parity shards"


def test_runtime_failures_surface_as_status_codes_without_a_device():
    """With no GPU in the process every HIP call fails: object creation must clean up after itself
    and report GS_EHIP (never crash, never hand back a half-made object), a launch must report the
    runtime's error, and the host-only entry points must keep working."""
    torch = pytest.importorskip("torch")
    if torch.cuda.is_available():
        pytest.skip("needs a process without a GPU")
    L = gs.lib()
    code = gs.gs_make_code(4, 2)
    vp = ctypes.c_void_p
    out = vp(0xDEAD)
    assert L.gs_pipe_create(code.handle, 1024, 2, ctypes.byref(out)) == gs.GS_EHIP and not out.value
    assert L.gs_last_hip_error() != 0
    out = vp(0xDEAD)
    assert L.gs_batch_create(code.handle, 4, ctypes.byref(out)) == gs.GS_EHIP and not out.value
    out = vp(0xDEAD)
    assert L.gs_pool_create(2, ctypes.byref(out)) == gs.GS_EHIP and not out.value
    good = (vp * 4)(0x1000, 0x2000, 0x3000, 0x4000)
    par = (vp * 2)(0x5000, 0x6000)
    assert L.gs_encode(code.handle, good, par, 64, None) == gs.GS_EHIP
    assert "HIP" in L.gs_strerror(gs.GS_EHIP).decode()
    R, surv = gs.gs_decode_matrix(code, [1, 3])
    assert surv == [0, 2, 4, 5] and R.shape == (2, 4)
    assert gs.gs_recompute_units(10, 1.0, 0.0, 0.0, 1.0, 0.1)[0] in range(11)


def test_product_and_oracle_share_nothing():
    """The package never imports the oracle (and the oracle never the package); neither shared
    library carries the other's entry points."""
    import ast
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

    def imports_of(path):
        names = set()
        for node in ast.walk(ast.parse(open(path).read())):
            if isinstance(node, ast.Import):
                names.update(a.name.split(".")[0] for a in node.names)
            elif isinstance(node, ast.ImportFrom) and node.module:
                names.add(node.module.split(".")[0])
        return names

    def names_in_code(path, word):
        tree = ast.parse(open(path).read())
        docstrings = set()
        for node in ast.walk(tree):
            if isinstance(node, (ast.Module, ast.FunctionDef, ast.ClassDef)) and node.body and \
                    isinstance(node.body[0], ast.Expr) and isinstance(node.body[0].value, ast.Constant):
                docstrings.add(id(node.body[0].value))
        hits = []
        for node in ast.walk(tree):
            if isinstance(node, ast.Constant) and isinstance(node.value, str) and id(node) not in docstrings \
                    and word in node.value.lower():
                hits.append(node.value)
            elif isinstance(node, ast.Name) and word in node.id.lower():
                hits.append(node.id)
            elif isinstance(node, ast.Attribute) and word in node.attr.lower():
                hits.append(node.attr)
        return hits

    pkg = os.path.join(root, "paper_2605_00831_amd")
    for f in os.listdir(pkg):
        if f.endswith(".py"):
            assert "oracle" not in imports_of(os.path.join(pkg, f)), f
            # nor names it in code (a path to its sources, a dlopen, a subprocess): no string
            # literal other than a docstring, and no identifier, contains the word
            assert not names_in_code(os.path.join(pkg, f), "oracle"), f
    for f in os.listdir(os.path.join(root, "oracle")):
        if f.endswith(".py"):
            assert "paper_2605_00831_amd" not in imports_of(os.path.join(root, "oracle", f)), f
    for f in os.listdir(os.path.join(pkg, "csrc")):
        if not f.endswith((".h", ".c", ".cpp", ".hip")):
            continue
        text = open(os.path.join(pkg, "csrc", f)).read()
        assert "gso_" not in text and "oracle/" not in text, f

    def exported(lib):
        out = subprocess.run(["nm", "-D", "--defined-only", lib], stdout=subprocess.PIPE, text=True, check=True).stdout
        return {line.split()[-1] for line in out.splitlines() if line.strip()}

    import oracle
    product, checker = exported(gs.LIB_PATH), exported(oracle.build())
    assert not any(s.startswith("gso_") for s in product)
    assert not any(s.startswith("gs_") for s in checker)


def test_no_kernel_spills_registers_to_scratch_memory(tmp_path):
    """Every kernel of the library fits its register budget: the device assembly of each .hip file
    reports private_segment_fixed_size 0 for every kernel (a spill would add scratch traffic and a
    scratch allocation per wavefront to HBM-bound kernels)."""
    import re
    import subprocess
    from paper_2605_00831_amd import build as hip_build
    hips = [f for f in hip_build.SOURCES if f.endswith(".hip")]
    procs = []
    for f in hips:
        out = str(tmp_path / (f + ".s"))
        cmd = [hip_build.HIPCC] + [x for x in hip_build.FLAGS if x != "-fPIC"] + \
              ["--offload-device-only", "-S", "-o", out, os.path.join(hip_build.CSRC, f)]
        procs.append((f, out, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    kernels = 0
    for f, out, p in procs:
        log, _ = p.communicate()
        assert p.returncode == 0, log
        meta = re.findall(r"\.name:\s+(\S+)\n\s+\.private_segment_fixed_size:\s+(\d+)", open(out).read())
        assert meta, f
        kernels += len(meta)
        spilled = [(n, int(b)) for n, b in meta if int(b) != 0]
        assert not spilled, spilled
    assert kernels > 100


def test_binding_passes_address_arrays_through_unchanged():
    import ctypes

    import numpy as np

    from paper_2605_00831_amd import binding
    a = (np.arange(12, dtype=np.uint64) * 4096).reshape(3, 4)
    p = binding._flat_ptrs(a, 4)
    assert ctypes.addressof(p.contents) == a.ctypes.data and p[7] == 7 * 4096
    q = binding._flat_ptrs([[1, 2, 3, 4], [5, 6, 7, 8]], 4)
    assert list(q) == [1, 2, 3, 4, 5, 6, 7, 8]
    for bad in (a[:, :3], a.astype(np.uint32), np.asfortranarray(a), a.reshape(-1)):
        with pytest.raises(ValueError):
            binding._flat_ptrs(bad, 4)
    with pytest.raises(ValueError):
        binding._flat_ptrs([[1, 2, 3]], 4)
    s = binding._size_array(np.array([5, 6], dtype=np.uint64))
    assert s[0] == 5 and s[1] == 6
    assert list(binding._size_array([7, 8])) == [7, 8]
