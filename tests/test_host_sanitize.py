"""Builds tests/host_sanitize.cpp (the library's host-side field and matrix
code, no HIP) with g++ under AddressSanitizer and UBSan and runs it."""
import os
import subprocess
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))


def test_host_field_and_matrix_code_is_clean_under_asan_ubsan():
    with tempfile.TemporaryDirectory() as d:
        exe = os.path.join(d, "host_sanitize")
        subprocess.check_call(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined",
                               "-fno-sanitize-recover=all", "-static-libasan", "-o", exe, os.path.join(HERE, "host_sanitize.cpp")])
        out = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
        assert out.returncode == 0, out.stdout
        assert out.stdout.strip().endswith("OK")


def test_host_side_of_every_entry_point_is_clean_under_asan_ubsan():
    """The library's own sources, host code only (no device code is compiled or linked, so this
    can only run where there is no GPU), with tests/host_api_sanitize.c as the driver."""
    import pytest
    torch = pytest.importorskip("torch")
    if torch.cuda.is_available():
        pytest.skip("host-only build: needs a process without a GPU")
    from paper_2605_00831_amd import build as hip_build
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all"]
    with tempfile.TemporaryDirectory() as d:
        procs, objs = [], []
        for src in hip_build.SOURCES:
            obj = os.path.join(d, os.path.splitext(src)[0] + ".o")
            cmd = [hip_build.HIPCC, "--offload-arch=gfx950", "--cuda-host-only", "-O1", "-g", "-std=c++17"] + san + \
                  ["-x", "hip", "-c", os.path.join(hip_build.CSRC, src), "-o", obj]
            procs.append(subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True))
            objs.append(obj)
        for p in procs:
            out, _ = p.communicate()
            assert p.returncode == 0, out
        drv = os.path.join(d, "drv.o")
        subprocess.check_call([hip_build.HIPCC, "-O1", "-g", "-x", "c"] + san +
                              ["-c", os.path.join(HERE, "host_api_sanitize.c"), "-o", drv])
        exe = os.path.join(d, "host_api_sanitize")
        # the device image is deliberately absent: its symbol stays unresolved and is never used without a GPU
        subprocess.check_call([hip_build.HIPCC, "--offload-arch=gfx950", "-static-libsan",
                               "-Wl,--unresolved-symbols=ignore-all"] + san + objs + [drv, "-o", exe])
        out = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
        assert out.returncode == 0, out.stdout[-3000:]
        assert out.stdout.strip().endswith("OK")
