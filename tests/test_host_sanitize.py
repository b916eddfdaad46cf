"""Builds tests/host_sanitize.cpp (the library's host-side field and matrix
code, no HIP) with g++ under AddressSanitizer and UBSan and runs it."""
import os
import subprocess
import tempfile

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def test_host_field_and_matrix_code_is_clean_under_asan_ubsan():
    with tempfile.TemporaryDirectory() as d:
        exe = os.path.join(d, "host_sanitize")
        subprocess.check_call(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined",
                               "-fno-sanitize-recover=all", "-static-libasan", "-o", exe, os.path.join(HERE, "host_sanitize.cpp")])
        out = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
        assert out.returncode == 0, out.stdout
        assert out.stdout.strip().endswith("OK")


SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all"]


TSAN = ["-fsanitize=thread"]


def compile_host_objects(tmp_path_factory, name, san):
    """The library's own sources compiled as host code only (no device code) under the given sanitizers.
    Programs linked from them can only run where there is no GPU."""
    torch = pytest.importorskip("torch")
    if torch.cuda.is_available():
        pytest.skip("host-only build: needs a process without a GPU")
    from paper_2605_00831_amd import build as hip_build
    d = str(tmp_path_factory.mktemp(name))
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
    return hip_build.HIPCC, d, objs


@pytest.fixture(scope="module")
def host_objects(tmp_path_factory):
    return compile_host_objects(tmp_path_factory, "host_objects", SAN)


def link_and_run(host_objects, driver, lang, san=SAN, env=None):
    hipcc, d, objs = host_objects
    drv = os.path.join(d, os.path.basename(driver) + ".o")
    std = ["-std=c++17"] if lang == "c++" else []
    subprocess.check_call([hipcc, "-O1", "-g", "-x", lang] + std + san +
                          ["-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-c", driver, "-o", drv])
    exe = os.path.join(d, os.path.basename(driver) + ".exe")
    # the device image is deliberately absent: its symbol stays unresolved and is never used without a GPU
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-static-libsan", "-pthread",
                           "-Wl,--unresolved-symbols=ignore-all"] + san + objs + [drv, "-o", exe])
    out = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300,
                         env=dict(os.environ, **(env or {})))
    assert out.returncode == 0, out.stdout[-3000:]
    assert out.stdout.strip().endswith("OK")


def test_host_side_of_every_entry_point_is_clean_under_asan_ubsan(host_objects):
    """tests/host_api_sanitize.c drives every entry point up to the launch, which fails in the
    runtime for want of a device."""
    link_and_run(host_objects, os.path.join(HERE, "host_api_sanitize.c"), "c")


def test_pipeline_pool_and_ring_orderings_hold_by_construction(host_objects):
    """tests/host_pipeline_order.cpp replaces the HIP runtime with a recorder that keeps a vector
    clock per enqueued operation, and checks the happens-before relations the checkpoint / restore
    pipelines, the stream pool and the descriptor ring rely on (removing any one of the pipelines'
    four event waits makes it fail); object creation under failing allocations leaks nothing."""
    link_and_run(host_objects, os.path.join(HERE, "host_pipeline_order.cpp"), "c++")


def test_shared_codes_and_process_wide_knobs_are_race_free_under_tsan(tmp_path_factory):
    """tests/host_threads_tsan.cpp: six threads use one set of codes at once, each with pipes, batches
    and a pool of its own, while one thread keeps changing the launch knobs and another makes and frees
    codes; ThreadSanitizer must stay silent (any report fails the run)."""
    objs = compile_host_objects(tmp_path_factory, "host_objects_tsan", TSAN)
    link_and_run(objs, os.path.join(HERE, "host_threads_tsan.cpp"), "c++", san=TSAN,
                 env={"TSAN_OPTIONS": "halt_on_error=1 exitcode=66"})
