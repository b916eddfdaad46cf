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
