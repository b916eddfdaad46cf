"""Builds tests/c_abi_roundtrip: a plain C program (tests/c_abi_roundtrip.c) that uses
the library through its C ABI with only the HIP runtime in the process, and checks the
results against the oracle's C file linked into the same program.  Test infrastructure:
run by the driver's build step here, where there is a compiler; tests/test_gpu_c_abi.py
runs the program on the GPU machine.

    python -m tests.build_c_check
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
C_CHECK = os.path.join(HERE, "c_abi_roundtrip")


def build_c_check(verbose=True):
    pkg = os.path.join(ROOT, "paper_2605_00831_amd")
    cmd = [HIPCC, "-O2", "-x", "c", os.path.join(HERE, "c_abi_roundtrip.c"),
           os.path.join(ROOT, "oracle", "gs_oracle.c"),
           "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-o", C_CHECK + ".tmp",
           "-L" + pkg, "-lghostserve_ec", "-Wl,-rpath,$ORIGIN/../paper_2605_00831_amd",
           "-L/opt/rocm/lib", "-lamdhip64", "-lpthread"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(C_CHECK + ".tmp", C_CHECK)
    return C_CHECK


if __name__ == "__main__":
    print("built", build_c_check())
