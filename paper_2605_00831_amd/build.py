"""Builds the HIP library in-tree:  python -m paper_2605_00831_amd.build

hipcc cross-compiles for gfx950 without a GPU.  The result,
paper_2605_00831_amd/libghostserve_ec.so, is what the binding loads.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libghostserve_ec.so")
SOURCES = ["gs_gf.cpp", "gs_api.cpp", "gs_pipeline.cpp", "gs_batch.cpp", "gs_plan.cpp", "gs_rdp.cpp", "gs_rdp_kernels.hip", "gs_kernels.hip"]
HEADERS = ["gs_gf.h", "gs_internal.h", "gs_launch.h", "gs_rdp.h", os.path.join("..", "..", "include", "ghostserve_ec.h")]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# packed-FP32 code generation is switched off for every HIP translation unit
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wextra",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def is_stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > t for f in SOURCES + HEADERS)


def build(verbose=True):
    """Compile every source and link the shared library (always recompiles)."""
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
        cmd = [HIPCC] + FLAGS + ["-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, out))
        if verbose and out.strip():
            print(out)
    tmp = LIB + ".%d.tmp" % os.getpid()
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


C_CHECK = os.path.join(os.path.dirname(HERE), "tests", "c_abi_roundtrip")


def build_c_check(verbose=True):
    """Plain C program against the C ABI (tests/c_abi_roundtrip.c), linked with the
    library and with the oracle's C file; tests/test_gpu_c_abi.py runs it."""
    root = os.path.dirname(HERE)
    cmd = [HIPCC, "-O2", "-x", "c", os.path.join(root, "tests", "c_abi_roundtrip.c"),
           os.path.join(root, "oracle", "gs_oracle.c"),
           "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-o", C_CHECK + ".tmp",
           "-L" + HERE, "-lghostserve_ec", "-Wl,-rpath,$ORIGIN/../paper_2605_00831_amd",
           "-L/opt/rocm/lib", "-lamdhip64", "-lpthread"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(C_CHECK + ".tmp", C_CHECK)
    return C_CHECK


STEP_LATENCY = os.path.join(HERE, "gs_step_latency")


def build_step_latency(verbose=True):
    """Native latency probe of the decode-step checkpoint (csrc/gs_step_latency.c); bench.py runs it."""
    cmd = [HIPCC, "-O2", "-x", "c", os.path.join(CSRC, "gs_step_latency.c"),
           "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-o", STEP_LATENCY + ".tmp",
           "-L" + HERE, "-lghostserve_ec", "-Wl,-rpath,$ORIGIN",
           "-L/opt/rocm/lib", "-lamdhip64"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(STEP_LATENCY + ".tmp", STEP_LATENCY)
    return STEP_LATENCY


if __name__ == "__main__":
    build()
    print("built", LIB)
    print("built", build_c_check())
    print("built", build_step_latency())
    sys.exit(0)
