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
SOURCES = ["gs_gf.cpp", "gs_api.cpp", "gs_pipeline.cpp", "gs_batch.cpp", "gs_plan.cpp", "gs_rdp.cpp", "gs_rdp_kernels.hip", "gs_kernels.hip", "gs_static.hip"]
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


if __name__ == "__main__":
    build()
    print("built", LIB)
    sys.exit(0)
