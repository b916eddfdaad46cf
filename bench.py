#!/usr/bin/env python3
"""Benchmark of the erasure-code hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

A "step" is one pass of the hot path over the workload's resident KV bytes:
build the code and the rebuild matrix on the host, encode the k data shards
into m parity shards (gs_encode), then lose shards and rebuild them from the
survivors (gs_reconstruct).  `value` is the data bytes that pass through those
two kernels per second of wall time, inputs already in HBM.  The PCIe legs
(parity D2H pipeline, H2D restore), the paged per-step path and the CPU
oracle's rate are measured outside the timed steps and reported as extra
fields of the same JSON line.  The default run then frees the headline
workload and times the other bulk workloads (70B long context, recovery
stress) and the bulk paged gather the same way, each with its own roofline
object, under "configs" and "paged_bulk".
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
PCIE_GEN5_X16_GBPS = 64.0       # per direction, theoretical

# HBM traffic of one encode launch measured with rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE, scaled by a plain copy kernel of known size.  Bytes per launch,
# valid for the kernel template and the default launch shape named beside it;
# a run with another launch shape reports null.
MEASURED_TRAFFIC = {   # (workload, code): (FETCH_SIZE and WRITE_SIZE scaled to bytes, kernel, profile)
    ("llama8b_prefill", "cauchy"): (51539234413, "apply_contig_kernel<2, true, 2, true>",
                                    "profiles/encode_contig_llama8b_prefill.md"),
    ("llama8b_prefill", "power"): (51539233697, "horner_contig_kernel<2, 2, true>",
                                   "profiles/horner_power_code_llama8b_prefill.md"),
    ("llama70b_longctx", "cauchy"): (53686501590, "apply_contig_kernel<2, true, 2, true>",
                                     "profiles/encode_contig_llama70b_longctx.md"),
    ("recovery_stress", "cauchy"): (5905690725, "apply_contig_kernel<3, true, 2, true>",
                                    "profiles/encode_contig_recovery_stress.md"),
}


def traffic_fields(workload, code, default_shape):
    t = MEASURED_TRAFFIC.get((workload, code))
    if t is None or not default_shape:
        return {"traffic": None, "traffic_source": None if t is None else
                "not reported: the launch shape of this run differs from the profiled one (%s)" % t[2]}
    return {"traffic": t[0], "traffic_source": "%s: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of %s at the default launch "
                                               "shape (LDS reservation on), an earlier run of this command (not re-measured by this run)" % (t[2], t[1])}


NATIVE_SRC = os.path.join(ROOT, "bench_native.c")
NATIVE_EXE = os.path.join(ROOT, "bench_native")


def build_native(verbose=True):
    """Compile bench_native.c (plain C against the library's C ABI and the HIP runtime)."""
    import subprocess
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    pkg = os.path.join(ROOT, "paper_2605_00831_amd")
    cmd = [hipcc, "-O2", "-x", "c", NATIVE_SRC, "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-o", NATIVE_EXE + ".tmp",
           "-L" + pkg, "-lghostserve_ec", "-Wl,-rpath,$ORIGIN/paper_2605_00831_amd", "-L/opt/rocm/lib", "-lamdhip64"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(NATIVE_EXE + ".tmp", NATIVE_EXE)
    return NATIVE_EXE


def profiler_preloaded():
    """True when this process runs under a profiler that preloads a tool library (rocprofv3 does).
    Such a library may have initialised the GPU before the interpreter started, and starting another
    program from a GPU-initialised process is not allowed on the GPU machines."""
    for var in ("LD_PRELOAD", "ROCP_TOOL_LIBRARIES", "HSA_TOOLS_LIB", "ROCPROFILER_LIBRARY_CTOR"):
        if "rocprof" in os.environ.get(var, "").lower() or (var != "LD_PRELOAD" and os.environ.get(var)):
            return True
    return False


def native_probe(log, *argv):
    """Run bench_native (plain C, no interpreter in its timed loops) as a child process and return its JSON."""
    import subprocess
    if profiler_preloaded():
        return {"skipped": "a profiler tool library is preloaded; child processes are not started under a profiler"}
    if not os.path.exists(NATIVE_EXE):
        return {"error": "bench_native has not been built"}
    try:
        outp = subprocess.run([NATIVE_EXE] + [str(a) for a in argv], capture_output=True, text=True, timeout=240)
        if outp.returncode != 0:
            return {"error": "exit %d: %s" % (outp.returncode, outp.stderr.strip()[-200:])}
        res = json.loads(outp.stdout.strip().splitlines()[-1])
    except (subprocess.TimeoutExpired, ValueError, IndexError) as e:
        return {"error": repr(e)[:200]}
    log("[bench] native %s: %s" % (argv[0], json.dumps(res)))
    return res


_PINNED = None


def pinned_arena(torch, nbytes=0):
    """One pinned host allocation made when the run starts and shared, one after the other, by every
    leg that ships parity over PCIe: pinning tens of GiB takes seconds of host time, and nothing is
    unpinned or re-pinned in the middle of the run."""
    global _PINNED
    if _PINNED is None or _PINNED.numel() < nbytes:
        _PINNED = None
        _PINNED = torch.empty(max(nbytes, 1 << 20), dtype=torch.uint8, pin_memory=True)
    return _PINNED


_DEVICE = None


def device_arena(torch, nbytes):
    """One device allocation that the bulk workloads take their shards from, one after the other.
    Giving tens of GiB back to the driver in the middle of a run (hipFree) is not free on this
    machine: for a few seconds afterwards the driver is busy with the released memory, parity D2H
    through the copy engines ran at 31 GB/s instead of 56 and the HBM-bound kernels lost 3 points.
    So nothing large is freed between the legs."""
    global _DEVICE
    if _DEVICE is None or _DEVICE.numel() < nbytes:
        _DEVICE = None
        _DEVICE = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    return _DEVICE


def pinned_slices(torch, sizes):
    """len(sizes) disjoint pinned host buffers out of the arena (each start 4 KiB aligned)"""
    offs, at = [], 0
    for n in sizes:
        offs.append(at)
        at += (n + 4095) // 4096 * 4096
    arena = pinned_arena(torch, at)
    return [arena[o:o + n] for o, n in zip(offs, sizes)]


def pctl(xs, q):
    xs = sorted(xs)
    return xs[min(len(xs) - 1, int(q * len(xs)))]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama8b_prefill",
                    choices=["llama8b_prefill", "llama70b_longctx", "recovery_stress", "tiny"])
    ap.add_argument("--code", default="cauchy", choices=["cauchy", "power", "power-tables"],
                    help="code of the timed step: the canonical Cauchy code (default), the power code "
                         "(Horner encode kernel), or the power code through the general table kernel")
    ap.add_argument("--no-extras", action="store_true", help="skip PCIe pipelines, paged steps and CPU baseline")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 8 GiB device-to-device copy kernel (counter calibration under rocprofv3 --pmc)")
    ap.add_argument("--cpu-sample-mib", type=int, default=4096, help="bytes per shard for the CPU oracle leg")
    ap.add_argument("--launch-shape", default=None, metavar="U,T,NT,ILV",
                    help="gs_set_launch_shape(unroll, tiles_per_wg, nontemporal, interleave_shift) for sweeps; "
                         "0 / -1 keep a knob's default")
    ap.add_argument("--no-occupancy-cap", action="store_true",
                    help="gs_set_occupancy_cap(0): bulk launches without the LDS reservation that limits workgroups per CU")
    ap.add_argument("--only", default=None, choices=["headline", "paged_bulk", "rdp_forms", "launch_sizes"],
                    help="headline: the timed steps of --workload and its extras, not the other bulk workloads; "
                         "paged_bulk / rdp_forms / launch_sizes: only that leg (for profiling runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2

    log = lambda *a: print(*a, file=sys.stderr, flush=True)
    # The decode-step latency probe is a plain C program: run it as a child process first, before
    # this process opens the GPU, so that the two never hold the device at the same time.
    native = None
    if not args.no_extras and args.only not in ("paged_bulk", "rdp_forms", "launch_sizes"):
        native = {"decode": native_probe(log, "decode", inputs_steps(), 32), "many": native_probe(log, "many")}

    import torch
    from paper_2605_00831_amd import binding as gs
    from paper_2605_00831_amd import inputs

    gs.lib()  # hard error if the HIP library has not been built
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    dev = "cuda:0"
    if args.launch_shape:
        u, t, nt, ilv = (int(x) for x in args.launch_shape.split(","))
        gs.gs_set_launch_shape(u, t, nt, ilv)
    if args.no_occupancy_cap:
        gs.gs_set_occupancy_cap(False)
    if args.only in (None, "headline"):
        # the 70B workload with its parity, the largest of the bulk workloads: every workload then sits at the
        # same offsets of the same allocation whether it is timed alone or as part of the default run
        device_arena(torch, 50 << 30)
    if not args.no_extras:
        t0 = time.perf_counter()
        pinned_arena(torch, (16 << 30) + (1 << 20))   # the 8B workload's parity; every other leg needs less
        log("[bench] pinned %.1f GiB of host memory in %.1f s" % (_PINNED.numel() / 2**30, time.perf_counter() - t0))
    if args.only == "paged_bulk":
        print(json.dumps({"paged_bulk": paged_bulk(torch, gs, inputs, log, pipelines=not args.no_extras,
                                                   calibrate=args.calibrate_copy)}), flush=True)
        return 0

    if args.only == "rdp_forms":
        print(json.dumps({"rdp_forms": rdp_forms(torch, gs, inputs, log, calibrate=args.calibrate_copy)}), flush=True)
        return 0

    if args.only == "launch_sizes":
        print(json.dumps({"launch_sizes": launch_sizes(torch, gs, log, cap=not args.no_occupancy_cap)}), flush=True)
        return 0

    cfg = inputs.CONFIGS[args.workload]
    t0 = time.perf_counter()
    # recovery_stress loses a data shard, another data shard and a parity shard (one of its seeded triples)
    k, m, S, erased, data, parity = workload_buffers(torch, inputs, args.workload)
    torch.cuda.synchronize()
    log("[bench] workload %s: k=%d m=%d S=%.3f GiB total %.1f GiB, inputs generated in %.1f s"
        % (args.workload, k, m, S / 2**30, k * S / 2**30, time.perf_counter() - t0))
    shards = data + parity

    kind = gs.GS_CAUCHY if args.code == "cauchy" else gs.GS_POWER
    gs.gs_set_power_horner(args.code != "power-tables")

    def step(ev=None):
        code = gs.gs_make_code(k, m, kind)
        gs.gs_decode_matrix(code, erased)
        if ev:
            ev[0].record()
        gs.gs_encode(code, data, parity, S)
        if ev:
            ev[1].record()
        gs.gs_reconstruct(code, shards, erased, S)
        if ev:
            ev[2].record()

    if args.calibrate_copy:
        # a plain elementwise copy of known size: reads 8 GiB, writes 8 GiB
        parity[0].copy_(data[0])
        torch.cuda.synchronize()
        log("[bench] calibration copy: %d bytes read, %d bytes written" % (S, S))

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(evs[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    enc_ms = [e[0].elapsed_time(e[1]) for e in evs]
    rec_ms = [e[1].elapsed_time(e[2]) for e in evs]
    enc_avg, rec_avg = sum(enc_ms) / len(enc_ms), sum(rec_ms) / len(rec_ms)
    ms_per_step = wall * 1e3 / args.steps
    data_bytes_per_step = 2 * k * S  # k*S through encode + k*S of stripe restored by reconstruct
    value = data_bytes_per_step / (ms_per_step * 1e-3) / 1e9
    log("[bench] step %.3f ms: encode %.3f ms, reconstruct %.3f ms" % (ms_per_step, enc_avg, rec_avg))

    enc_alg_bytes = (k + m) * S
    rec_alg_bytes = (k + len(erased)) * S
    achieved = enc_alg_bytes / (enc_avg * 1e-3) / 1e9
    out = {
        "metric": "encode+reconstruct GB/s (data bytes) on 1 MI355X",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u8",
        "data": "synthetic",
        "config": {"workload": args.workload, "k": k, "m": m, "shard_bytes": S, "kv_dtype": cfg.get("dtype", "uniform bytes + bf16"),
                   "erased": erased, "code": args.code,
                   "launch": "gs_encode + gs_reconstruct, default launch shape"},
        "encode_GBps_data": round(k * S / (enc_avg * 1e-3) / 1e9, 1),
        "reconstruct_GBps_data": round(k * S / (rec_avg * 1e-3) / 1e9, 1),
        "encode_ms": round(enc_avg, 4),
        "reconstruct_ms": round(rec_avg, 4),
        "reconstruct_hbm_frac": round(rec_alg_bytes / (rec_avg * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "roofline": {
            "kernel": "%s (encode, k=%d m=%d)" % ("horner_contig_kernel" if args.code == "power" and m >= 2
                                                   else "apply_contig_kernel", k, m),
            "bound": "hbm",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBPS, 4),
            "algorithmic_bytes_per_launch": enc_alg_bytes,
            "avg_launch_ms": round(enc_avg, 4),
            **traffic_fields(args.workload, args.code, args.launch_shape is None and not args.no_occupancy_cap),
        },
    }

    # the paper's own headline figures, on its hardware: context, not a target and not comparable
    out["paper_context"] = {
        "checkpoint_latency_gain_vs_cpu_replication": "2.7x (prefill, average; Section 6.2)",
        "recovery_latency_gain": "2.1x (single batch; abstract and Section 6.2; the conclusion swaps the two figures)",
        "hardware": "8x NVIDIA H200 over NVLink, host link PCIe Gen 4; end-to-end serving latencies, "
                    "no kernel GB/s is printed in the paper's text",
    }
    if not args.no_extras:
        out.update(extras(torch, gs, inputs, args, cfg, k, m, S, data, parity, shards, erased, log, native))

    if args.only is None and args.code == "cauchy":
        # the other bulk workloads, timed the same way after the headline workload's buffers are gone
        del data, parity, shards
        out["configs"] = [dict(workload=args.workload, kernel=out["roofline"]["kernel"],
                               algorithmic_bytes_per_launch=enc_alg_bytes, avg_launch_ms=out["roofline"]["avg_launch_ms"],
                               frac=out["roofline"]["frac"], reconstruct_ms=out["reconstruct_ms"],
                               reconstruct_frac=out["reconstruct_hbm_frac"], erased=erased,
                               checkpoint_ms=out.get("checkpoint", {}).get("latency_ms"),
                               restore_ms=out.get("restore", {}).get("latency_ms"))]
        for name in ("llama8b_prefill", "llama70b_longctx", "recovery_stress"):
            if name != args.workload:
                out["configs"].append(bulk_config(torch, gs, inputs, name, max(args.steps, 20), args.warmup, log,
                                                  pipelines=not args.no_extras,
                                                  default_shape=args.launch_shape is None and not args.no_occupancy_cap))
        out["paged_bulk"] = paged_bulk(torch, gs, inputs, log, pipelines=not args.no_extras)
        out["code_shapes"] = code_shapes(torch, gs, log)
        out["rdp_forms"] = rdp_forms(torch, gs, inputs, log)
        out["launch_sizes"] = launch_sizes(torch, gs, log, cap=not args.no_occupancy_cap)

    print(json.dumps(out), flush=True)
    return 0


def inputs_steps():
    from paper_2605_00831_amd import inputs
    return inputs.CONFIGS["decode_paged"]["steps"]


def workload_buffers(torch, inputs, name, dev="cuda:0"):
    """(k, m, S, erased, data shards, parity shards) of a bulk workload, generated on the device
    inside the device arena."""
    cfg = inputs.CONFIGS[name]
    k, m = cfg["k"], cfg["m"]
    total = inputs.config_total_bytes(name)
    S = total // k
    erased = list(cfg.get("erased", (2, 5, 9) if name == "recovery_stress" else (1, 3) if k >= 4 else (0,)))[:m]
    arena = device_arena(torch, (k + m) * S)
    buf = arena[:total]
    if name == "recovery_stress":
        half = (k // 2) * S
        inputs.uniform_bytes_device(inputs.config_seed(name), half, dev, out=buf[:half])
        inputs.kv_bytes_device(inputs.config_seed(name) + 1, total - half, "bf16", 1.0, dev, out=buf[half:])
    else:
        inputs.kv_bytes_device(inputs.config_seed(name), total, cfg["dtype"], cfg["sigma"], dev, out=buf)
    data = [buf[j * S:(j + 1) * S] for j in range(k)]
    parity = [arena[(k + i) * S:(k + i + 1) * S] for i in range(m)]
    return k, m, S, erased, data, parity


def bulk_config(torch, gs, inputs, name, launches, warmup, log, pipelines=True, default_shape=True):
    """One more bulk workload: `launches` encode and reconstruct launches, each between events on the
    launch stream, then (optionally) the checkpoint and restore pipelines of that workload."""
    cfg = inputs.CONFIGS[name]
    k, m, S, erased, data, parity = workload_buffers(torch, inputs, name)
    shards = data + parity
    code = gs.gs_make_code(k, m)
    for _ in range(max(warmup, 1)):
        gs.gs_encode(code, data, parity, S)
        gs.gs_reconstruct(code, shards, erased, S)
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(launches)]
    for ev in evs:
        ev[0].record()
        gs.gs_encode(code, data, parity, S)
        ev[1].record()
        gs.gs_reconstruct(code, shards, erased, S)
        ev[2].record()
    torch.cuda.synchronize()
    enc = sum(e[0].elapsed_time(e[1]) for e in evs) / launches
    rec = sum(e[1].elapsed_time(e[2]) for e in evs) / launches
    enc_bytes, rec_bytes = (k + m) * S, (k + len(erased)) * S
    res = {"workload": name, "k": k, "m": m, "shard_bytes": S, "erased": erased, "launches": launches,
           "kernel": "apply_contig_kernel (encode, k=%d m=%d)" % (k, m),
           "algorithmic_bytes_per_launch": enc_bytes, "avg_launch_ms": round(enc, 4),
           "achieved": round(enc_bytes / enc / 1e6, 1), "frac": round(enc_bytes / enc / 1e6 / HBM_PEAK_GBPS, 4),
           "encode_GBps_data": round(k * S / enc / 1e6, 1),
           "reconstruct_algorithmic_bytes_per_launch": rec_bytes, "reconstruct_ms": round(rec, 4),
           "reconstruct_frac": round(rec_bytes / rec / 1e6 / HBM_PEAK_GBPS, 4),
           "reconstruct_GBps_data": round(k * S / rec / 1e6, 1),
           **traffic_fields(name, "cauchy", default_shape)}
    if pipelines:
        chunk_tokens = cfg.get("chunk_tokens")
        if chunk_tokens:
            chunk = chunk_tokens * cfg["batch"] * inputs.bytes_per_token(cfg["layers"]) // k
        else:
            chunk = max(16, (S // 4 + 15) // 16 * 16)
        host = pinned_slices(torch, [S] * m)
        pipe = gs.gs_pipe_create(code, chunk, 2)

        def best(fn, n=5):
            ts = []
            for _ in range(n):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                fn()
                gs.gs_pipe_sync(pipe)
                ts.append(time.perf_counter() - t0)
            return min(ts)
        ck = best(lambda: gs.gs_checkpoint(pipe, data, S, host))
        rs = best(lambda: gs.gs_restore(pipe, shards, host, erased, S))
        n_back = sum(1 for s in gs.gs_decode_matrix(code, erased)[1] if s >= k)
        res.update({"chunk_bytes_per_shard": chunk, "checkpoint_ms": round(ck * 1e3, 2),
                    "checkpoint_parity_GBps": round(m * S / ck / 1e9, 2),
                    "checkpoint_frac_of_pcie_gen5_x16": round(m * S / ck / 1e9 / PCIE_GEN5_X16_GBPS, 3),
                    "restore_ms": round(rs * 1e3, 2), "restore_parity_shards_from_host": n_back,
                    "restore_parity_h2d_GBps": round(n_back * S / rs / 1e9, 2)})
        gs.gs_pipe_destroy(pipe)
        del host
    log("[bench] config %s: %s" % (name, json.dumps(res)))
    return res


def code_shapes(torch, gs, log):
    """gs_encode over 40 GiB in total (data + parity) for a range of code shapes, default launch shape:
    how the number of streams and of parity rows moves the HBM fraction.  Events around 7 launches."""
    total = 40 << 30
    arena = device_arena(torch, total)
    arena[:total].random_(0, 256)   # the rate depends on the data: all-zero buffers run about 2 points faster
    rows = []
    for k, m in ((1, 1), (2, 1), (2, 2), (4, 1), (4, 2), (8, 1), (8, 2), (8, 3), (8, 4), (16, 1), (16, 2), (16, 4), (1, 4)):
        S = total // (k + m) // 4096 * 4096
        shards = [arena[j * S:(j + 1) * S] for j in range(k + m)]
        code = gs.gs_make_code(k, m)
        for _ in range(2):
            gs.gs_encode(code, shards[:k], shards[k:], S)
        torch.cuda.synchronize()
        n = 7
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
        evs[0].record()
        for i in range(n):
            gs.gs_encode(code, shards[:k], shards[k:], S)
            evs[i + 1].record()
        torch.cuda.synchronize()
        ms = sorted(evs[i].elapsed_time(evs[i + 1]) for i in range(n))[n // 2]
        rows.append({"k": k, "m": m, "shard_bytes": S, "encode_ms": round(ms, 4),
                     "frac": round((k + m) * S / ms / 1e6 / HBM_PEAK_GBPS, 4)})
    log("[bench] code shapes: " + json.dumps(rows))
    return rows


def launch_sizes(torch, gs, log, cap=True):
    """One launch against its size, 64 KiB to 1 GiB per shard (4+2 and 8+2; encode, and the rebuild of
    shards 1 and 3): microseconds per launch from events around back-to-back launches, the HBM fraction
    that is, and for launches that do not fill the chip the time from the call to an idle stream as a
    host thread sees it.  Bulk sizes are timed with the LDS reservation on and off.  The library picks
    a kernel form by size (four streams' loads together up to 1024 workgroups of 8 KiB per stream, one
    stream at a time above, fewer workgroups per CU from 48 MiB on); this leg shows all three regimes.
    (The small-launch form against the bulk form on small launches is timed from C, without the
    interpreter's per-call cost: `many_chunks.from_c`, `decode_step.native`.)"""
    arena = device_arena(torch, 11 << 30)
    arena[:11 << 30].random_(0, 256)   # never time fresh (all-zero) memory: it runs about 2 points faster than real bytes
    rows = []

    def per_launch_us(fn, n):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        best = None
        for _ in range(5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(n):
                fn()
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1000.0 / n
            best = us if best is None or us < best else best
        return best

    def to_idle_us(fn, n=200):
        ts = []
        for i in range(n + 20):
            t0 = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            if i >= 20:
                ts.append(time.perf_counter() - t0)
        return pctl(ts, 50) * 1e6

    for k, m in ((4, 2), (8, 2)):
        code = gs.gs_make_code(k, m)
        for S in (64 << 10, 1 << 20, 4 << 20, 8 << 20, 16 << 20, 32 << 20, 48 << 20, 64 << 20, 96 << 20, 128 << 20,
                  256 << 20, 1 << 30):
            shards = [arena[j * S:(j + 1) * S] for j in range(k + m)]
            enc = lambda: gs.gs_encode(code, shards[:k], shards[k:], S)
            rec = lambda: gs.gs_reconstruct(code, shards, [1, 3], S)
            enc()
            n = 200 if S <= (8 << 20) else 40 if S <= (128 << 20) else 10
            row = {"k": k, "m": m, "shard_bytes": S, "workgroups": (S + 8191) // 8192}
            for name, fn in (("encode", enc), ("reconstruct", rec)):
                us = per_launch_us(fn, n)
                row[name] = {"us": round(us, 2), "frac": round((k + m) * S / us / 1e3 / HBM_PEAK_GBPS, 4)}
                if S <= (8 << 20):
                    row[name]["call_to_idle_us"] = round(to_idle_us(fn), 1)
                if cap and S >= (48 << 20):
                    gs.gs_set_occupancy_cap(False)
                    try:
                        us = per_launch_us(fn, n)
                    finally:
                        gs.gs_set_occupancy_cap(True)
                    row[name]["frac_without_reservation"] = round((k + m) * S / us / 1e3 / HBM_PEAK_GBPS, 4)
                if S >= (16 << 20):
                    # the form of small launches at this size: the loads of four streams issued together,
                    # with the reservation of the size and (the design before one stream at a time) without
                    gs.gs_set_size_forms(2)
                    try:
                        us = per_launch_us(fn, n)
                        row[name]["frac_four_streams_together"] = round((k + m) * S / us / 1e3 / HBM_PEAK_GBPS, 4)
                        if cap and S >= (48 << 20):
                            gs.gs_set_occupancy_cap(False)
                            us = per_launch_us(fn, n)
                            row[name]["frac_four_streams_together_without_reservation"] = \
                                round((k + m) * S / us / 1e3 / HBM_PEAK_GBPS, 4)
                    finally:
                        gs.gs_set_size_forms(1)
                        gs.gs_set_occupancy_cap(cap)
            rows.append(row)
    # a rebuild of three shards with the all-ones parity among the survivors: one lost shard as a plain XOR
    # (the default) against three lookup rows (gs_set_size_forms(0)), in one process on the same buffers
    k, m, S, erased = 8, 3, 512 << 20, [2, 5, 9]
    code = gs.gs_make_code(k, m)
    shards = [arena[j * S:(j + 1) * S] for j in range(k + m)]
    gs.gs_encode(code, shards[:k], shards[k:], S)
    rec = lambda: gs.gs_reconstruct(code, shards, erased, S)
    row = {"k": k, "m": m, "shard_bytes": S, "erased": erased}
    for name, on in (("xor_fold", True), ("lookup_rows", False), ("xor_fold_again", True), ("lookup_rows_again", False)):
        gs.gs_set_size_forms(on)
        try:
            us = per_launch_us(rec, 10)
        finally:
            gs.gs_set_size_forms(True)
        row[name] = {"us": round(us, 2), "frac": round((k + len(erased)) * S / us / 1e3 / HBM_PEAK_GBPS, 4)}
    rows.append({"rebuild_of_three_shards": row})
    log("[bench] launch sizes: " + json.dumps(rows))
    return rows


def paged_bulk(torch, gs, inputs, log, pipelines=True, calibrate=False):
    """Bulk paged gather (the recovery-stress shape on a paged pool): 64 planes of 272 MiB, shards of
    2 GiB gathered through a block table, 32 KiB pages (16-token blocks) and 2 KiB pages (token slots),
    behind a seeded random permutation and, as controls, behind identity tables and behind permutations
    of runs of consecutive pages; 4+2, 8+3 and the paper's default ratio 8+2.
    Each case: events around 10 launches on the launch stream.  Then the paged checkpoint / restore
    pipelines (8+3, 32 KiB pages, shards {2, 5} and parity shard 9 lost)."""
    dev = "cuda:0"
    n_planes, shard_per_plane = 64, 32 << 20
    # room for 8 shards per plane plus a margin, so that one identity control can keep its shards off
    # power-of-two distances from each other (equal offsets of streams exactly 32 MiB apart fall on the
    # same DRAM banks, which costs the contiguous kernels the same 5 points)
    plane_bytes = 8 * (shard_per_plane + (2 << 20))
    S = n_planes * shard_per_plane
    arena = device_arena(torch, n_planes * plane_bytes + 3 * S)
    pool = inputs.kv_bytes_device(inputs.config_seed("recovery_stress") + 7, n_planes * plane_bytes, "bf16", 1.0, dev,
                                  out=arena[:n_planes * plane_bytes])
    base = torch.tensor([pool.data_ptr() + p * plane_bytes for p in range(n_planes)], dtype=torch.int64, device=dev)
    par = [arena[n_planes * plane_bytes + i * S: n_planes * plane_bytes + (i + 1) * S] for i in range(3)]
    if calibrate:
        # a plain elementwise copy of known size (counter calibration under rocprofv3 --pmc)
        par[0].copy_(par[1])
        torch.cuda.synchronize()
        log("[bench] calibration copy: %d bytes read, %d bytes written" % (S, S))
    cases = []
    tables = {}
    for page in (32768, 2048):
        ppp, pps = plane_bytes // page, shard_per_plane // page
        perm = inputs.block_table_np(inputs.config_seed("recovery_stress"), 8, pps, ppp)
        skew = (2 << 20) // page   # identity control: shard j starts at j * (32 MiB + 2 MiB) of its plane
        ident = (np.arange(8, dtype=np.int32)[:, None] * (pps + skew) + np.arange(pps, dtype=np.int32)[None, :])
        dense = np.arange(8 * pps, dtype=np.int32).reshape(8, pps)
        variants = [("random permutation", perm), ("identity, shards 34 MiB apart", ident),
                    ("identity, shards 32 MiB apart", dense)]
        if page == 32768:
            # an allocator that hands out pages in runs: the pool permuted in units of 2, 8 and 128 pages
            rng = np.random.default_rng(inputs.config_seed("recovery_stress") + inputs.TABLE_SEED_OFFSET + 1)
            for run in (2, 8, 128):
                starts = rng.permutation(ppp // run)[: 8 * pps // run]
                runs = (starts[:, None] * run + np.arange(run)[None, :]).reshape(8, pps)
                variants.append(("random permutation of runs of %d pages (%d KiB)" % (run, run * page >> 10), runs))
        for tname, tab in variants:
            table = torch.from_numpy(np.ascontiguousarray(tab.astype(np.int32))).to(dev)
            tables[(page, tname)] = table
            for k, m in ((4, 2), (8, 3), (8, 2)):
                code = gs.gs_make_code(k, m)
                fn = lambda: gs.gs_encode_paged(code, base, n_planes, page, ppp, table, pps, par[:m])
                for _ in range(3):
                    fn()
                torch.cuda.synchronize()
                n = 10
                evs = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
                evs[0].record()
                for i in range(n):
                    fn()
                    evs[i + 1].record()
                torch.cuda.synchronize()
                ms = sum(evs[i].elapsed_time(evs[i + 1]) for i in range(n)) / n
                alg = (k + m) * S
                cases.append({"k": k, "m": m, "page_bytes": page, "table": tname, "shard_bytes": S, "launches": n,
                              "roofline": {"kernel": "apply_paged_kernel (encode, k=%d m=%d)" % (k, m), "bound": "hbm",
                                           "achieved": round(alg / ms / 1e6, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                           "frac": round(alg / ms / 1e6 / HBM_PEAK_GBPS, 4), "traffic": None,
                                           "algorithmic_bytes_per_launch": alg, "avg_launch_ms": round(ms, 4)}})
    # controls: the contiguous kernel on shards of the same length laid out back to back, and the paged
    # kernel over exactly those addresses (one plane, identity table)
    controls = []
    page = 32768
    one_plane = torch.tensor([arena.data_ptr()], dtype=torch.int64, device=dev)
    for k, m in ((4, 2), (8, 3)):
        code = gs.gs_make_code(k, m)
        shards = [arena[j * S:(j + 1) * S] for j in range(k + m)]
        ident = torch.arange(k * (S // page), dtype=torch.int32, device=dev).reshape(k, S // page).contiguous()
        for name, fn in (("gs_encode, contiguous shards", lambda: gs.gs_encode(code, shards[:k], shards[k:], S)),
                         ("gs_encode_paged, one plane, identity table, the same addresses",
                          lambda: gs.gs_encode_paged(code, one_plane, 1, page, (k + m) * (S // page), ident, S // page, shards[k:]))):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(10):
                fn()
            b.record()
            torch.cuda.synchronize()
            ms = a.elapsed_time(b) / 10
            controls.append({"k": k, "m": m, "what": name, "shard_bytes": S, "avg_launch_ms": round(ms, 4),
                             "frac": round((k + m) * S / ms / 1e6 / HBM_PEAK_GBPS, 4)})
    res = {"pool": "%d planes x %d MiB, %d MiB of every shard per plane" % (n_planes, plane_bytes >> 20, shard_per_plane >> 20),
           "cases": cases, "controls": controls}
    if pipelines:
        k, m, page, erased = 8, 3, 32768, [2, 5, 9]
        ppp, pps = plane_bytes // page, shard_per_plane // page
        table = tables[(page, "random permutation")]
        code = gs.gs_make_code(k, m)
        host = pinned_slices(torch, [S] * m)
        chunk = S // 8
        pipe = gs.gs_pipe_create(code, chunk, 2)

        def best(fn, n=5):
            ts = []
            for _ in range(n):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                fn()
                gs.gs_pipe_sync(pipe)
                ts.append(time.perf_counter() - t0)
            return min(ts)
        ck = best(lambda: gs.gs_checkpoint_paged(pipe, base, n_planes, page, ppp, table, pps, host))
        rs = best(lambda: gs.gs_restore_paged(pipe, base, n_planes, page, ppp, table, pps, host, erased, parity_out=par))
        res["pipelines"] = {"k": k, "m": m, "page_bytes": page, "erased": erased, "chunk_bytes_per_shard": chunk,
                            "checkpoint_paged_ms": round(ck * 1e3, 2), "checkpoint_parity_GBps": round(m * S / ck / 1e9, 2),
                            "checkpoint_frac_of_pcie_gen5_x16": round(m * S / ck / 1e9 / PCIE_GEN5_X16_GBPS, 3),
                            "restore_paged_ms": round(rs * 1e3, 2), "restore_parity_h2d_GBps": round(2 * S / rs / 1e9, 2)}
        gs.gs_pipe_destroy(pipe)
    log("[bench] paged bulk: " + json.dumps(res))
    return res


def extras(torch, gs, inputs, args, cfg, k, m, S, data, parity, shards, erased, log, native=None):
    res = {}
    dev = "cuda:0"
    code = gs.gs_make_code(k, m)

    # ---- checkpoint latency: chunked encode overlapped with parity D2H into pinned memory
    chunk_tokens = cfg.get("chunk_tokens")
    if chunk_tokens:
        per_tok = inputs.bytes_per_token(cfg["layers"])
        chunk = chunk_tokens * cfg["batch"] * per_tok // k
    else:
        chunk = max(16, (S // 4 + 15) // 16 * 16)
    host = pinned_slices(torch, [S] * m)
    # plain pinned D2H / H2D rate of one parity shard, same run
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    host[0].copy_(parity[0], non_blocking=True)
    torch.cuda.synchronize()
    d2h = S / (time.perf_counter() - t0) / 1e9
    t0 = time.perf_counter()
    parity[0].copy_(host[0], non_blocking=True)
    torch.cuda.synchronize()
    h2d = S / (time.perf_counter() - t0) / 1e9
    # context: shipping the data itself (full replication) instead of the parity
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for j in range(k):
        host[j % m].copy_(data[j], non_blocking=True)
    torch.cuda.synchronize()
    replication = time.perf_counter() - t0
    pipe = gs.gs_pipe_create(code, chunk, 2)
    lat = []
    for _ in range(3):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        gs.gs_checkpoint(pipe, data, S, host)
        gs.gs_pipe_sync(pipe)
        lat.append(time.perf_counter() - t0)
    ck = min(lat)
    # the same pipeline once more with its per-chunk timing on: when each chunk's encode ran and
    # when its parity had landed in host memory (ms since the call began)
    gs.gs_pipe_set_timing(pipe, True)
    gs.gs_checkpoint(pipe, data, S, host)
    timeline = gs.gs_pipe_chunk_times(pipe)
    gs.gs_pipe_set_timing(pipe, False)
    # serial reference: encode everything, then copy everything
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    gs.gs_encode(code, data, parity, S)
    for i in range(m):
        host[i].copy_(parity[i], non_blocking=True)
    torch.cuda.synchronize()
    serial = time.perf_counter() - t0
    res["checkpoint"] = {
        "latency_ms": round(ck * 1e3, 2), "chunk_bytes_per_shard": chunk, "parity_bytes": m * S,
        "parity_GBps": round(m * S / ck / 1e9, 2),
        "frac_of_pcie_gen5_x16": round(m * S / ck / 1e9 / PCIE_GEN5_X16_GBPS, 3),
        "plain_pinned_d2h_GBps": round(d2h, 2), "plain_pinned_h2d_GBps": round(h2d, 2),
        "frac_of_plain_d2h": round(m * S / ck / 1e9 / d2h, 3),
        "unpipelined_encode_then_copy_ms": round(serial * 1e3, 2),
        "data_GBps_pcie_inclusive": round(k * S / ck / 1e9, 1),
        "timeline_ms": [{"chunk": c, "encode": [round(kb, 2), round(ke, 2)], "parity_in_host_memory": round(ce, 2)}
                        for c, (kb, ke, ce) in enumerate(timeline)],
        "encode_busy_ms": round(sum(ke - kb for kb, ke, _ in timeline), 2),
        "full_replication_d2h_ms": round(replication * 1e3, 2),
        "replication_over_checkpoint": round(replication / ck, 2),
    }
    log("[bench] checkpoint %.1f ms (parity %.1f GB/s, plain D2H %.1f GB/s, unpipelined %.1f ms)"
        % (ck * 1e3, m * S / ck / 1e9, d2h, serial * 1e3))

    # ---- what the checkpoint costs other GPU work: a stream of HBM-bound 1 GiB device copies
    # (stand-in for serving kernels), timed alone and while a checkpoint runs beside it
    a_buf = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 256)
    b_buf = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    side, cstream = torch.cuda.Stream(), torch.cuda.Stream()

    def side_copies(n):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(side):
            e0.record(side)
            for _ in range(n):
                b_buf.copy_(a_buf)
            e1.record(side)
        return e0, e1

    e0, e1 = side_copies(50)
    torch.cuda.synchronize()
    n_side = max(10, int(0.8 * ck * 1e3 / (e0.elapsed_time(e1) / 50)))
    e0, e1 = side_copies(n_side)
    torch.cuda.synchronize()
    alone_ms = e0.elapsed_time(e1)
    gs.gs_checkpoint(pipe, data, S, host, cstream.cuda_stream)
    e0, e1 = side_copies(n_side)
    gs.gs_pipe_sync(pipe)
    torch.cuda.synchronize()
    beside_ms = e0.elapsed_time(e1)
    res["checkpoint"]["concurrent_work"] = {
        "what": "%d device copies of 1 GiB on another stream" % n_side, "alone_ms": round(alone_ms, 2),
        "beside_checkpoint_ms": round(beside_ms, 2), "slowdown": round(beside_ms / alone_ms, 4)}
    log("[bench] concurrent work: alone %.1f ms, beside a checkpoint %.1f ms" % (alone_ms, beside_ms))
    del a_buf, b_buf

    # ---- restore latency: parity H2D overlapped with reconstruct
    lat = []
    for _ in range(2):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        gs.gs_restore(pipe, data + parity, host, erased, S)
        gs.gs_pipe_sync(pipe)
        lat.append(time.perf_counter() - t0)
    n_par = len(erased)  # every erased data shard pulls one parity shard back
    gs.gs_pipe_set_timing(pipe, True)
    gs.gs_restore(pipe, data + parity, host, erased, S)
    rtl = gs.gs_pipe_chunk_times(pipe)
    gs.gs_pipe_set_timing(pipe, False)
    res["restore"] = {"latency_ms": round(min(lat) * 1e3, 2), "erased": erased,
                      "parity_h2d_GBps": round(n_par * S / min(lat) / 1e9, 2),
                      "timeline_ms": [{"chunk": c, "parity_on_device": round(ce, 2),
                                       "reconstruct": [round(kb, 2), round(ke, 2)]}
                                      for c, (kb, ke, ce) in enumerate(rtl)],
                      "reconstruct_busy_ms": round(sum(ke - kb for kb, ke, _ in rtl), 2)}
    log("[bench] restore %.1f ms" % (min(lat) * 1e3))
    gs.gs_pipe_destroy(pipe)

    # ---- hybrid recovery plan from the rates measured above: how many of the leading chunks to
    # recompute, for recompute costs given as multiples of one chunk's restore time
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    gs.gs_reconstruct(code, shards, erased, S)
    b.record()
    torch.cuda.synchronize()
    n_chunks = (S + chunk - 1) // chunk
    h2d_s = n_par * chunk / (h2d * 1e9)
    rec_s = a.elapsed_time(b) * 1e-3 * chunk / S
    stage = max(h2d_s, rec_s)
    plan = {}
    for mult in (0.25, 0.5, 1.0, 2.0, 4.0):
        r, t = gs.gs_recompute_units(n_chunks, mult * stage, 0.0, 0.0, h2d_s, rec_s)
        plan["recompute_cost_x%g" % mult] = {"recompute_chunks": r, "makespan_ms": round(t * 1e3, 2)}
    res["recovery_plan"] = {"n_chunks": n_chunks, "h2d_ms_per_chunk": round(h2d_s * 1e3, 3),
                            "reconstruct_ms_per_chunk": round(rec_s * 1e3, 3), "plans": plan}
    log("[bench] recovery plan: " + json.dumps(res["recovery_plan"]))

    # ---- the XOR-only RDP code on the same shards (needs k <= 16 and whole stripes)
    if k <= 16 and m >= 2:
        rdp = gs.gs_make_code(k, 2, gs.GS_RDP)
        stripe = (gs.gs_rdp_prime(rdp) - 1) * gs.gs_rdp_cell_bytes(rdp)
        Sr = S // stripe * stripe
        if Sr:
            def ev_ms(fn, n=5):
                ts = []
                for _ in range(n + 1):
                    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    a.record()
                    fn()
                    b.record()
                    torch.cuda.synchronize()
                    ts.append(a.elapsed_time(b))
                return sorted(ts[1:])[n // 2]
            enc = ev_ms(lambda: gs.gs_encode(rdp, data, parity[:2], Sr))
            rec = ev_ms(lambda: gs.gs_reconstruct(rdp, data + parity[:2], erased[:2], Sr))
            res["rdp"] = {"prime": gs.gs_rdp_prime(rdp), "cell_bytes": gs.gs_rdp_cell_bytes(rdp), "shard_bytes": Sr,
                          "encode_ms": round(enc, 4), "encode_hbm_frac": round((k + 2) * Sr / enc / 1e6 / HBM_PEAK_GBPS, 4),
                          "reconstruct_ms": round(rec, 4),
                          "reconstruct_hbm_frac": round((k + len(erased[:2])) * Sr / rec / 1e6 / HBM_PEAK_GBPS, 4)}
            # the same encode through the paged entry point (one plane over the arena, identity table,
            # a page = a cell) and as one grouped launch over 16 chunks of whole stripes
            cell = gs.gs_rdp_cell_bytes(rdp)
            lo = min(d.data_ptr() for d in data)
            if all((d.data_ptr() - lo) % cell == 0 for d in data):
                pps = Sr // cell
                tab = torch.stack([torch.arange(pps, dtype=torch.int32, device=dev) + (d.data_ptr() - lo) // cell
                                   for d in data]).contiguous()
                span = max(d.data_ptr() for d in data) + Sr - lo
                one_plane = torch.tensor([lo], dtype=torch.int64, device=dev)
                pg = ev_ms(lambda: gs.gs_encode_paged(rdp, one_plane, 1, cell, span // cell, tab, pps, parity[:2]))
                res["rdp"]["encode_paged_identity_ms"] = round(pg, 4)
                res["rdp"]["encode_paged_identity_hbm_frac"] = round((k + 2) * Sr / pg / 1e6 / HBM_PEAK_GBPS, 4)
            n_g = 16
            per = Sr // stripe // n_g * stripe
            if per:
                batch = gs.gs_batch_create(rdp, n_g)
                gd = [[d[c * per:(c + 1) * per] for d in data] for c in range(n_g)]
                gp = [[q[c * per:(c + 1) * per] for q in parity[:2]] for c in range(n_g)]
                gr = ev_ms(lambda: gs.gs_encode_batch(batch, gd, gp, [per] * n_g))
                res["rdp"]["encode_grouped_16_chunks_ms"] = round(gr, 4)
                res["rdp"]["encode_grouped_16_chunks_hbm_frac"] = round((k + 2) * per * n_g / gr / 1e6 / HBM_PEAK_GBPS, 4)
                gs.gs_batch_destroy(batch)
            log("[bench] rdp: " + json.dumps(res["rdp"]))
            gs.gs_encode(code, data, parity, S)   # put the Reed-Solomon parity back
            torch.cuda.synchronize()

    # ---- CPU oracle on the same bytes (bounded sample), all host cores
    import oracle
    # threads the oracle runs on: the CPUs this process may use, at most 16 (the GPU machine's CPU share
    # for one GPU; its nproc reports the whole machine)
    nthreads = min(len(os.sched_getaffinity(0)) or 1, 16)
    Ss = min(S, args.cpu_sample_mib << 20)
    host_data = [d[:Ss].cpu().numpy() for d in data]
    P = oracle.generator(k, m)
    t0 = time.perf_counter()
    want = oracle.encode(P, host_data, nthreads=nthreads)
    cpu_s = time.perf_counter() - t0
    gs.gs_encode(code, data, parity, S)
    torch.cuda.synchronize()
    same = all(np.array_equal(parity[i][:Ss].cpu().numpy(), want[i]) for i in range(m))
    res["cpu_baseline"] = {"value": round(k * Ss / cpu_s / 1e9, 3), "unit": "GB/s", "cores": nthreads,
                           "host_cpus_online": os.cpu_count(),
                           "host_cpus_this_process_may_use": len(os.sched_getaffinity(0)),
                           "kind": "oracle",
                           "sample": "encode of the first %d MiB of each of the %d shards (%.1f GiB of data), %.1f s"
                                     % (Ss >> 20, k, k * Ss / 2**30, cpu_s),
                           "gpu_parity_matches_oracle_on_sample": bool(same)}
    log("[bench] oracle on %d threads: %.3f GB/s; GPU parity equal on sample: %s" % (nthreads, k * Ss / cpu_s / 1e9, same))
    # the same oracle on one thread, on a sixteenth of that sample
    S1 = max(16, Ss // 16)
    one = [d[:S1] for d in host_data]
    t0 = time.perf_counter()
    oracle.encode(P, one, nthreads=1)
    one_s = time.perf_counter() - t0
    res["cpu_baseline"]["one_thread_GBps"] = round(k * S1 / one_s / 1e9, 3)
    log("[bench] oracle on 1 thread: %.3f GB/s (%.1f s)" % (k * S1 / one_s / 1e9, one_s))
    del host_data, want, one

    # ---- streaming decode-step checkpoint (paged, k=4, m=1), latency over 1000 steps
    res["decode_step"] = decode_steps(torch, gs, inputs, log, native["decode"] if native else None)
    # ---- many small chunks: one launch per chunk, a stream per chunk, or one grouped launch
    res["many_chunks"] = {"through_python_binding": many_chunks(torch, gs, log),
                          "from_c": native["many"] if native else None}
    # ---- per-chunk latency breakdown against chunk size (the shape of the paper's kernel microbenchmark)
    res["chunk_sweep"] = chunk_sweep(torch, gs, inputs, log)
    return res


def chunk_sweep(torch, gs, inputs, log):
    """70B-shaped KV, batch 16, 8:2 code: for each chunk size the time of the
    encode kernel, of the reconstruct kernel (two shards lost) and of the
    parity D2H of one chunk; events on the launch stream, median of 7."""
    k, m, batch = 8, 2, 16
    per_tok = inputs.bytes_per_token(80)
    code = gs.gs_make_code(k, m)
    rows = []
    max_S = 4096 * batch * per_tok // k
    buf = torch.empty((k + m) * max_S, dtype=torch.uint8, device="cuda")
    buf.random_(0, 256)
    host = pinned_slices(torch, [m * max_S])[0]

    def med(fn):
        ts = []
        for _ in range(9):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            b.record()
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b))
        return sorted(ts[2:])[3]

    for tokens in (256, 512, 1024, 2048, 4096):
        S = tokens * batch * per_tok // k
        shards = [buf[r * max_S: r * max_S + S] for r in range(k + m)]
        enc = med(lambda: gs.gs_encode(code, shards[:k], shards[k:], S))
        rec = med(lambda: gs.gs_reconstruct(code, shards, [1, 3], S))
        d2h = med(lambda: [host[i * S:(i + 1) * S].copy_(shards[k + i], non_blocking=True) for i in range(m)])
        rows.append({"chunk_tokens": tokens, "data_bytes": k * S, "encode_ms": round(enc, 4),
                     "reconstruct_ms": round(rec, 4), "parity_d2h_ms": round(d2h, 3),
                     "encode_frac_of_d2h": round(enc / d2h, 4)})
    log("[bench] chunk sweep: " + json.dumps(rows))
    return rows


def rdp_forms(torch, gs, inputs, log, calibrate=False):
    """The XOR-only RDP code in all of its forms, k = 4, 8, 16 (p = 5, 11, 17), shards of about 1 GiB in
    cells of 32 KiB: contiguous encode, rebuild of two data shards and of one, the paged encode behind an
    identity table and behind a seeded random permutation of the pool's pages (a cell = a page), and the
    grouped launch over 16 chunks.  Events around 10 launches each; fractions are algorithmic bytes
    (shards read + shards written) over the 8 TB/s HBM peak."""
    dev = "cuda:0"
    cell = 32768
    out = []
    device_arena(torch, 18 * ((1 << 30) + (2 << 20)))   # the widest code's shards: nothing is freed between the three
    for k in (4, 8, 16):
        code = gs.gs_make_rdp_code(k, cell)
        p = gs.gs_rdp_prime(code)
        stripe = (p - 1) * cell
        S = (1 << 30) // (16 * stripe) * (16 * stripe)      # 16 chunks of whole stripes
        gap = 2 << 20                                       # keeps shards off power-of-two distances
        arena = device_arena(torch, (k + 2) * (S + gap))
        inputs.kv_bytes_device(inputs.config_seed("llama8b_prefill") + 40 + k, k * (S + gap), "bf16", 1.0, dev,
                               out=arena[:k * (S + gap)])
        sh = [arena[j * (S + gap): j * (S + gap) + S] for j in range(k + 2)]
        if calibrate and k == 4:
            sh[k].copy_(sh[0])      # a plain copy of known size (counter calibration under rocprofv3 --pmc)
            torch.cuda.synchronize()
            log("[bench] calibration copy: %d bytes read, %d bytes written" % (S, S))

        def ms_of(fn, n=10):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(n):
                fn()
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) / n

        row = {"k": k, "prime": p, "cell_bytes": cell, "shard_bytes": S}

        def put(name, ms, shards_moved):
            row[name] = {"ms": round(ms, 4), "frac": round(shards_moved * S / ms / 1e6 / HBM_PEAK_GBPS, 4)}

        put("encode", ms_of(lambda: gs.gs_encode(code, sh[:k], sh[k:], S)), k + 2)
        two = [0, k - 1] if k > 1 else [0, k]
        put("reconstruct_two_data_shards", ms_of(lambda: gs.gs_reconstruct(code, sh, two, S)), k + 2)
        put("reconstruct_one_data_shard", ms_of(lambda: gs.gs_reconstruct(code, sh, [1], S)), k + 1)
        gs.gs_encode(code, sh[:k], sh[k:], S)
        # paged: one plane over the data part of the arena, a page = a cell
        lo = arena.data_ptr()
        pps, ppp = S // cell, k * (S + gap) // cell
        one_plane = torch.tensor([lo], dtype=torch.int64, device=dev)
        ident = torch.stack([torch.arange(pps, dtype=torch.int32, device=dev) + j * ((S + gap) // cell)
                             for j in range(k)]).contiguous()
        put("encode_paged_identity_table",
            ms_of(lambda: gs.gs_encode_paged(code, one_plane, 1, cell, ppp, ident, pps, sh[k:])), k + 2)
        perm = torch.from_numpy(inputs.block_table_np(inputs.config_seed("llama8b_prefill") + k, k, pps, ppp)).to(dev)
        put("encode_paged_random_table",
            ms_of(lambda: gs.gs_encode_paged(code, one_plane, 1, cell, ppp, perm, pps, sh[k:])), k + 2)
        n_g, per = 16, S // 16
        batch = gs.gs_batch_create(code, n_g)
        addr = np.array([[t.data_ptr() + c * per for t in sh] for c in range(n_g)], dtype=np.uint64)
        a_in, a_out = np.ascontiguousarray(addr[:, :k]), np.ascontiguousarray(addr[:, k:])
        sizes = np.full(n_g, per, dtype=np.uint64)
        put("encode_grouped_16_chunks", ms_of(lambda: gs.gs_encode_batch(batch, a_in, a_out, sizes)), k + 2)
        gs.gs_batch_destroy(batch)
        out.append(row)
    log("[bench] rdp forms: " + json.dumps(out))
    return out


def many_chunks(torch, gs, log):
    """Recovery of many chunks at once (one lost shard of an 8+2 code) and
    per-request encodes (4+1), three ways; host-timed enqueue -> sync, median."""
    def wall(fn, iters=15, warm=3):
        for _ in range(warm):
            fn()
        ts = []
        for _ in range(iters):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            ts.append(time.perf_counter() - t0)
        return sorted(ts)[len(ts) // 2] * 1e3

    out = []
    for k, m, er, S, n in [(8, 2, [3], 2 << 20, 64), (8, 2, [3, 6], 256 << 10, 256), (4, 1, None, 512 << 10, 64)]:
        code = gs.gs_make_code(k, m)
        big = torch.empty(n * (k + m) * S, dtype=torch.uint8, device="cuda")
        big.random_(0, 256)
        shards = [[big[(c * (k + m) + r) * S:(c * (k + m) + r + 1) * S] for r in range(k + m)] for c in range(n)]
        sizes = [S] * n
        batch = gs.gs_batch_create(code, n)
        pool = gs.gs_pool_create(16)
        if er is None:
            data, par = [row[:k] for row in shards], [row[k:] for row in shards]
            forms = {"one_launch_per_chunk_ms": lambda: [gs.gs_encode(code, data[c], par[c], S) for c in range(n)],
                     "stream_pool_16_ms": lambda: gs.gs_encode_streams(code, pool, data, par, sizes),
                     "grouped_launch_ms": lambda: gs.gs_encode_batch(batch, data, par, sizes)}
            traffic = (k + m) * S * n
        else:
            forms = {"one_launch_per_chunk_ms": lambda: [gs.gs_reconstruct(code, shards[c], er, S) for c in range(n)],
                     "stream_pool_16_ms": lambda: gs.gs_reconstruct_streams(code, pool, shards, er, sizes),
                     "grouped_launch_ms": lambda: gs.gs_reconstruct_batch(batch, shards, er, sizes)}
            traffic = (k + len(er)) * S * n
        # the grouped call once more with the addresses kept in numpy arrays (what an engine that tracks
        # its buffers by address would hand over): no per-pointer work in the interpreter
        addr = np.array([[t.data_ptr() for t in row_] for row_ in shards], dtype=np.uint64)
        sizes_np = np.array(sizes, dtype=np.uint64)
        if er is None:
            a_in, a_out = np.ascontiguousarray(addr[:, :k]), np.ascontiguousarray(addr[:, k:])
            forms["grouped_launch_address_arrays_ms"] = lambda: gs.gs_encode_batch(batch, a_in, a_out, sizes_np)
        else:
            forms["grouped_launch_address_arrays_ms"] = lambda: gs.gs_reconstruct_batch(batch, addr, er, sizes_np)
        row = {"op": "encode" if er is None else "reconstruct", "k": k, "m": m, "erased": er,
               "chunks": n, "shard_bytes": S}
        for name, fn in forms.items():
            row[name] = round(wall(fn), 4)
        row["grouped_launch_traffic_GBps"] = round(traffic / row["grouped_launch_ms"] / 1e6, 1)
        out.append(row)
        gs.gs_batch_destroy(batch)
        gs.gs_pool_destroy(pool)
        del big, shards
    log("[bench] many chunks: " + json.dumps(out))
    return out


def decode_steps(torch, gs, inputs, log, native=None):
    c = inputs.CONFIGS["decode_paged"]
    k, m, steps = c["k"], c["m"], c["steps"]
    n_planes = c["layers"] * 2
    block_tokens, slot_bytes = c["block_tokens"], 8 * 128 * 2
    seqs_per_shard = c["batch"] // k
    blocks_per_seq = (steps + 20 + block_tokens - 1) // block_tokens  # every step writes a fresh token slot
    n_blocks = c["batch"] * blocks_per_seq
    pages_per_plane = n_blocks * block_tokens
    dev = "cuda:0"
    pool = inputs.kv_bytes_device(inputs.config_seed("decode_paged"), n_planes * pages_per_plane * slot_bytes,
                                  c["dtype"], c["sigma"], dev)
    plane_bytes = pages_per_plane * slot_bytes
    base = torch.tensor([pool.data_ptr() + p * plane_bytes for p in range(n_planes)], dtype=torch.int64, device=dev)
    rng = np.random.default_rng(inputs.config_seed("decode_paged") + inputs.TABLE_SEED_OFFSET)
    # sequence q owns blocks_per_seq blocks scattered over the pool; at step s it writes slot
    # s mod 16 of its block s div 16, so no page is touched twice during the run
    blocks = rng.permutation(n_blocks).reshape(blocks_per_seq, k, seqs_per_shard)
    tables = torch.from_numpy(np.stack([(blocks[s // block_tokens] * block_tokens + (s % block_tokens)).astype(np.int32)
                                        for s in range(steps + 20)])).to(dev)
    table = tables[0].clone()
    out_bytes = n_planes * seqs_per_shard * slot_bytes
    par = [torch.empty(out_bytes, dtype=torch.uint8, device=dev) for _ in range(m)]
    host = pinned_slices(torch, [out_bytes] * m)
    code = gs.gs_make_code(k, m)
    torch.cuda.synchronize()

    def run(fn):
        lat = []
        for s in range(steps + 20):
            table.copy_(tables[s])  # the engine moves every sequence to its next slot
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            lat.append((time.perf_counter() - t0) * 1e6)
        lat = lat[20:]
        return {"p50_us": round(pctl(lat, 0.5), 1), "p99_us": round(pctl(lat, 0.99), 1),
                "mean_us": round(sum(lat) / len(lat), 1)}

    res = {"new_kv_bytes_per_step": k * out_bytes, "steps": steps}
    res["eager_encode_only"] = run(lambda: gs.gs_encode_paged(code, base, n_planes, slot_bytes, pages_per_plane,
                                                              table, seqs_per_shard, par))

    def eager_d2h():
        gs.gs_encode_paged(code, base, n_planes, slot_bytes, pages_per_plane, table, seqs_per_shard, par)
        for i in range(m):
            host[i].copy_(par[i], non_blocking=True)
    res["eager_encode_d2h"] = run(eager_d2h)
    # the kernel writes its parity straight into pinned host memory: no staging buffer, no copy
    res["eager_encode_into_pinned_host"] = run(lambda: gs.gs_encode_paged(
        code, base, n_planes, slot_bytes, pages_per_plane, table, seqs_per_shard, host))
    g0 = gs.gs_step_graph_create(code, base, n_planes, slot_bytes, pages_per_plane, table, seqs_per_shard, par, None)
    res["graph_encode_only"] = run(lambda: gs.gs_step_graph_launch(g0))
    g1 = gs.gs_step_graph_create(code, base, n_planes, slot_bytes, pages_per_plane, table, seqs_per_shard, par, host)
    res["graph_encode_d2h"] = run(lambda: gs.gs_step_graph_launch(g1))
    gs.gs_step_graph_destroy(g0)
    gs.gs_step_graph_destroy(g1)
    if native is not None:
        res["native"] = native
    log("[bench] decode step: " + json.dumps(res))
    return res


if __name__ == "__main__":
    sys.exit(main())
