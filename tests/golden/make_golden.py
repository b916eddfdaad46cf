"""Writes tests/golden/*.txt.  Calls only the CPU oracle and the seeded input
generators (never the HIP library), so every stored value is the oracle's.

The paper prints no worked example of a code word, a generator matrix or a
field polynomial, so there is no value of the paper's to store; these files
freeze what the pinned oracle produces for the five measured workloads' codes
and for the tiny workload, so that a later change to the oracle shows up as a
diff here.  Run:  python tests/golden/make_golden.py
"""
import hashlib
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2605_00831_amd import inputs  # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))


def generators():
    lines = ["# parity block P (m x k, hex, one row per line) of the canonical code",
             "# source: oracle.generator (Vandermonde route, normalised); Section 2 / 4.1 fix only k:m"]
    for k, m in [(4, 2), (4, 1), (8, 2), (8, 3), (3, 2), (5, 3), (10, 4)]:
        lines.append("k=%d m=%d" % (k, m))
        for row in oracle.generator(k, m):
            lines.append("  " + bytes(row).hex())
    return "\n".join(lines) + "\n"


def tiny_digests():
    c = inputs.CONFIGS["tiny"]
    total = inputs.config_total_bytes("tiny")
    buf = inputs.kv_bytes_np(inputs.config_seed("tiny"), total, c["dtype"], c["sigma"])
    data = [np.ascontiguousarray(s) for s in inputs.split_shards(buf, c["k"])]
    par = oracle.encode(oracle.generator(c["k"], c["m"]), data, nthreads=8)
    lines = ["# sha256 of each shard of the tiny workload (fp16 N(0,1), 8 MiB, k=4, m=2)",
             "# source: oracle.encode on inputs.kv_bytes_np(seed 0x67530000)"]
    for j, d in enumerate(data):
        lines.append("data%d %s" % (j, hashlib.sha256(d.tobytes()).hexdigest()))
    for i, p in enumerate(par):
        lines.append("parity%d %s" % (i, hashlib.sha256(p.tobytes()).hexdigest()))
    return "\n".join(lines) + "\n"


if __name__ == "__main__":
    with open(os.path.join(HERE, "generators.txt"), "w") as f:
        f.write(generators())
    with open(os.path.join(HERE, "tiny_digests.txt"), "w") as f:
        f.write(tiny_digests())
    print("wrote generators.txt, tiny_digests.txt")
