"""The stored fixtures under tests/golden/ are the oracle's output (written by
tests/golden/make_golden.py).  They must still be what the oracle produces,
and the parts with a plain definition must also satisfy that definition."""
import hashlib
import os

import numpy as np

import oracle
from paper_2605_00831_amd import inputs
from tests import _gfref
from tests.golden import make_golden

HERE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def test_generators_file_is_current_and_matches_closed_form():
    with open(os.path.join(HERE, "generators.txt")) as f:
        text = f.read()
    assert text == make_golden.generators()
    cur, rows = None, {}
    for line in text.splitlines():
        if line.startswith("k="):
            k, m = [int(x.split("=")[1]) for x in line.split()]
            cur = (k, m)
            rows[cur] = []
        elif line.startswith("  "):
            rows[cur].append(bytes.fromhex(line.strip()))
    for (k, m), rr in rows.items():
        want = _gfref.cauchy_normalised(k, m)
        assert [bytes(r) for r in want] == rr


def test_tiny_digests_file_is_current_and_parity0_is_xor():
    with open(os.path.join(HERE, "tiny_digests.txt")) as f:
        text = f.read()
    assert text == make_golden.tiny_digests()
    dig = dict(line.split() for line in text.splitlines() if not line.startswith("#"))
    c = inputs.CONFIGS["tiny"]
    buf = inputs.kv_bytes_np(inputs.config_seed("tiny"), inputs.config_total_bytes("tiny"),
                             c["dtype"], c["sigma"])
    data = inputs.split_shards(buf, 4)
    x = np.bitwise_xor.reduce(np.stack(data), axis=0)
    assert hashlib.sha256(x.tobytes()).hexdigest() == dig["parity0"]
    p1 = _gfref.encode_np(_gfref.cauchy_normalised(4, 2), data)[1]
    assert hashlib.sha256(p1.tobytes()).hexdigest() == dig["parity1"]
