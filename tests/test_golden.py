"""The oracle against its frozen outputs under tests/golden/ (written by tests/golden/make_golden.py from
the oracle alone): a change to the oracle's arithmetic shows up here even if every relative pin still
holds.  The paper prints no worked example for this path, so these are not the paper's numbers."""
import hashlib
import importlib.util
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))


def load_maker():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_oracle_reproduces_the_frozen_tiny_decode_step_and_merge():
    ctx, out, merged = load_maker().tiny_case()
    seen = 0
    for line in open(os.path.join(HERE, "golden", "c1_decode_and_merge.txt")):
        if line.startswith("#"):
            continue
        key, *vals = line.split()
        if key == "ctx_lens":
            assert [int(v) for v in vals] == [int(c) for c in ctx]
        elif key == "hidden_out":
            i, k, v = int(vals[0]), int(vals[1]), float(vals[2])
            assert abs(out[i, k] - v) <= 1e-12 * max(1.0, abs(v))
            seen += 1
        elif key == "row_rms":
            assert abs(np.sqrt((out[int(vals[0])] ** 2).mean()) - float(vals[1])) <= 1e-12
        elif key == "hidden_out_sum":
            assert abs(out.sum() - float(vals[0])) <= 1e-9
        elif key == "hidden_out_abs_sum":
            assert abs(np.abs(out).sum() - float(vals[0])) <= 1e-9
        elif key == "merged_pool_sha256":
            assert hashlib.sha256(np.ascontiguousarray(merged).tobytes()).hexdigest() == vals[0]
    assert seen == out.shape[0] * len(range(0, out.shape[1], 37))
