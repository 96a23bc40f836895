"""The oracle still reproduces the record it wrote of itself (guards against silent edits)."""
import importlib.util
import json
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))


def test_oracle_matches_its_stored_record():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    now = mod.compute()
    with open(os.path.join(HERE, "golden", "tiny_stage.json")) as f:
        ref = json.load(f)
    assert now["order"] == ref["order"]
    for key in ("Y_sum", "dX_abs_sum", "Y0_first4"):
        assert np.allclose(now[key], ref[key], rtol=1e-12, atol=1e-12), key
    for n, v in ref["G_l2"].items():
        assert abs(now["G_l2"][n] - v) <= 1e-12 * max(1.0, abs(v)), n
