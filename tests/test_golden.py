"""The oracle still reproduces the stored small cases (tests/golden/, written by make_golden.py from the oracle
alone; the paper prints no worked example, so these are regression values, not paper values)."""
import importlib.util
import json
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))


def test_oracle_reproduces_golden_cases():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    now = mod.cases()
    with open(os.path.join(HERE, "golden", "oracle_small_cases.json")) as f:
        stored = json.load(f)
    assert now["ids"] == stored["ids"] and now["ids_with_3_pinned"] == stored["ids_with_3_pinned"]
    for key in ("scores", "O_first_row_head0_first8", "sse_of_chunk"):
        assert np.allclose(now[key], stored[key], rtol=1e-12, atol=1e-15), key
    assert abs(now["O_sum"] - stored["O_sum"]) < 1e-10
