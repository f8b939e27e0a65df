"""Writes tests/golden/oracle_small_cases.json: outputs of the fp64 oracle on small seeded inputs.

The paper prints no worked numeric example for any stage, so no fixture here is a printed value.  These numbers are
the oracle's own (this script calls nothing but `oracle/` and the seeded input generators) and serve one purpose: a
later edit of the oracle that changes its arithmetic shows up as a diff against them.  The pins that tie the oracle
to the paper and to the mathematics are the tests/test_oracle_*.py files, not this file.

Run from the repository root:  python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import pafu_oracle as orc  # noqa: E402
from paper_2601_21896_amd import workloads as wl  # noqa: E402


def cases():
    cfg = wl.scaled(wl.C0, frame_tokens=8, cache_frames=3, chunk_frames=1, k=10)     # n = 24, Lc = 8
    d = wl.make_layer_inputs(cfg, bias=True)
    kv = {x: wl.round_to_bf16(d[x]) for x in ("K_cache", "V_cache", "Q", "K_chunk", "V_chunk")}
    step = orc.step_single(d["X_cache"], d["X_chunk"], d["W1"], d["b1"], d["W2"], d["b2"], kv["K_cache"], kv["V_cache"],
                           kv["Q"], kv["K_chunk"], kv["V_chunk"], k=10, block_len=4)
    pinned = orc.select_topk(step["scores"][:24].astype(np.float32), 10, n_pinned=3)
    sse = orc.sse_score(kv["Q"], kv["K_chunk"], block_len=4)
    return {
        "config": "C0 scaled: 2 heads x 64, 24 cached + 8 chunk tokens, k = 10, L_B = 4, seed %d" % d["seed"],
        "scores": step["scores"].tolist(),
        "ids": step["ids"].tolist(),
        "ids_with_3_pinned": pinned.tolist(),
        "O_first_row_head0_first8": step["O"][0, 0, :8].tolist(),
        "O_sum": float(step["O"].sum()),
        "sse_of_chunk": sse.tolist(),
    }


if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_small_cases.json")
    with open(out, "w") as f:
        json.dump(cases(), f, indent=1)
    print("wrote", out)
