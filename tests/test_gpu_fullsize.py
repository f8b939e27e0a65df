"""Parity at the benchmark's full sizes, in the launch configuration bench.py times (pafu_step, SINGLE mode).

Scores, indices and the compacted cache are compared in full (the oracle does these in seconds);
attention on sampled query rows the oracle computes one by one: every 37th row plus the first and last
row of every frame block.  Teacher-forced selection as in the other step tests."""
import numpy as np
import pytest
import torch

from oracle import pafu_oracle as orc
from paper_2601_21896_amd import binding as B
from paper_2601_21896_amd import workloads as wl
from tests.gpu_util import ATTN_MAX_ABS, ATTN_REL_FRO, DEV, SCORE_MAX_ABS, attn_errors, dev, host

pytestmark = pytest.mark.gpu


def _sample_rows(cfg):
    rows = set(range(0, cfg.Lc, 37))
    for f in range(cfg.chunk_frames):
        rows.add(f * cfg.frame_tokens)
        rows.add((f + 1) * cfg.frame_tokens - 1)
    return np.array(sorted(rows))


def _run_full(cfg, L_B, score_rows=None, structure="uniform"):
    d = wl.make_layer_inputs(cfg, structure=structure)
    n, Lc, N, D, k = cfg.n, cfg.Lc, cfg.N, cfg.D, cfg.k
    X = dev(np.concatenate([d["X_cache"], d["X_chunk"]]), "bf16")
    scores = torch.empty(n + Lc, device=DEV)
    ids = torch.empty(k, dtype=torch.int32, device=DEV)
    K_out = torch.empty(k, N, D, device=DEV, dtype=torch.bfloat16)
    V_out = torch.empty_like(K_out)
    SL_out = torch.empty(k, device=DEV)
    O = torch.empty(Lc, N, D, device=DEV, dtype=torch.bfloat16)
    args = B.make_step_args(B.PAFU_MODE_SINGLE, N, D, n, Lc, k, L_B, X[:n], X[n:], dev(d["W1"], "bf16"), None,
                            dev(d["W2"]), None, dev(d["K_cache"], "bf16"), dev(d["V_cache"], "bf16"), None,
                            dev(d["Q"], "bf16"), dev(d["K_chunk"], "bf16"), dev(d["V_chunk"], "bf16"), scores, ids,
                            K_out, V_out, SL_out, O)
    B.pafu_step(args)
    torch.cuda.synchronize()
    got_s = host(scores)
    Xall = np.concatenate([d["X_cache"], d["X_chunk"]])
    srows = np.arange(n + Lc) if score_rows is None else score_rows
    want_s = orc.smlp_score(Xall[srows], d["W1"], None, d["W2"], None)
    assert np.abs(got_s[srows] - want_s).max() < SCORE_MAX_ABS
    assert np.abs(want_s).max() > 0.05                     # the head's output is not trivially small
    want_ids = orc.select_topk(got_s[:n], k)               # teacher-forced on the device's fp32 scores
    assert np.array_equal(host(ids), want_ids)
    Kk, Vk, SLk = orc.compact_kv(d["K_cache"], d["V_cache"], got_s[:n], want_ids)
    assert np.array_equal(host(K_out), Kk) and np.array_equal(host(V_out), Vk) and np.array_equal(host(SL_out), SLk)
    # the salient tokens (+2 sigma features) are what the structured scores pick up
    rows = _sample_rows(cfg)
    want_O = orc.chunk_attention(d["Q"], Kk, Vk, d["K_chunk"], d["V_chunk"], block_len=L_B, rows=rows)
    max_abs, rel = attn_errors(host(O)[rows], want_O)
    assert max_abs < ATTN_MAX_ABS and rel < ATTN_REL_FRO, (max_abs, rel)
    return d, got_s, want_ids


def test_c1_full_step_paper_block_length():
    _run_full(wl.C1, wl.C1.Lc)


def test_c1_full_step_frame_blocks_and_coherent_salience():
    # L_B = one frame: the block mask is live in the last 3 x 1560 keys
    _run_full(wl.C1, wl.C1.frame_tokens, structure="coherent")


def test_c4_full_step_sampled():
    cfg = wl.C4
    srows = np.arange(0, cfg.n + cfg.Lc, 16)
    _run_full(cfg, cfg.Lc, score_rows=srows)
