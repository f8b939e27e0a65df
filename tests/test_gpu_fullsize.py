"""Parity at the benchmark's full sizes, in the launch configurations bench.py times.

Single layers (Wan-1.3B and Wan-14B shapes) go through pafu_step in SINGLE mode; the 30-layer step through
pafu_step_layers and pafu_step_layers_shared; the 60-chunk rollout and its budget sweep through pafu_step in
ROLLOUT mode with the oracle's rollout run beside it.

Scores, indices and the compacted cache are compared in full (the oracle does these in seconds).  Attention is
compared on every query row at the Wan-1.3B single layer; where that would take minutes (30 layers, 60 chunks, the
Wan-14B layer) on sampled query rows the oracle computes one by one: every 37th row plus the first and last row of
every frame block.  Teacher-forced selection as in the other step tests: the device's own fp32 scores are fed to the
oracle's selection, so indices and cache must match bit for bit."""
import numpy as np
import pytest
import torch

from oracle import pafu_oracle as orc
from paper_2601_21896_amd import binding as B
from paper_2601_21896_amd import workloads as wl
from tests.gpu_util import ATTN_MAX_ABS, ATTN_REL_FRO, DEV, SCORE_MAX_ABS, attn_errors, dev, host, step_workspace

pytestmark = pytest.mark.gpu


def _sample_rows(cfg):
    rows = set(range(0, cfg.Lc, 37))
    for f in range(cfg.chunk_frames):
        rows.add(f * cfg.frame_tokens)
        rows.add((f + 1) * cfg.frame_tokens - 1)
    return np.array(sorted(rows))


def _run_full(cfg, L_B, score_rows=None, structure="uniform", all_rows=False, workspace=True):
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
    if workspace:                                          # with it the attention launch cuts its work into equal runs
        step_workspace(args)
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
    rows = np.arange(Lc) if all_rows else _sample_rows(cfg)
    want_O = orc.chunk_attention(d["Q"], Kk, Vk, d["K_chunk"], d["V_chunk"], block_len=L_B, rows=rows)
    max_abs, rel = attn_errors(host(O)[rows], want_O)
    assert max_abs < ATTN_MAX_ABS and rel < ATTN_REL_FRO, (max_abs, rel)
    return d, got_s, want_ids


def test_c1_full_step_paper_block_length():
    _run_full(wl.C1, wl.C1.Lc, all_rows=True)


def test_c1_full_step_frame_blocks_and_coherent_salience():
    # L_B = one frame: the block mask is live in the last 3 x 1560 keys
    _run_full(wl.C1, wl.C1.frame_tokens, structure="coherent", all_rows=True)


def test_c1_full_step_without_workspace():
    # no workspace: one workgroup per (head, query tile), nothing merged
    _run_full(wl.C1, wl.C1.Lc, workspace=False)


def test_c1_one_frame_chunk_takes_the_equal_run_split():
    # a one-frame chunk (1560 queries = 84 items on 256 compute units) over the full cache: with the workspace the
    # attention launch cuts the key axis into equal runs and merges partial results
    _run_full(wl.scaled(wl.C1, chunk_frames=1), wl.C1.frame_tokens, all_rows=True)


def test_c4_full_step_sampled():
    cfg = wl.C4
    srows = np.arange(0, cfg.n + cfg.Lc, 16)
    _run_full(cfg, cfg.Lc, score_rows=srows)


# ------------------------------------------------------------------ 30 layers at the Wan-1.3B layer shapes
C2_SEED = wl.BASE_SEED + 2


class _Layer:
    """One layer of the 30-layer step: seeded host inputs, their device copies, fresh output buffers."""

    def __init__(self, cfg, seed):
        self.cfg = cfg
        self.d = d = wl.make_layer_inputs(cfg, seed=seed)
        n = cfg.n
        self.X = dev(np.concatenate([d["X_cache"], d["X_chunk"]]), "bf16")
        self.W1, self.W2 = dev(d["W1"], "bf16"), dev(d["W2"])
        self.K, self.V = dev(d["K_cache"], "bf16"), dev(d["V_cache"], "bf16")
        self.Q, self.Kn, self.Vn = dev(d["Q"], "bf16"), dev(d["K_chunk"], "bf16"), dev(d["V_chunk"], "bf16")
        assert self.X.shape[0] == n + cfg.Lc

    def outputs(self):
        cfg = self.cfg
        self.scores = torch.full((cfg.n + cfg.Lc,), float("nan"), device=DEV)
        self.ids = torch.full((cfg.k,), -1, dtype=torch.int32, device=DEV)
        self.K_out = torch.zeros(cfg.k, cfg.N, cfg.D, device=DEV, dtype=torch.bfloat16)
        self.V_out = torch.zeros_like(self.K_out)
        self.SL_out = torch.zeros(cfg.k, device=DEV)
        self.O = torch.zeros(cfg.Lc, cfg.N, cfg.D, device=DEV, dtype=torch.bfloat16)

    def args(self, L_B, workspace=None):
        cfg, n = self.cfg, self.cfg.n
        return B.make_step_args(B.PAFU_MODE_SINGLE, cfg.N, cfg.D, n, cfg.Lc, cfg.k, L_B, self.X[:n], self.X[n:],
                                self.W1, None, self.W2, None, self.K, self.V, None, self.Q, self.Kn, self.Vn,
                                self.scores, self.ids, self.K_out, self.V_out, self.SL_out, self.O,
                                workspace=workspace)


@pytest.fixture(scope="module")
def c2_layers():
    layers = [_Layer(wl.C1, C2_SEED + 1000 * l) for l in range(wl.C2_LAYERS)]
    yield layers
    layers.clear()
    torch.cuda.empty_cache()


def test_c2_thirty_layers_independent_indices(c2_layers):
    cfg = wl.C1
    n, k, L_B = cfg.n, cfg.k, cfg.Lc
    rows = _sample_rows(cfg)
    for L in c2_layers:
        L.outputs()
    ws = torch.empty(B.pafu_attention_workspace_bytes(cfg.Lc, cfg.N, cfg.D), dtype=torch.uint8, device=DEV)
    B.pafu_step_layers([L.args(L_B, ws) for L in c2_layers])      # the layers may share one workspace
    torch.cuda.synchronize()
    seen = set()
    for l, L in enumerate(c2_layers):
        d = L.d
        got_s = host(L.scores)
        want_s = orc.smlp_score(np.concatenate([d["X_cache"], d["X_chunk"]]), d["W1"], None, d["W2"], None)
        assert np.abs(got_s - want_s).max() < SCORE_MAX_ABS, l
        want_ids = orc.select_topk(got_s[:n], k)
        assert np.array_equal(host(L.ids), want_ids), l
        Kk, Vk, SLk = orc.compact_kv(d["K_cache"], d["V_cache"], got_s[:n], want_ids)
        assert np.array_equal(host(L.K_out), Kk) and np.array_equal(host(L.V_out), Vk), l
        assert np.array_equal(host(L.SL_out), SLk), l
        want_O = orc.chunk_attention(d["Q"], Kk, Vk, d["K_chunk"], d["V_chunk"], block_len=L_B, rows=rows)
        max_abs, rel = attn_errors(host(L.O)[rows], want_O)
        assert max_abs < ATTN_MAX_ABS and rel < ATTN_REL_FRO, (l, max_abs, rel)
        seen.add(want_ids[:64].tobytes())
    assert len(seen) == len(c2_layers)          # every layer made its own selection


def test_c2_thirty_layers_shared_indices(c2_layers):
    cfg = wl.C1
    n, k, L_B = cfg.n, cfg.k, cfg.Lc
    rows = _sample_rows(cfg)
    idx = len(c2_layers) - 1                   # the head reads the final layer (Sec. 3.3)
    for L in c2_layers:
        L.outputs()
    ws = torch.empty(B.pafu_attention_workspace_bytes(cfg.Lc, cfg.N, cfg.D), dtype=torch.uint8, device=DEV)
    # only the index layer brings a workspace: the others borrow it
    B.pafu_step_layers_shared([L.args(L_B, ws if l == idx else None) for l, L in enumerate(c2_layers)], idx)
    torch.cuda.synchronize()
    d = c2_layers[idx].d
    got_s = host(c2_layers[idx].scores)
    want_s = orc.smlp_score(np.concatenate([d["X_cache"], d["X_chunk"]]), d["W1"], None, d["W2"], None)
    assert np.abs(got_s - want_s).max() < SCORE_MAX_ABS
    want_ids = orc.select_topk(got_s[:n], k)
    assert np.array_equal(host(c2_layers[idx].ids), want_ids)
    assert np.array_equal(host(c2_layers[idx].SL_out), got_s[:n][want_ids])
    for l, L in enumerate(c2_layers):
        Kk, Vk, _ = orc.compact_kv(L.d["K_cache"], L.d["V_cache"], got_s[:n], want_ids)
        assert np.array_equal(host(L.K_out), Kk) and np.array_equal(host(L.V_out), Vk), l
        want_O = orc.chunk_attention(L.d["Q"], Kk, Vk, L.d["K_chunk"], L.d["V_chunk"], block_len=L_B, rows=rows)
        max_abs, rel = attn_errors(host(L.O)[rows], want_O)
        assert max_abs < ATTN_MAX_ABS and rel < ATTN_REL_FRO, (l, max_abs, rel)
        if l != idx:                            # only the index layer writes scores and indices
            assert torch.all(L.ids == -1) and torch.all(torch.isnan(L.scores))


# ------------------------------------------------------------------ 60-chunk rollout at the Wan-1.3B layer shapes
def _rollout_full(k, n_chunks):
    """pafu_step ROLLOUT beside the oracle's rollout (teacher-forced on the chunk scores): indices, K, V and the
    score list bit-exact after every step, attention on the sampled rows."""
    cfg = wl.C1
    N, D, Lc, L_B = cfg.N, cfg.D, cfg.Lc, cfg.Lc
    rows = _sample_rows(cfg)
    W1, b1, W2, b2 = wl.make_rollout_weights(cfg)
    dW1, dW2 = dev(W1, "bf16"), dev(W2)
    cap = k + Lc
    slabs = [dict(K=torch.zeros(cap, N, D, device=DEV, dtype=torch.bfloat16),
                  V=torch.zeros(cap, N, D, device=DEV, dtype=torch.bfloat16),
                  SL=torch.zeros(cap, device=DEV)) for _ in range(2)]
    st = orc.RolloutState(N, D, np.float32)
    ids = torch.empty(k, dtype=torch.int32, device=DEV)
    O = torch.empty(Lc, N, D, device=DEV, dtype=torch.bfloat16)
    ws = torch.empty(B.pafu_attention_workspace_bytes(Lc, N, D), dtype=torch.uint8, device=DEV)
    n, cur, sizes, evictions = 0, 0, [], 0
    for t in range(n_chunks):
        c = wl.make_chunk_inputs(cfg, t)
        src, dst = slabs[cur], slabs[1 - cur]
        n_kept = min(k, n)
        args = B.make_step_args(B.PAFU_MODE_ROLLOUT, N, D, n, Lc, k, L_B, None, dev(c["X_chunk"], "bf16"), dW1, None,
                                dW2, None, src["K"], src["V"], src["SL"], dev(c["Q"], "bf16"),
                                dev(c["K_chunk"], "bf16"), dev(c["V_chunk"], "bf16"), None, ids, dst["K"], dst["V"],
                                dst["SL"], O, workspace=ws)
        B.pafu_step(args)
        torch.cuda.synchronize()
        s_chunk = host(dst["SL"][n_kept:n_kept + Lc])
        out = orc.rollout_step(st, c["X_chunk"], W1, b1, W2, b2, c["Q"], c["K_chunk"], c["V_chunk"], k, L_B,
                               forced_chunk_scores_f32=s_chunk, rows=rows)
        assert np.abs(s_chunk - out["s_chunk"]).max() < SCORE_MAX_ABS, t
        assert np.array_equal(host(ids)[:n_kept], out["ids"]), t
        evictions += int(n > k)
        n = n_kept + Lc
        assert n == st.n
        assert np.array_equal(host(dst["K"][:n]), st.K) and np.array_equal(host(dst["V"][:n]), st.V), t
        assert np.array_equal(host(dst["SL"][:n]), st.SL), t
        max_abs, rel = attn_errors(host(O)[rows], out["O"])
        assert max_abs < ATTN_MAX_ABS and rel < ATTN_REL_FRO, (t, max_abs, rel)
        sizes.append(n)
        cur = 1 - cur
    return sizes, evictions


def test_c3_rollout_sixty_chunks():
    sizes, evictions = _rollout_full(wl.C3_K, wl.C3_CHUNKS)
    assert sizes[:5] == [4680, 9360, 14040, 17160, 17160] and sizes[-1] == wl.C3_K + wl.C1.Lc
    assert evictions == wl.C3_CHUNKS - 3


@pytest.mark.parametrize("k,n_chunks", [(8190, 8), (16380, 8), (32760, 11)])
def test_c3_rollout_budget_sweep(k, n_chunks):
    sizes, evictions = _rollout_full(k, n_chunks)
    assert sizes[-1] == k + wl.C1.Lc and evictions >= 2
