"""Pins for the oracle's chunk attention (Sec. 3.2 softmax definition and block
boundaries; App. A block length) and for the step / rollout composition (Alg. 2)."""
import math

import numpy as np
import pytest
import torch

from oracle.pafu_oracle import (RolloutState, chunk_attention, compact_kv, rollout_step,
                                select_topk, smlp_score, step_single)


def _rand(rng, n, Lc, N, D):
    Q = rng.standard_normal((Lc, N, D))
    Kc = rng.standard_normal((n, N, D))
    Vc = rng.standard_normal((n, N, D))
    Kn = rng.standard_normal((Lc, N, D))
    Vn = rng.standard_normal((Lc, N, D))
    return Q, Kc, Vc, Kn, Vn


def _loops(Q, Kc, Vc, Kn, Vn, L_B):
    Lq, N, D = Q.shape
    n, Lc = Kc.shape[0], Kn.shape[0]
    O = np.zeros((Lq, N, D))
    for h in range(N):
        for i in range(Lq):
            keys, vals = [], []
            for j in range(n):
                keys.append(Kc[j, h]); vals.append(Vc[j, h])
            for j in range(Lc):
                if j // L_B <= i // L_B:
                    keys.append(Kn[j, h]); vals.append(Vn[j, h])
            z = [sum(Q[i, h, d] * kk[d] for d in range(D)) / math.sqrt(D) for kk in keys]
            m = max(z)
            e = [math.exp(v - m) for v in z]
            tot = sum(e)
            for d in range(D):
                O[i, h, d] = sum(e[j] * vals[j][d] for j in range(len(e))) / tot
    return O


@pytest.mark.parametrize("n,Lc,L_B", [(5, 6, 2), (0, 4, 1), (3, 7, 3), (4, 4, 100)])
def test_brute_force_loops(n, Lc, L_B):
    rng = np.random.default_rng(n * 10 + Lc)
    args = _rand(rng, n, Lc, 2, 4)
    got = chunk_attention(*args, block_len=L_B)
    assert np.allclose(got, _loops(*args, L_B), rtol=1e-12, atol=1e-13)


def test_full_budget_is_textbook_attention():
    # no mask and all keys kept -> softmax(QK^T/sqrt(D))V over cache+chunk (library SDPA, fp64)
    rng = np.random.default_rng(1)
    n, Lc, N, D = 37, 21, 3, 16
    Q, Kc, Vc, Kn, Vn = _rand(rng, n, Lc, N, D)
    got = chunk_attention(Q, Kc, Vc, Kn, Vn, block_len=Lc)
    K_all = np.concatenate([Kc, Kn]); V_all = np.concatenate([Vc, Vn])
    t = lambda a: torch.from_numpy(a).permute(1, 0, 2)[None]
    want = torch.nn.functional.scaled_dot_product_attention(t(Q), t(K_all), t(V_all))[0].permute(1, 0, 2).numpy()
    assert np.allclose(got, want, rtol=1e-12, atol=1e-13)


def test_block_len_one_is_causal_inside_the_chunk():
    rng = np.random.default_rng(2)
    Lc, N, D = 19, 2, 8
    Q, Kc, Vc, Kn, Vn = _rand(rng, 0, Lc, N, D)
    got = chunk_attention(Q, Kc, Vc, Kn, Vn, block_len=1)
    t = lambda a: torch.from_numpy(a).permute(1, 0, 2)[None]
    want = torch.nn.functional.scaled_dot_product_attention(t(Q), t(Kn), t(Vn), is_causal=True)[0].permute(1, 0, 2).numpy()
    assert np.allclose(got, want, rtol=1e-12, atol=1e-13)


def test_block_mask_matches_explicit_mask_in_library_sdpa():
    rng = np.random.default_rng(3)
    n, Lc, N, D, L_B = 11, 20, 2, 8, 6
    Q, Kc, Vc, Kn, Vn = _rand(rng, n, Lc, N, D)
    got = chunk_attention(Q, Kc, Vc, Kn, Vn, block_len=L_B)
    mask = torch.ones(Lc, n + Lc, dtype=torch.bool)
    for i in range(Lc):
        for j in range(Lc):
            mask[i, n + j] = (j // L_B) <= (i // L_B)
    t = lambda a: torch.from_numpy(a).permute(1, 0, 2)[None]
    want = torch.nn.functional.scaled_dot_product_attention(
        t(Q), t(np.concatenate([Kc, Kn])), t(np.concatenate([Vc, Vn])), attn_mask=mask)[0].permute(1, 0, 2).numpy()
    assert np.allclose(got, want, rtol=1e-12, atol=1e-13)


def test_softmax_rows_sum_to_one_and_mask_zeroes():
    rng = np.random.default_rng(4)
    n, Lc, L_B = 9, 12, 4
    args = _rand(rng, n, Lc, 2, 8)
    _, P = chunk_attention(*args, block_len=L_B, return_P=True)
    assert np.allclose(P.sum(axis=2), 1.0, atol=1e-14)
    for i in range(Lc):
        for j in range(Lc):
            if j // L_B > i // L_B:
                assert np.all(P[:, i, n + j] == 0.0)
            else:
                assert np.all(P[:, i, n + j] > 0.0)
    assert np.all(P[:, :, :n] > 0.0)


def test_order_of_retained_rows_does_not_matter():
    rng = np.random.default_rng(5)
    n, Lc = 15, 6
    Q, Kc, Vc, Kn, Vn = _rand(rng, n, Lc, 2, 8)
    perm = rng.permutation(n)
    a = chunk_attention(Q, Kc, Vc, Kn, Vn, block_len=Lc)
    b = chunk_attention(Q, Kc[perm], Vc[perm], Kn, Vn, block_len=Lc)
    assert np.allclose(a, b, rtol=1e-12, atol=1e-14)
    # with no mask, a key may sit in either segment
    c = chunk_attention(Q, Kc[:10], Vc[:10], np.concatenate([Kc[10:], Kn]), np.concatenate([Vc[10:], Vn]),
                        block_len=10 ** 6)
    assert np.allclose(a, c[:Lc], rtol=1e-12, atol=1e-14)


def test_degenerate_closed_forms():
    rng = np.random.default_rng(6)
    n, Lc, N, D = 7, 5, 2, 8
    Q, Kc, Vc, Kn, Vn = _rand(rng, n, Lc, N, D)
    # one visible key: no cache, L_B=1, query 0 sees only chunk key 0
    o = chunk_attention(Q, Kc[:0], Vc[:0], Kn, Vn, block_len=1)
    assert np.allclose(o[0], Vn[0], atol=1e-15)
    # K = 0 -> uniform weights -> mean of visible V rows
    o = chunk_attention(Q, 0 * Kc, Vc, 0 * Kn, Vn, block_len=2)
    for i in range(Lc):
        vis = np.concatenate([Vc, Vn[: (i // 2 + 1) * 2]])
        assert np.allclose(o[i], vis.mean(axis=0), atol=1e-14)
    # V constant -> output constant
    o = chunk_attention(Q, Kc, 0 * Vc + 3.5, Kn, 0 * Vn + 3.5, block_len=2)
    assert np.allclose(o, 3.5, atol=1e-13)
    # adding one vector to every key shifts each row's logits by a constant: output unchanged
    c = 40.0 * rng.standard_normal((1, N, D))
    a = chunk_attention(Q, Kc, Vc, Kn, Vn, block_len=2)
    b = chunk_attention(Q, Kc + c, Vc, Kn + c, Vn, block_len=2)
    assert np.allclose(a, b, rtol=1e-9, atol=1e-10)
    # 1/sqrt(D) really is the scale: scaling Q by sqrt(D) with scale=1/D... use explicit scale
    d = chunk_attention(Q * math.sqrt(D), Kc, Vc, Kn, Vn, block_len=2, scale=1.0 / D)
    assert np.allclose(a, d, rtol=1e-12, atol=1e-13)


def test_heads_independent_rows_subset_and_convex_hull():
    rng = np.random.default_rng(7)
    n, Lc, N, D = 6, 9, 3, 4
    Q, Kc, Vc, Kn, Vn = _rand(rng, n, Lc, N, D)
    a = chunk_attention(Q, Kc, Vc, Kn, Vn, block_len=3)
    Q2 = Q.copy(); Q2[:, 1] += 1.0
    b = chunk_attention(Q2, Kc, Vc, Kn, Vn, block_len=3)
    assert np.array_equal(a[:, 0], b[:, 0]) and np.array_equal(a[:, 2], b[:, 2])
    assert not np.allclose(a[:, 1], b[:, 1])
    rows = np.array([8, 0, 4])
    assert np.allclose(chunk_attention(Q, Kc, Vc, Kn, Vn, block_len=3, rows=rows), a[rows], rtol=1e-13, atol=1e-15)
    V_all = np.concatenate([Vc, Vn])
    assert np.all(a <= V_all.max(axis=0)[None] + 1e-12) and np.all(a >= V_all.min(axis=0)[None] - 1e-12)


# ---------------------------------------------------------------- step / rollout
def _step_inputs(rng, n, Lc, N, D, M):
    H = N * D
    return dict(X_cache=rng.standard_normal((n, H)), X_chunk=rng.standard_normal((Lc, H)),
                W1=rng.standard_normal((M, H)) * 0.1, b1=None, W2=rng.standard_normal((1, M)), b2=None,
                K_cache=rng.standard_normal((n, N, D)), V_cache=rng.standard_normal((n, N, D)),
                Q=rng.standard_normal((Lc, N, D)), K_chunk=rng.standard_normal((Lc, N, D)),
                V_chunk=rng.standard_normal((Lc, N, D)))


def test_step_full_budget_equals_full_attention_and_leaves_cache_unchanged():
    rng = np.random.default_rng(8)
    n, Lc, N, D = 20, 8, 2, 4
    inp = _step_inputs(rng, n, Lc, N, D, 6)
    for k in (n, n + 3):
        r = step_single(**inp, k=k, block_len=Lc)
        assert r["ids"].tolist() == list(range(n))
        assert np.array_equal(r["K_kept"], inp["K_cache"]) and np.array_equal(r["V_kept"], inp["V_cache"])
        full = chunk_attention(inp["Q"], inp["K_cache"], inp["V_cache"], inp["K_chunk"], inp["V_chunk"], block_len=Lc)
        assert np.array_equal(r["O"], full)


def test_step_is_the_composition_and_honours_forced_scores():
    rng = np.random.default_rng(9)
    n, Lc, N, D, k = 30, 8, 2, 4, 11
    inp = _step_inputs(rng, n, Lc, N, D, 6)
    r = step_single(**inp, k=k, block_len=4)
    s = smlp_score(np.concatenate([inp["X_cache"], inp["X_chunk"]]), inp["W1"], None, inp["W2"], None)
    assert np.array_equal(r["scores"], s)
    ids = select_topk(s[:n].astype(np.float32), k)
    assert np.array_equal(r["ids"], ids)
    Kk, Vk, SLk = compact_kv(inp["K_cache"], inp["V_cache"], s[:n].astype(np.float32), ids)
    assert np.array_equal(r["K_kept"], Kk) and np.array_equal(r["SL_kept"], SLk)
    assert np.array_equal(r["O"], chunk_attention(inp["Q"], Kk, Vk, inp["K_chunk"], inp["V_chunk"], block_len=4))
    forced = np.arange(n + Lc, dtype=np.float32)
    r2 = step_single(**inp, k=k, block_len=4, forced_scores_f32=forced)
    assert r2["ids"].tolist() == list(range(n - k, n))


def test_rollout_sizes_competition_and_resume():
    rng = np.random.default_rng(10)
    N, D, Lc, k, M = 2, 4, 6, 10, 5
    H = N * D
    W1 = rng.standard_normal((M, H)) * 0.3
    W2 = rng.standard_normal((1, M))
    chunks = [dict(X_chunk=rng.standard_normal((Lc, H)), Q=rng.standard_normal((Lc, N, D)),
                   K_chunk=rng.standard_normal((Lc, N, D)), V_chunk=rng.standard_normal((Lc, N, D)))
              for _ in range(6)]
    st = RolloutState(N, D, np.float64)
    sizes, snap = [], None
    for t, c in enumerate(chunks):
        n_before = st.n
        out = rollout_step(st, c["X_chunk"], W1, None, W2, None, c["Q"], c["K_chunk"], c["V_chunk"], k, Lc)
        assert len(out["ids"]) == min(k, n_before)
        sizes.append(st.n)
        # the chunk is appended whole, with its scores, after the retained rows
        assert np.array_equal(st.K[-Lc:], c["K_chunk"]) and np.array_equal(st.SL[-Lc:], out["s_chunk"].astype(np.float32))
        if n_before <= k:
            assert out["ids"].tolist() == list(range(n_before))      # below budget nothing is evicted
        if t == 2:
            snap = st.copy()
    assert sizes == [6, 12, 16, 16, 16, 16]                          # min(k, n) + Lc
    # old and new tokens compete: the retained set is the top-k of stored+previous-chunk scores
    st2 = snap.copy()
    for c in chunks[3:]:
        rollout_step(st2, c["X_chunk"], W1, None, W2, None, c["Q"], c["K_chunk"], c["V_chunk"], k, Lc)
    assert np.array_equal(st2.K, st.K) and np.array_equal(st2.V, st.V) and np.array_equal(st2.SL, st.SL)
    # stored scores are never refreshed: every stored score is one some chunk produced
    produced = np.concatenate([smlp_score(c["X_chunk"], W1, None, W2, None).astype(np.float32) for c in chunks])
    assert set(st.SL.tolist()) <= set(produced.tolist())


# ---------------------------------------------------------------------- shared indices across layers (Sec. 3.3)
def test_shared_step_uses_one_index_list_for_every_layer():
    from oracle.pafu_oracle import step_single_shared
    rng = np.random.default_rng(21)
    n, Lc, N, D, k = 24, 6, 2, 4, 9
    inp = _step_inputs(rng, n, Lc, N, D, 6)
    kv_keys = ("K_cache", "V_cache", "Q", "K_chunk", "V_chunk")
    layers = [{key: rng.standard_normal(inp[key].shape) for key in kv_keys} for _ in range(2)]
    layers.append({key: inp[key] for key in kv_keys})          # the index layer's own cache goes last
    head = {key: inp[key] for key in ("X_cache", "X_chunk", "W1", "b1", "W2", "b2")}
    r = step_single_shared(**head, layers=layers, k=k, block_len=3)
    own = step_single(**inp, k=k, block_len=3)
    # the index layer behaves exactly like an independent step ...
    assert np.array_equal(r["ids"], own["ids"]) and np.array_equal(r["scores"], own["scores"])
    assert np.array_equal(r["layers"][2]["O"], own["O"]) and np.array_equal(r["layers"][2]["K_kept"], own["K_kept"])
    assert np.array_equal(r["SL_kept"], own["SL_kept"])
    # ... and every other layer keeps the SAME rows of its own cache, attends over them row by row as written
    for L, out in zip(layers[:2], r["layers"][:2]):
        for row, i in enumerate(r["ids"]):
            assert np.array_equal(out["K_kept"][row], L["K_cache"][i]) and np.array_equal(out["V_kept"][row], L["V_cache"][i])
        loops = _loops(L["Q"], L["K_cache"][r["ids"]], L["V_cache"][r["ids"]], L["K_chunk"], L["V_chunk"], 3)
        assert np.allclose(out["O"], loops, rtol=1e-12, atol=1e-13)
    # with a frame sink the first tokens stay in every layer
    r2 = step_single_shared(**head, layers=layers, k=k, block_len=3, n_pinned=4)
    assert r2["ids"][:4].tolist() == [0, 1, 2, 3]


def test_shared_rollout_keeps_layers_in_lockstep():
    from oracle.pafu_oracle import rollout_step_shared
    rng = np.random.default_rng(22)
    N, D, Lc, k, M, n_layers = 2, 4, 5, 8, 5, 3
    H = N * D
    W1 = rng.standard_normal((M, H)) * 0.3
    W2 = rng.standard_normal((1, M))
    states = [RolloutState(N, D, np.float64) for _ in range(n_layers)]
    solo = RolloutState(N, D, np.float64)                      # the index layer run on its own
    for t in range(5):
        X = rng.standard_normal((Lc, H))
        chunks = [dict(Q=rng.standard_normal((Lc, N, D)), K_chunk=rng.standard_normal((Lc, N, D)),
                       V_chunk=rng.standard_normal((Lc, N, D))) for _ in range(n_layers)]
        out = rollout_step_shared(states, n_layers - 1, X, W1, None, W2, None, chunks, k, Lc)
        ref = rollout_step(solo, X, W1, None, W2, None, chunks[-1]["Q"], chunks[-1]["K_chunk"], chunks[-1]["V_chunk"], k, Lc)
        assert np.array_equal(out["ids"], ref["ids"]) and np.array_equal(out["O"][-1], ref["O"])
        assert np.array_equal(states[-1].K, solo.K) and np.array_equal(states[-1].SL, solo.SL)
        assert len({st.n for st in states}) == 1                # all layers hold the same number of rows
    assert states[0].n == min(k, 4 * Lc) + Lc
