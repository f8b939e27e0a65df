"""GPU parity of pafu_step / pafu_step_layers (SINGLE and ROLLOUT) against the oracle.

Teacher-forced comparison: the device's own fp32 scores are fed to the oracle's selection, so ids and
the compacted cache must match bit for bit; the scores themselves within 1e-3; attention within
max-abs 2e-2 and relative Frobenius 5e-3."""
import numpy as np
import pytest
import torch

from oracle import pafu_oracle as orc
from paper_2601_21896_amd import binding as B
from paper_2601_21896_amd import workloads as wl
from tests.gpu_util import ATTN_MAX_ABS, ATTN_REL_FRO, DEV, SCORE_MAX_ABS, attn_errors, dev, host

pytestmark = pytest.mark.gpu


def _single(cfg, d, k, L_B, contiguous_features=True, n_pinned=0):
    n, Lc, N, D = d["n"], cfg.Lc, cfg.N, cfg.D
    dt = cfg.dtype
    rb = wl.round_to_bf16
    kv = {x: rb(d[x]) for x in ("K_cache", "V_cache", "Q", "K_chunk", "V_chunk")}
    if contiguous_features:
        X = dev(np.concatenate([d["X_cache"], d["X_chunk"]]), dt)
        x_cache, x_chunk = X[:n], X[n:]
    else:
        x_cache, x_chunk = dev(d["X_cache"], dt), dev(d["X_chunk"], dt)
    n_kept = min(k, n)
    scores = torch.empty(n + Lc, device=DEV)
    ids = torch.full((max(n_kept, 1),), -1, dtype=torch.int32, device=DEV)
    K_out = torch.zeros(max(n_kept, 1), N, D, device=DEV, dtype=torch.bfloat16)
    V_out = torch.zeros_like(K_out)
    SL_out = torch.zeros(max(n_kept, 1), device=DEV)
    O = torch.empty(Lc, N, D, device=DEV, dtype=torch.bfloat16)
    # the argument struct holds raw pointers only: keep every device tensor alive next to it
    w = [dev(d["W1"], dt), dev(d["b1"]), dev(d["W2"]), dev(d["b2"])]
    t = [dev(kv["K_cache"], "bf16") if n else None, dev(kv["V_cache"], "bf16") if n else None,
         dev(kv["Q"], "bf16"), dev(kv["K_chunk"], "bf16"), dev(kv["V_chunk"], "bf16")]
    args = B.make_step_args(B.PAFU_MODE_SINGLE, N, D, n, Lc, k, L_B, x_cache if n else None, x_chunk,
                            w[0], w[1], w[2], w[3], t[0], t[1], None, t[2], t[3], t[4],
                            scores, ids, K_out, V_out, SL_out, O, n_pinned=n_pinned)
    args._keep = (w, t, x_cache, x_chunk)
    return args, kv, scores, ids, K_out, V_out, SL_out, O, n_kept


def _check_single(cfg, d, k, L_B, args_pack, n_pinned=0):
    args, kv, scores, ids, K_out, V_out, SL_out, O, n_kept = args_pack
    torch.cuda.synchronize()
    got_s = host(scores)
    ref = orc.step_single(d["X_cache"], d["X_chunk"], d["W1"], d["b1"], d["W2"], d["b2"], kv["K_cache"], kv["V_cache"],
                          kv["Q"], kv["K_chunk"], kv["V_chunk"], k, L_B, forced_scores_f32=got_s, n_pinned=n_pinned)
    assert np.abs(got_s - ref["scores"]).max() < SCORE_MAX_ABS
    assert np.array_equal(host(ids)[:n_kept], ref["ids"])
    assert np.array_equal(host(K_out)[:n_kept], ref["K_kept"]) and np.array_equal(host(V_out)[:n_kept], ref["V_kept"])
    assert np.array_equal(host(SL_out)[:n_kept], ref["SL_kept"])
    max_abs, rel = attn_errors(host(O), ref["O"])
    assert max_abs < ATTN_MAX_ABS and rel < ATTN_REL_FRO, (max_abs, rel)
    # free-running check: indices may differ from the oracle's own selection only near the threshold
    own = orc.select_topk(ref["scores"][: d["n"]].astype(np.float32), k, n_pinned)
    diff = set(own.tolist()) ^ set(ref["ids"].tolist())
    if diff and n_kept:
        kth = np.sort(ref["scores"][: d["n"]])[::-1][n_kept - 1]
        assert all(abs(ref["scores"][i] - kth) < SCORE_MAX_ABS for i in diff)


@pytest.mark.parametrize("contig", [True, False])
def test_step_single_c0(contig):
    cfg = wl.C0
    d = wl.make_layer_inputs(cfg, bias=True)
    pack = _single(cfg, d, cfg.k, cfg.Lc, contiguous_features=contig)
    B.pafu_step(pack[0])
    _check_single(cfg, d, cfg.k, cfg.Lc, pack)


@pytest.mark.parametrize("k_mode,L_B", [("half", 0), ("all", 0), ("more", 0), ("zero", 0), ("half", 60)])
def test_step_single_c1_shaped(k_mode, L_B):
    cfg = wl.scaled(wl.C1, frame_tokens=60, cache_frames=9, chunk_frames=3, k=270)     # n = 540, Lc = 180
    d = wl.make_layer_inputs(cfg)
    k = {"half": 270, "all": 540, "more": 1000, "zero": 0}[k_mode]
    L_B = L_B or cfg.Lc
    pack = _single(cfg, d, k, L_B)
    B.pafu_step(pack[0])
    _check_single(cfg, d, k, L_B, pack)
    if k_mode in ("all", "more"):      # budget >= cache: cache unchanged
        assert np.array_equal(host(pack[4]), wl.round_to_bf16(d["K_cache"]))


@pytest.mark.parametrize("n_pinned", [60, 270, 400])
def test_step_single_with_frame_sink(n_pinned):
    # the first n_pinned cached tokens (one frame = 60 tokens here) survive whatever their scores are
    cfg = wl.scaled(wl.C1, frame_tokens=60, cache_frames=9, chunk_frames=3, k=270)     # n = 540, Lc = 180
    d = wl.make_layer_inputs(cfg)
    d["X_cache"][:n_pinned] -= 3.0                      # make the pinned tokens the least salient ones
    d["X_cache"] = wl.round_to_bf16(d["X_cache"])       # keep the device cast exact
    pack = _single(cfg, d, 270, cfg.Lc, n_pinned=n_pinned)
    B.pafu_step(pack[0])
    _check_single(cfg, d, 270, cfg.Lc, pack, n_pinned=n_pinned)
    kept = host(pack[3])[:270]
    assert kept[:min(n_pinned, 270)].tolist() == list(range(min(n_pinned, 270)))


def test_step_single_empty_cache():
    cfg = wl.scaled(wl.C1, frame_tokens=50, cache_frames=0, chunk_frames=2, k=10)
    d = wl.make_layer_inputs(cfg)
    pack = _single(cfg, d, 10, cfg.Lc)
    B.pafu_step(pack[0])
    _check_single(cfg, d, 10, cfg.Lc, pack)


def test_step_layers_independent():
    cfg = wl.scaled(wl.C1, frame_tokens=40, cache_frames=6, chunk_frames=2, k=120)
    layers = [wl.make_layer_inputs(cfg, seed=wl.BASE_SEED + 2 + 1000 * l) for l in range(3)]
    packs = [_single(cfg, d, cfg.k, cfg.Lc) for d in layers]
    B.pafu_step_layers([p[0] for p in packs])
    ids_seen = []
    for d, p in zip(layers, packs):
        _check_single(cfg, d, cfg.k, cfg.Lc, p)
        ids_seen.append(host(p[3]).tolist())
    assert ids_seen[0] != ids_seen[1]


def test_step_layers_many_layers_with_different_cache_sizes():
    # more layers than one batched selection launch holds, cache sizes differ from layer to layer (one is empty)
    packs, metas = [], []
    for l in range(34):
        frames = [0, 2, 5, 3][l % 4]
        cfg = wl.scaled(wl.C1, frame_tokens=16, cache_frames=frames, chunk_frames=1, k=40)
        d = wl.make_layer_inputs(cfg, seed=wl.BASE_SEED + 11 + 1000 * l)
        packs.append(_single(cfg, d, 40, cfg.Lc))
        metas.append((cfg, d))
    B.pafu_step_layers([p[0] for p in packs])
    for (cfg, d), p in zip(metas, packs):
        _check_single(cfg, d, 40, cfg.Lc, p)


def _rollout(cfg, k, n_chunks, L_B, stop_at=None, resume=None, n_pinned=0):
    """Runs the device rollout beside the oracle's (teacher-forced on the chunk scores)."""
    N, D, Lc = cfg.N, cfg.D, cfg.Lc
    W1, b1, W2, b2 = wl.make_rollout_weights(cfg, bias=True)
    dW1, db1, dW2, db2 = dev(W1, "bf16"), dev(b1), dev(W2), dev(b2)
    cap = k + Lc
    slabs = [dict(K=torch.zeros(cap, N, D, device=DEV, dtype=torch.bfloat16),
                  V=torch.zeros(cap, N, D, device=DEV, dtype=torch.bfloat16),
                  SL=torch.zeros(cap, device=DEV)) for _ in range(2)]
    st = orc.RolloutState(N, D, np.float32)
    n, cur, t0 = 0, 0, 0
    if resume is not None:
        n, t0 = resume["n"], resume["t"]
        for key in ("K", "V", "SL"):
            slabs[0][key][:n] = resume[key]
        st = resume["oracle"].copy()
    ids = torch.empty(max(k, 1), dtype=torch.int32, device=DEV)
    O = torch.empty(Lc, N, D, device=DEV, dtype=torch.bfloat16)
    sizes = []
    for t in range(t0, n_chunks):
        c = wl.make_chunk_inputs(cfg, t)
        src, dst = slabs[cur], slabs[1 - cur]
        n_kept = min(k, n)
        args = B.make_step_args(B.PAFU_MODE_ROLLOUT, N, D, n, Lc, k, L_B, None, dev(c["X_chunk"], "bf16"), dW1, db1,
                                dW2, db2, src["K"], src["V"], src["SL"], dev(c["Q"], "bf16"), dev(c["K_chunk"], "bf16"),
                                dev(c["V_chunk"], "bf16"), None, ids, dst["K"], dst["V"], dst["SL"], O,
                                n_pinned=n_pinned)
        B.pafu_step(args)
        torch.cuda.synchronize()
        s_chunk = host(dst["SL"][n_kept:n_kept + Lc])
        out = orc.rollout_step(st, c["X_chunk"], W1, b1, W2, b2, c["Q"], c["K_chunk"], c["V_chunk"], k, L_B,
                               forced_chunk_scores_f32=s_chunk, n_pinned=n_pinned)
        assert np.abs(s_chunk - out["s_chunk"]).max() < SCORE_MAX_ABS
        assert np.array_equal(host(ids)[:n_kept], out["ids"]), t
        n = n_kept + Lc
        assert n == st.n
        assert np.array_equal(host(dst["K"][:n]), st.K) and np.array_equal(host(dst["V"][:n]), st.V), t
        assert np.array_equal(host(dst["SL"][:n]), st.SL), t
        max_abs, rel = attn_errors(host(O), out["O"])
        assert max_abs < ATTN_MAX_ABS and rel < ATTN_REL_FRO, (t, max_abs, rel)
        sizes.append(n)
        cur = 1 - cur
        if stop_at is not None and t + 1 == stop_at:
            return dict(n=n, t=t + 1, K=slabs[cur]["K"][:n].clone(), V=slabs[cur]["V"][:n].clone(),
                        SL=slabs[cur]["SL"][:n].clone(), oracle=st.copy()), sizes
    return dict(n=n, K=slabs[cur]["K"][:n].clone(), V=slabs[cur]["V"][:n].clone(), SL=slabs[cur]["SL"][:n].clone()), sizes


def test_rollout_matches_oracle_and_resumes_bit_identically():
    cfg = wl.scaled(wl.C1, frame_tokens=30, chunk_frames=3, cache_frames=0, k=240)     # Lc = 90, k = 8 frames
    full, sizes = _rollout(cfg, 240, 8, cfg.Lc)
    assert sizes == [90, 180, 270, 330, 330, 330, 330, 330]
    snap, _ = _rollout(cfg, 240, 8, cfg.Lc, stop_at=4)
    resumed, _ = _rollout(cfg, 240, 8, cfg.Lc, resume=snap)
    for key in ("K", "V", "SL"):
        assert torch.equal(full[key], resumed[key])


def test_rollout_full_budget_never_evicts():
    cfg = wl.scaled(wl.C1, frame_tokens=20, chunk_frames=2, cache_frames=0, k=10 ** 6)
    N, D, Lc = cfg.N, cfg.D, cfg.Lc
    out, sizes = _rollout(wl.scaled(cfg, k=400), 400, 5, 20)
    assert sizes == [40, 80, 120, 160, 200]


@pytest.mark.parametrize("N,D", [(40, 128), (52, 128), (3, 64)])
def test_rollout_row_sizes_on_both_sides_of_the_fused_append(N, D):
    # rows of 10 KiB (appended by the compaction launch), 13 KiB (beyond the unrolled copy: generic compaction and a
    # separate append) and 384 B; the oracle comparison inside _rollout covers the whole slab after every step
    cfg = wl.scaled(wl.C1, N=N, D=D, M=32, frame_tokens=12, chunk_frames=2, cache_frames=0, k=60)     # Lc = 24
    out, sizes = _rollout(cfg, 60, 6, cfg.Lc)
    assert sizes == [24, 48, 72, 84, 84, 84]


def test_rollout_with_zero_budget_keeps_only_the_chunk():
    # k = 0: every step evicts the whole cache (the selection that rides in the scoring launch writes no index, the
    # compaction launch has no row to gather and only appends the chunk), attention sees the chunk alone
    cfg = wl.scaled(wl.C1, frame_tokens=30, chunk_frames=3, cache_frames=0, k=0)     # Lc = 90
    out, sizes = _rollout(cfg, 0, 4, cfg.Lc)
    assert sizes == [90, 90, 90, 90]


def test_rollout_with_frame_sink_keeps_the_first_frame():
    cfg = wl.scaled(wl.C1, frame_tokens=30, chunk_frames=3, cache_frames=0, k=240)     # Lc = 90
    first = wl.round_to_bf16(wl.make_chunk_inputs(cfg, 0)["K_chunk"])[:30]
    out, sizes = _rollout(cfg, 240, 8, cfg.Lc, n_pinned=30)
    assert sizes == [90, 180, 270, 330, 330, 330, 330, 330]
    # the first frame of the first chunk still heads the cache after five evictions
    assert np.array_equal(host(out["K"][:30]), first)
    plain, _ = _rollout(cfg, 240, 8, cfg.Lc)
    assert not torch.equal(plain["K"], out["K"])


# ------------------------------------------------------------------ shared indices across layers (Sec. 3.3)
@pytest.mark.parametrize("n_pinned", [0, 40])
def test_step_layers_shared_single(n_pinned):
    cfg = wl.scaled(wl.C1, frame_tokens=40, cache_frames=6, chunk_frames=2, k=120)      # n = 240, Lc = 80
    layers = [wl.make_layer_inputs(cfg, seed=wl.BASE_SEED + 7 + 1000 * l) for l in range(3)]
    idx = 2
    packs = [_single(cfg, d, cfg.k, cfg.Lc, n_pinned=n_pinned) for d in layers]
    for p in packs[:idx]:
        p[3].fill_(-5)                                       # ids of the other layers must stay untouched
    B.pafu_step_layers_shared([p[0] for p in packs], idx)
    torch.cuda.synchronize()
    d = layers[idx]
    got_s = host(packs[idx][2])
    kvs = [p[1] for p in packs]
    ref = orc.step_single_shared(d["X_cache"], d["X_chunk"], d["W1"], d["b1"], d["W2"], d["b2"], kvs, cfg.k, cfg.Lc,
                                 forced_scores_f32=got_s, n_pinned=n_pinned)
    assert np.abs(got_s - ref["scores"]).max() < SCORE_MAX_ABS
    n_kept = cfg.k
    assert np.array_equal(host(packs[idx][3])[:n_kept], ref["ids"])
    assert np.array_equal(host(packs[idx][6])[:n_kept], ref["SL_kept"])
    for l, (p, out) in enumerate(zip(packs, ref["layers"])):
        assert np.array_equal(host(p[4])[:n_kept], out["K_kept"]) and np.array_equal(host(p[5])[:n_kept], out["V_kept"]), l
        max_abs, rel = attn_errors(host(p[7]), out["O"])
        assert max_abs < ATTN_MAX_ABS and rel < ATTN_REL_FRO, (l, max_abs, rel)
    for p in packs[:idx]:
        assert torch.all(p[3] == -5)
    # the layers do differ: same rows kept, different contents
    assert not np.array_equal(host(packs[0][4]), host(packs[1][4]))


def test_step_layers_shared_rollout():
    cfg = wl.scaled(wl.C1, frame_tokens=30, chunk_frames=2, cache_frames=0, k=150)      # Lc = 60
    N, D, Lc, k, n_layers, idx = cfg.N, cfg.D, cfg.Lc, 150, 3, 2
    W1, b1, W2, b2 = wl.make_rollout_weights(cfg, bias=True)
    dW = (dev(W1, "bf16"), dev(b1), dev(W2), dev(b2))
    cap = k + Lc
    slabs = [[dict(K=torch.zeros(cap, N, D, device=DEV, dtype=torch.bfloat16),
                   V=torch.zeros(cap, N, D, device=DEV, dtype=torch.bfloat16),
                   SL=torch.zeros(cap, device=DEV)) for _ in range(2)] for _ in range(n_layers)]
    states = [orc.RolloutState(N, D, np.float32) for _ in range(n_layers)]
    ids = torch.empty(k, dtype=torch.int32, device=DEV)
    Os = [torch.empty(Lc, N, D, device=DEV, dtype=torch.bfloat16) for _ in range(n_layers)]
    n, cur = 0, 0
    for t in range(6):
        chunks = [wl.make_chunk_inputs(cfg, 10 * t + l) for l in range(n_layers)]
        X = chunks[idx]["X_chunk"]
        n_kept = min(k, n)
        args = []
        for l in range(n_layers):
            src, dst, c = slabs[l][cur], slabs[l][1 - cur], chunks[l]
            is_idx = l == idx
            args.append(B.make_step_args(
                B.PAFU_MODE_ROLLOUT, N, D, n, Lc, k, Lc, None, dev(X, "bf16"), dW[0], dW[1], dW[2], dW[3],
                src["K"], src["V"], src["SL"] if is_idx else None, dev(c["Q"], "bf16"), dev(c["K_chunk"], "bf16"),
                dev(c["V_chunk"], "bf16"), None, ids if is_idx else None, dst["K"], dst["V"],
                dst["SL"] if is_idx else None, Os[l], n_pinned=30))
        B.pafu_step_layers_shared(args, idx)
        torch.cuda.synchronize()
        s_chunk = host(slabs[idx][1 - cur]["SL"][n_kept:n_kept + Lc])
        out = orc.rollout_step_shared(states, idx, X, W1, b1, W2, b2, chunks, k, Lc, forced_chunk_scores_f32=s_chunk,
                                      n_pinned=30)
        assert np.abs(s_chunk - out["s_chunk"]).max() < SCORE_MAX_ABS
        assert np.array_equal(host(ids)[:n_kept], out["ids"]), t
        n = n_kept + Lc
        for l in range(n_layers):
            dst = slabs[l][1 - cur]
            assert np.array_equal(host(dst["K"][:n]), states[l].K) and np.array_equal(host(dst["V"][:n]), states[l].V), (t, l)
            max_abs, rel = attn_errors(host(Os[l]), out["O"][l])
            assert max_abs < ATTN_MAX_ABS and rel < ATTN_REL_FRO, (t, l, max_abs, rel)
        assert np.array_equal(host(slabs[idx][1 - cur]["SL"][:n]), states[idx].SL), t
        cur = 1 - cur
    assert n == k + Lc


def test_step_layers_rollout_independent_indices():
    # pafu_step_layers in ROLLOUT: every layer scores its own chunk, selects on its own stored list, and the one
    # compaction launch also appends every layer's chunk rows; each layer against its own oracle rollout
    cfg = wl.scaled(wl.C1, frame_tokens=30, chunk_frames=2, cache_frames=0, k=150)      # Lc = 60
    N, D, Lc, k, n_layers = cfg.N, cfg.D, cfg.Lc, 150, 3
    W1, b1, W2, b2 = wl.make_rollout_weights(cfg, bias=True)
    dW = (dev(W1, "bf16"), dev(b1), dev(W2), dev(b2))
    cap = k + Lc
    slabs = [[dict(K=torch.zeros(cap, N, D, device=DEV, dtype=torch.bfloat16),
                   V=torch.zeros(cap, N, D, device=DEV, dtype=torch.bfloat16),
                   SL=torch.zeros(cap, device=DEV)) for _ in range(2)] for _ in range(n_layers)]
    states = [orc.RolloutState(N, D, np.float32) for _ in range(n_layers)]
    ids = [torch.empty(k, dtype=torch.int32, device=DEV) for _ in range(n_layers)]
    Os = [torch.empty(Lc, N, D, device=DEV, dtype=torch.bfloat16) for _ in range(n_layers)]
    n, cur = 0, 0
    for t in range(5):
        chunks = [wl.make_chunk_inputs(cfg, 10 * t + l) for l in range(n_layers)]
        n_kept = min(k, n)
        args = []
        for l in range(n_layers):
            src, dst, c = slabs[l][cur], slabs[l][1 - cur], chunks[l]
            args.append(B.make_step_args(
                B.PAFU_MODE_ROLLOUT, N, D, n, Lc, k, Lc, None, dev(c["X_chunk"], "bf16"), dW[0], dW[1], dW[2], dW[3],
                src["K"], src["V"], src["SL"], dev(c["Q"], "bf16"), dev(c["K_chunk"], "bf16"),
                dev(c["V_chunk"], "bf16"), None, ids[l], dst["K"], dst["V"], dst["SL"], Os[l]))
        B.pafu_step_layers(args)
        torch.cuda.synchronize()
        for l in range(n_layers):
            dst, c = slabs[l][1 - cur], chunks[l]
            s_chunk = host(dst["SL"][n_kept:n_kept + Lc])
            out = orc.rollout_step(states[l], c["X_chunk"], W1, b1, W2, b2, c["Q"], c["K_chunk"], c["V_chunk"], k, Lc,
                                   forced_chunk_scores_f32=s_chunk)
            assert np.abs(s_chunk - out["s_chunk"]).max() < SCORE_MAX_ABS
            assert np.array_equal(host(ids[l])[:n_kept], out["ids"]), (t, l)
            m = n_kept + Lc
            assert np.array_equal(host(dst["K"][:m]), states[l].K) and np.array_equal(host(dst["V"][:m]), states[l].V), (t, l)
            assert np.array_equal(host(dst["SL"][:m]), states[l].SL), (t, l)
            max_abs, rel = attn_errors(host(Os[l]), out["O"])
            assert max_abs < ATTN_MAX_ABS and rel < ATTN_REL_FRO, (t, l, max_abs, rel)
        n = n_kept + Lc
        cur = 1 - cur
    assert n == k + Lc
