#!/usr/bin/env python3
"""Benchmark of the PaFu-KV chunk step on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input: score all cached and
chunk tokens with the S-MLP, select the top-k cached tokens, compact K/V/SL, and attend from the chunk's
queries over the retained cache plus the chunk (pafu_step, SINGLE mode).  The default workload is the
Wan-1.3B-shaped single layer in bf16 (12 heads x 128, 32760 cached + 4680 chunk tokens, budget 16380).

Prints ONE JSON line: ms per step (inputs resident in HBM), a per-stage breakdown and the duration of the
dominant kernel (attention, dense bf16 MFMA) measured with events that the library records on the launch
stream inside whole steps, the parity of the last step's buffers against the fp64 oracle, a sustained
figure from a run of at least a second, and the oracle timed on this machine's host cores.  The process exits
with status 1 when a parity figure is out of tolerance.
"""

from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E
METRIC = "ms per AR chunk step (score+select+compact+attn), MFMA util and HBM GB/s"
FP8_SCALES = (-5, -6)         # log2 of the K and V scales of the 8-bit cache: |K| <= 14, |V| <= 7 representable
TOL = {"score_max_abs": 1e-3, "attn_max_abs": 2e-2, "attn_rel_fro": 5e-3}   # the benchmark spec's tolerances

# HBM bytes per attention launch from rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE, scaled by a copy kernel): a figure
# from a separate counter run whose summary is tracked under profiles/, NOT re-measured by this run.
ATTENTION_TRAFFIC = {
    # profiles/step_C1_hbm_traffic_pmc.md: 107200 KiB x 1.98 fetched + 14040 KiB written
    ("C1", True): (int((107200 * 1.98 + 14040) * 1024), "profiles/step_C1_hbm_traffic_pmc.md"),
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="C1", choices=["C1", "C4", "C2", "C0", "C3", "SSE", "ATTN"])
    ap.add_argument("--budget", type=int, default=0, help="C3 only: cache budget k in tokens (default 8 frames = 12480)")
    ap.add_argument("--block-len", type=int, default=0, help="L_B (0 = chunk length, the paper's setting)")
    ap.add_argument("--structure", default="uniform", choices=["uniform", "coherent"])
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle leg (then no parity figures either)")
    ap.add_argument("--sets", type=int, default=3, help="input buffer sets rotated between steps")
    ap.add_argument("--shared-index", action="store_true",
                    help="C2 only: score + select once on the last layer, every layer reuses its indices (Sec. 3.3)")
    ap.add_argument("--head", default="benchmark", choices=["benchmark", "paper"],
                    help="S-MLP widths: the benchmark's (F = H, M from the config, 1 output) or App. A's "
                         "([Q|K|V] = 3H inputs, 1024 hidden, 12 outputs averaged)")
    ap.add_argument("--pinned", type=int, default=0, help="frame sink: cached tokens [0, pinned) are never evicted")
    ap.add_argument("--graph", action="store_true",
                    help="time replays of the step captured as a HIP graph (one graph per input set); the stage "
                         "breakdown still comes from eager steps")
    ap.add_argument("--sustained-s", type=float, default=1.0,
                    help="length of the extra back-to-back run behind sustained_ms_per_step (0 = skip)")
    ap.add_argument("--chunk-frames", type=int, default=0, help="ATTN only: frames per chunk (default 3)")
    ap.add_argument("--no-attention-workspace", action="store_true",
                    help="ATTN only: call pafu_chunk_attention without a workspace (never cuts its work into equal runs)")
    ap.add_argument("--shape", default="C1", choices=["C1", "C4"],
                    help="ATTN only: heads, frame size and budget of the Wan-1.3B (C1) or Wan-14B (C4) layer")
    ap.add_argument("--data", default="normal", choices=["normal", "zeros"],
                    help="ATTN only: N(0,1) tensors (default) or all-zero tensors (same instructions, no operand toggling)")
    ap.add_argument("--kv", default="bf16", choices=["bf16", "fp8"],
                    help="storage of the K/V cache: bf16, or 8-bit E4M3 codes with power-of-two scales 2^-5 (K), 2^-6 (V)")
    ap.add_argument("--library", default="", help="load this build of libpafu.so instead of the in-tree default")
    return ap.parse_args()


def event_pair_ms(evs):
    return [evs[i].elapsed_time(evs[i + 1]) for i in range(len(evs) - 1)]


def new_events(torch, count):
    """Timing events whose handles exist (torch creates them lazily at the first record)."""
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(count)]
    for e in evs:
        e.record()
    return evs


def sse(a, torch, np, B, wl):
    """Teacher-side salience score (Sec. 3.2, Eq. 4-5) at the Wan-1.3B teacher shape: 21 frames x 1560 tokens,
    12 heads x 128, blocks of 3 frames.  Not the headline metric: a second measured workload."""
    cfg = wl.C1
    L, N, D, L_B = cfg.n, cfg.N, cfg.D, a.block_len or cfg.Lc
    dev = "cuda:0"
    rng = np.random.Generator(np.random.PCG64(wl.BASE_SEED + 9))
    c = rng.uniform(0.5, 2.0, size=(N * D,)).astype(np.float32)
    sets = []
    for s_ in range(2):
        Q = torch.from_numpy(rng.standard_normal((L, N * D), dtype=np.float32)).to(dev).to(torch.bfloat16)
        K = (torch.from_numpy(rng.standard_normal((L, N * D), dtype=np.float32)) * torch.from_numpy(c)).to(dev)
        sets.append((Q.view(L, N, D), K.to(torch.bfloat16).view(L, N, D)))
    out = torch.empty(L, device=dev)
    ws = torch.empty(B.pafu_sse_workspace_bytes(L, N) // 4, device=dev)
    for i in range(a.warmup):
        B.pafu_sse_score(sets[i % 2][0], sets[i % 2][1], L_B, out, ws)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(a.steps):
        B.pafu_sse_score(sets[i % 2][0], sets[i % 2][1], L_B, out, ws)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / a.steps
    flops = 2 * 2.0 * L * L * D * N          # two passes over Q K^T
    print(json.dumps({
        "metric": "ms per SSE salience score (Eq. 4-5)", "value": ms, "unit": "ms", "n_gpus": 1, "steps": a.steps,
        "warmup": a.warmup, "ms_per_step": ms, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "SSE: %d tokens (21 frames x 1560), %d heads x %d, L_B=%d" % (L, N, D, L_B)},
        "roofline": {"kernel": "sse_pass_kernel (both passes)", "bound": "mfma", "achieved": flops / ms / 1e9,
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": flops / ms / 1e9 / PEAK_BF16_TFLOPS,
                     "traffic": None, "flops_per_launch": flops},
        "cpu_baseline": None}))


def attention_only(a, torch, np, B, wl):
    """The attention stage alone at the Wan-1.3B (or Wan-14B) layer shape (retained cache + chunk), launched back to
    back: the workload of the kernel studies under profiles/ (N(0,1) or all-zero tensors, any build of the library)."""
    cfg = wl.CONFIGS[a.shape]
    dev = "cuda:0"
    N, D, k = cfg.N, cfg.D, cfg.k
    Lc = (a.chunk_frames or cfg.chunk_frames) * cfg.frame_tokens
    L_B = a.block_len or Lc
    g = torch.Generator(device=dev)
    g.manual_seed(wl.BASE_SEED)

    def tensor(rows):
        if a.data == "zeros":
            return torch.zeros(rows, N, D, device=dev, dtype=torch.bfloat16)
        return torch.randn(rows, N, D, device=dev, generator=g).to(torch.bfloat16)
    sets = [(tensor(Lc), tensor(k), tensor(k), tensor(Lc), tensor(Lc)) for _ in range(max(1, a.sets))]
    if a.kv == "fp8":       # both key segments as codes
        def codes(Kt, Vt):
            Kq = torch.empty(Kt.shape[0], N * D, dtype=torch.uint8, device=dev)
            Vq = torch.empty_like(Kq)
            B.pafu_quantize_kv(Kt, Vt, FP8_SCALES[0], FP8_SCALES[1], Kq, Vq)
            return Kq, Vq
        sets = [(Q,) + codes(Kc, Vc) + codes(Kn, Vn) for Q, Kc, Vc, Kn, Vn in sets]
    O = torch.empty(Lc, N, D, device=dev, dtype=torch.bfloat16)
    ws = torch.empty(B.pafu_attention_workspace_bytes(Lc, N, D), dtype=torch.uint8, device=dev)

    def run(i):
        Q, Kc, Vc, Kn, Vn = sets[i % len(sets)]
        w = None if a.no_attention_workspace else ws
        if a.kv == "fp8":
            B.pafu_chunk_attention_fp8(Q, Kc, Vc, k, Kn, Vn, L_B, FP8_SCALES[0], FP8_SCALES[1], O, workspace=w)
        else:
            B.pafu_chunk_attention(Q, Kc, Vc, k, Kn, Vn, L_B, O, workspace=w)
    for i in range(a.warmup):
        run(i)
    torch.cuda.synchronize()
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(a.steps + 1)]
    evs[0].record()
    for i in range(a.steps):
        run(i)
        evs[i + 1].record()
    torch.cuda.synchronize()
    t = np.array(event_pair_ms(evs))
    ms = float(evs[0].elapsed_time(evs[-1]) / a.steps)
    pairs = Lc * k + sum(min(Lc, (i // L_B + 1) * L_B) for i in range(Lc))
    flops = 4.0 * pairs * D * N
    print(json.dumps({
        "metric": "ms per chunk-attention launch", "value": ms, "unit": "ms", "n_gpus": 1, "steps": a.steps,
        "warmup": a.warmup, "ms_per_step": ms, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic (%s)" % ("N(0,1)" if a.data == "normal" else "all zeros"),
        "config": {"workload": "ATTN: %d queries x (%d retained + %d chunk keys), %d heads x %d, L_B=%d" %
                               (Lc, k, Lc, N, D, L_B), "library": a.library or "in-tree libpafu.so",
                   "kv_storage": a.kv},
        "median_ms": float(np.median(t)), "min_ms": float(t.min()),
        "roofline": {"kernel": "chunk_attention_kernel", "bound": "mfma", "achieved": flops / ms / 1e9,
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": flops / ms / 1e9 / PEAK_BF16_TFLOPS,
                     "traffic": None, "flops_per_launch": flops, "avg_launch_ms": ms},
        "cpu_baseline": None}))


def rollout(a, torch, np, B, wl):
    """C3: 60 sequential chunks at the Wan-1.3B layer shapes, fixed budget; steady-state ms per step, per-stage
    durations from the library's stage events, peak cache bytes."""
    dev = "cuda:0"
    bf = torch.bfloat16
    cfg = wl.C1
    N, D, Lc, H, M = cfg.N, cfg.D, cfg.Lc, cfg.H, cfg.M
    k = a.budget or wl.C3_K
    n_chunks = wl.C3_CHUNKS
    cap = k + Lc
    W1n, b1n, W2n, b2n = wl.make_rollout_weights(cfg)
    t = lambda arr, b16=False: (torch.from_numpy(np.ascontiguousarray(arr)).to(dev).to(bf) if b16
                                else torch.from_numpy(np.ascontiguousarray(arr)).to(dev))
    W1, W2 = t(W1n, True), t(W2n)
    pool = []
    for c in range(4):      # chunk inputs cycle through 4 generated sets (fresh K/V/features per chunk seed)
        ci = wl.make_chunk_inputs(cfg, c)
        pool.append(dict(X=t(ci["X_chunk"], True), Q=t(ci["Q"], True), K=t(ci["K_chunk"], True), V=t(ci["V_chunk"], True)))
    fp8 = a.kv == "fp8"
    kvb = 1 if fp8 else 2
    if fp8:
        slabs = [dict(K=torch.zeros(cap, N * D, device=dev, dtype=torch.uint8),
                      V=torch.zeros(cap, N * D, device=dev, dtype=torch.uint8), SL=torch.zeros(cap, device=dev))
                 for _ in range(2)]
    else:
        slabs = [dict(K=torch.zeros(cap, N, D, device=dev, dtype=bf), V=torch.zeros(cap, N, D, device=dev, dtype=bf),
                      SL=torch.zeros(cap, device=dev)) for _ in range(2)]
    kv_args = dict(kv_dtype=B.PAFU_FP8_E4M3, k_scale_log2=FP8_SCALES[0], v_scale_log2=FP8_SCALES[1]) if fp8 else {}
    ids = torch.empty(max(k, 1), dtype=torch.int32, device=dev)
    O = torch.empty(Lc, N, D, device=dev, dtype=bf)
    ws = torch.empty(B.pafu_attention_workspace_bytes(Lc, N, D), dtype=torch.uint8, device=dev)
    stage_names = ("score", "select", "compact", "attention")
    def make_args(step, n, cur):
        c = pool[step % len(pool)]
        src, dst = slabs[cur], slabs[1 - cur]
        return B.make_step_args(B.PAFU_MODE_ROLLOUT, N, D, n, Lc, k, Lc, None, c["X"], W1, None, W2, None, src["K"],
                                src["V"], src["SL"], c["Q"], c["K"], c["V"], None, ids, dst["K"], dst["V"],
                                dst["SL"], O, n_pinned=a.pinned, workspace=ws, **kv_args)

    times, sizes, stage_t = [], [], []
    for rep in range(2):    # first pass warms up; the second gives the per-stage times (host waits after every step)
        n, cur = 0, 0
        times, sizes, stage_t = [], [], []
        for step in range(n_chunks):
            args = make_args(step, n, cur)
            sev = new_events(torch, 5)
            B.set_stage_events(args, sev)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            B.pafu_step(args)
            e1.record()
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1))
            stage_t.append(event_pair_ms(sev))
            n = min(k, n) + Lc
            sizes.append(n)
            cur = 1 - cur
    synced = times
    # The headline pass: the same rollout with all steps queued on the stream at once (cache sizes are known on the
    # host in advance: n' = min(k, n) + Lc, and stream order carries the dependence from step to step), one event
    # between steps, one host synchronisation at the end.
    n, cur = 0, 0
    marks, keep = [torch.cuda.Event(enable_timing=True) for _ in range(n_chunks + 1)], []
    marks[0].record()
    for step in range(n_chunks):
        args = make_args(step, n, cur)
        keep.append(args)
        B.pafu_step(args)
        marks[step + 1].record()
        n = min(k, n) + Lc
        cur = 1 - cur
    torch.cuda.synchronize()
    times = event_pair_ms(marks)
    steady = times[5:]
    st = np.array(stage_t[5:])
    n_steady = sizes[-1]
    n_kept = min(k, n_steady - Lc)
    flops = 4.0 * Lc * (n_kept + Lc) * D * N
    attn_ms = float(np.mean(st[:, 3]))
    peak_cache = 2 * (cap * N * D * kvb * 2 + cap * 4)
    # between the events around compaction: the gather of the retained rows (read + write, K and V, ids, scores) and
    # the chunk's rows put behind them (bf16: copied by the same launch; 8-bit: quantised, 2 bytes in, 1 out)
    bytes_compact = 2 * (2 * n_kept * N * D * kvb) + 3 * n_kept * 4 + 2 * Lc * N * D * (2 + kvb)
    out = {
        "metric": METRIC, "value": float(np.median(steady)), "unit": "ms",
        "n_gpus": 1, "steps": len(steady), "warmup": n_chunks + 5, "ms_per_step": float(np.median(steady)),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "C3: %d-chunk rollout, 12 heads x 128, chunk %d queries, budget %d tokens, steady cache "
                               "%d tokens, S-MLP %d->%d->1" % (n_chunks, Lc, k, n_steady, H, M), "kv_storage": a.kv},
        "ms_per_step_host_waits": float(np.median(synced[5:])),
        "min_ms": float(np.min(steady)), "first_steps_ms": [float(x) for x in times[:5]], "cache_sizes_first_steps": sizes[:6],
        "peak_cache_bytes": peak_cache,
        "stages": {s: {"ms": float(np.mean(st[:, j])), "min_ms": float(np.min(st[:, j]))} for j, s in enumerate(stage_names)},
        "stage_note": "ROLLOUT: the selection on the stored list is done by one workgroup of the scoring launch (lists up "
                      "to 65536 scores), so the interval after scoring is empty; the compaction launch also appends the "
                      "chunk's rows (bf16) / is followed by the chunk's quantisation (8-bit), both inside 'compact'",
        "compact_bytes": bytes_compact,
        "compact_GB/s": bytes_compact / float(np.mean(st[:, 2])) / 1e6 if n_kept else None,
        "roofline": {"kernel": "chunk_attention_kernel", "bound": "mfma", "achieved": flops / attn_ms / 1e9,
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": flops / attn_ms / 1e9 / PEAK_BF16_TFLOPS,
                     "traffic": None, "flops_per_launch": flops, "avg_launch_ms": attn_ms,
                     "note": "steady-state launches (cache %d + chunk %d keys), events recorded by the library "
                             "around the attention launch inside each step" % (n_kept, Lc)},
        "cpu_baseline": None,
    }
    print(json.dumps(out))


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build measures one GPU only (the path has no multi-GPU part); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    from paper_2601_21896_amd import binding as B
    from paper_2601_21896_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    if a.library:
        B.LIB_PATH = os.path.abspath(a.library)
    B.library()
    dev = "cuda:0"
    torch.cuda.set_device(0)

    if a.workload == "C3":
        rollout(a, torch, np, B, wl)
        return
    if a.workload == "SSE":
        sse(a, torch, np, B, wl)
        return
    if a.workload == "ATTN":
        attention_only(a, torch, np, B, wl)
        return
    n_layers = wl.C2_LAYERS if a.workload == "C2" else 1
    cfg = wl.C1 if a.workload == "C2" else wl.CONFIGS[a.workload]
    N, D, n, Lc, k, H, M = cfg.N, cfg.D, cfg.n, cfg.Lc, cfg.k, cfg.H, cfg.M
    L_B = a.block_len or Lc
    n_kept = min(k, n)
    bf = torch.bfloat16
    is_bf16 = cfg.dtype == "bf16"

    def to_dev(arr, bf16=False):
        t = torch.from_numpy(np.ascontiguousarray(arr)).to(dev)
        return t.to(bf) if bf16 else t

    # ---- inputs: one generated layer; further layers / buffer sets are token-rolled copies (same
    # distribution, different addresses) so that no step re-reads what the previous one left in cache
    t0 = time.time()
    d = wl.make_layer_inputs(cfg, structure=a.structure)
    # the tiny config is generated in fp32: Q/K/V are rounded to bf16 once at the boundary, features stay fp32
    kvq = {x: (d[x] if is_bf16 else wl.round_to_bf16(d[x])) for x in ("K_cache", "V_cache", "Q", "K_chunk", "V_chunk")}
    base = dict(
        X=to_dev(np.concatenate([d["X_cache"], d["X_chunk"]]), is_bf16),
        K=to_dev(kvq["K_cache"], True), V=to_dev(kvq["V_cache"], True),
        Q=to_dev(kvq["Q"], True), Kn=to_dev(kvq["K_chunk"], True), Vn=to_dev(kvq["V_chunk"], True),
    )
    W1 = to_dev(d["W1"], is_bf16)
    W2, b1, b2 = to_dev(d["W2"]), None, None
    paper_head = a.head == "paper"
    n_seg = 3 if paper_head else 1
    if paper_head:
        # App. A "S-MLP": the head reads [Q | K | V] of the final layer (3 H features), 1024 hidden units, 12 outputs
        # averaged.  Segments two and three are token-rolled copies of the generated features.
        M = 1024
        hw = wl.make_head_weights(wl.scaled(cfg, M=M, n_out=12), np.random.Generator(np.random.PCG64(wl.BASE_SEED + 77)),
                                  F=3 * H, bias=True)
        W1, b1, W2, b2 = to_dev(hw[0], True), to_dev(hw[1]), to_dev(hw[2]), to_dev(hw[3])

    def feature_segments(X):
        if not paper_head:
            return (X[:n],), (X[n:],)
        segs = [X, torch.cat([torch.roll(X[:n], 311, 0), torch.roll(X[n:], 311, 0)]),
                torch.cat([torch.roll(X[:n], 733, 0), torch.roll(X[n:], 733, 0)])]
        return tuple(t[:n] for t in segs), tuple(t[n:] for t in segs)
    n_sets = max(1, a.sets) if n_layers == 1 else 1
    fp8 = a.kv == "fp8"
    kvb = 1 if fp8 else 2
    kv_args = dict(kv_dtype=B.PAFU_FP8_E4M3, k_scale_log2=FP8_SCALES[0], v_scale_log2=FP8_SCALES[1]) if fp8 else {}
    sets = []
    for s in range(n_sets * n_layers):
        if s == 0:
            cur = dict(base)
        else:
            sh = 977 * s
            cur = dict(X=torch.cat([torch.roll(base["X"][:n], sh, 0), torch.roll(base["X"][n:], sh, 0)]),
                       K=torch.roll(base["K"], sh, 0), V=torch.roll(base["V"], sh, 0),
                       Q=torch.roll(base["Q"], sh, 0), Kn=torch.roll(base["Kn"], sh, 0),
                       Vn=torch.roll(base["Vn"], sh, 0))
        cur.update(scores=torch.empty(n + Lc, device=dev), ids=torch.empty(max(n_kept, 1), dtype=torch.int32, device=dev),
                   SL_out=torch.empty(max(n_kept, 1), device=dev), O=torch.empty(Lc, N, D, device=dev, dtype=bf))
        if fp8:     # the cache arrives as codes; the output slab also takes the quantised chunk rows
            Kq = torch.empty(n, N * D, dtype=torch.uint8, device=dev)
            Vq = torch.empty_like(Kq)
            B.pafu_quantize_kv(cur["K"], cur["V"], FP8_SCALES[0], FP8_SCALES[1], Kq, Vq)
            cur.update(K=Kq, V=Vq, K_out=torch.empty(n_kept + Lc, N * D, device=dev, dtype=torch.uint8),
                       V_out=torch.empty(n_kept + Lc, N * D, device=dev, dtype=torch.uint8))
        else:
            cur.update(K_out=torch.empty(max(n_kept, 1), N, D, device=dev, dtype=bf),
                       V_out=torch.empty(max(n_kept, 1), N, D, device=dev, dtype=bf))
        cur["x_cache"], cur["x_chunk"] = feature_segments(cur["X"])
        cur["x_all"] = tuple(torch.cat([c_, n_]) for c_, n_ in zip(cur["x_cache"], cur["x_chunk"])) if paper_head \
            else (cur["X"],)
        # scoring part (the output-averaged second layer) + the attention launch's partial-result slots; the layers
        # of a multi-layer step share one
        cur["ws"] = torch.empty((M + 64) * 4 + B.pafu_attention_workspace_bytes(Lc, N, D) + 512, dtype=torch.uint8,
                                device=dev) if (s == 0 or n_layers == 1) else sets[0]["ws"]
        cur["args"] = B.make_step_args(B.PAFU_MODE_SINGLE, N, D, n, Lc, k, L_B, cur["x_cache"], cur["x_chunk"], W1, b1,
                                       W2, b2, cur["K"], cur["V"], None, cur["Q"], cur["Kn"], cur["Vn"], cur["scores"],
                                       cur["ids"], cur["K_out"], cur["V_out"], cur["SL_out"], cur["O"],
                                       workspace=cur["ws"], n_pinned=a.pinned, **kv_args)
        sets.append(cur)
    torch.cuda.synchronize()
    gen_s = time.time() - t0
    shared = a.shared_index and n_layers > 1
    idx_layer = n_layers - 1

    def run_step(i):
        if n_layers == 1:
            B.pafu_step(sets[i % n_sets]["args"])
        elif shared:
            B.pafu_step_layers_shared([s["args"] for s in sets], idx_layer)
        else:
            B.pafu_step_layers([s["args"] for s in sets])

    run_step_eager = run_step
    if a.graph:
        # the library enqueues kernels only, so a step captures as it stands; one graph per rotated input set
        run_step_eager(0)
        torch.cuda.synchronize()
        graphs = []
        for i in range(n_sets if n_layers == 1 else 1):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                run_step_eager(i)
            graphs.append(g)
        torch.cuda.synchronize()

        def run_step(i):
            graphs[i % len(graphs)].replay()

    def timed_window(warmup, steps):
        """warmup untimed steps, then `steps` whole steps between two events with nothing else on the stream."""
        for i in range(warmup):
            run_step(i)
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        for i in range(steps):
            run_step(i)
        ev1.record()
        torch.cuda.synchronize()
        return ev0.elapsed_time(ev1) / steps, (time.perf_counter() - t_start) * 1e3 / steps

    # ---- the first window after the chip sat idle behind the host-side input generation: W warm-up steps, K timed.
    # A step is so short that W + K of them end before the power management has settled the clock, so this window
    # is reported (first_window_ms_per_step) but is not the headline.
    first_ms, _ = timed_window(a.warmup, a.steps)

    # ---- sustained: at least --sustained-s seconds of steps launched back to back (the chip's power management
    # averages over a longer window than K steps); it also brings the clock to where a serving loop runs
    sustained = None
    if a.sustained_s > 0:
        n_sus = max(a.steps, int(a.sustained_s * 1e3 / first_ms) + 1)
        s0, s1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s0.record()
        for i in range(n_sus):
            run_step(i)
        s1.record()
        torch.cuda.synchronize()
        sustained = {"ms_per_step": s0.elapsed_time(s1) / n_sus, "steps": n_sus}

    # ---- whole-step timing: the headline.  W warm-up steps, then K steps between two events, nothing else on the
    # stream, at the settled clock.
    ms_per_step, wall_ms = timed_window(a.warmup, a.steps)

    # ---- the same steps again with the library's stage events attached: every kernel of every step is bracketed by
    # HIP events that pafu_step itself records on the launch stream (no host round trip between the stages).
    recorded = []
    for i in range(a.steps):
        layers = sets if n_layers > 1 else [sets[i % n_sets]]
        step_evs = []
        for s_ in layers:
            sev = new_events(torch, 5)
            B.set_stage_events(s_["args"], sev)
            step_evs.append(sev)
        eva, evb = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        eva.record()
        run_step_eager(i)
        evb.record()
        recorded.append((eva, evb, step_evs))
    torch.cuda.synchronize()
    for s_ in sets:
        B.set_stage_events(s_["args"], [None] * 5)
    ms_with_events = float(np.mean([x.elapsed_time(y) for x, y, _ in recorded]))
    attn_ms = [sev[3].elapsed_time(sev[4]) for _, _, se in recorded for sev in se]
    if n_layers == 1:
        score_ms = [se[0][0].elapsed_time(se[0][1]) for _, _, se in recorded]
        select_ms = [se[0][1].elapsed_time(se[0][2]) for _, _, se in recorded]
        compact_ms = [se[0][2].elapsed_time(se[0][3]) for _, _, se in recorded]
        select_note = None
    else:
        # Multi-layer steps: all scoring first, then ONE selection launch for up to 32 layers, then ONE compaction
        # launch for up to 32 layers, then attention layer by layer.  The library records "after selection" once per
        # step (on layer 0, or on the index layer); compaction = from there to the start of layer 0's attention,
        # shared out over the layers.
        scoring = [idx_layer] if shared else list(range(n_layers))
        sel_layer = idx_layer if shared else 0
        score_ms = [se[l][0].elapsed_time(se[l][1]) for _, _, se in recorded for l in scoring]
        select_ms = [se[scoring[-1]][1].elapsed_time(se[sel_layer][2]) for _, _, se in recorded]
        compact_ms = [se[sel_layer][2].elapsed_time(se[0][3]) / n_layers for _, _, se in recorded]
        select_note = "one launch per step for %s; compaction: one launch for all %d layers, time per layer" % (
            "the index layer" if shared else "all %d layers" % n_layers, n_layers)
    avg = {"score": float(np.mean(score_ms)), "select": float(np.mean(select_ms)), "compact": float(np.mean(compact_ms)),
           "attention": float(np.mean(attn_ms))}
    mn = {"score": float(np.min(score_ms)), "select": float(np.min(select_ms)), "compact": float(np.min(compact_ms)),
          "attention": float(np.min(attn_ms))}

    # ---- the floor of a stage between two events on this stream: an empty kernel
    probe = [torch.cuda.Event(enable_timing=True) for _ in range(41)]
    probe[0].record()
    for i in range(40):
        B.pafu_launch_probe()
        probe[i + 1].record()
    torch.cuda.synchronize()
    empty_ms = float(np.median(event_pair_ms(probe)))

    # ---- algorithmic work per launch (one layer)
    T = n + Lc
    eb = 2 if is_bf16 else 4
    visible_pairs = Lc * n_kept + sum(min(Lc, (i // L_B + 1) * L_B) for i in range(Lc))
    attn_flops = 4.0 * visible_pairs * D * N
    F_in = n_seg * H
    bytes_score = T * F_in * eb + M * F_in * eb + T * 4
    bytes_select = n * 4 + n_kept * 4
    bytes_compact = 2 * (2 * n_kept * N * D * kvb) + 2 * n_kept * 4 + n_kept * 4
    attn_tflops = attn_flops / (avg["attention"] * 1e-3) / 1e12
    stages = {
        "score": {"ms": avg["score"], "min_ms": mn["score"], "GB/s": bytes_score / avg["score"] / 1e6,
                  "frac_hbm": bytes_score / avg["score"] / 1e6 / PEAK_HBM_GBS,
                  "TFLOP/s": 2.0 * T * F_in * M / avg["score"] / 1e9},
        "select": {"ms": avg["select"], "min_ms": mn["select"],
                   "GB/s": bytes_select * (1 if n_layers == 1 or shared else n_layers) / max(avg["select"], 1e-9) / 1e6,
                   "empty_kernel_ms": empty_ms, "x_empty_kernel": avg["select"] / empty_ms if empty_ms > 0 else None,
                   "note": select_note},
        "compact": {"ms": avg["compact"], "min_ms": mn["compact"], "GB/s": bytes_compact / avg["compact"] / 1e6,
                    "frac_hbm": bytes_compact / avg["compact"] / 1e6 / PEAK_HBM_GBS, "salient": a.structure,
                    "bytes": bytes_compact,
                    "note": "includes quantising the chunk's K/V into the slab" if fp8 else None},
        "attention": {"ms": avg["attention"], "min_ms": mn["attention"], "TFLOP/s": attn_tflops,
                      "frac_mfma": attn_tflops / PEAK_BF16_TFLOPS},
    }
    # cross-check of the event-measured attention duration: the kernels of a step run back to back, so inside the
    # plain timed steps (no stage events) the attention launch lasts the step minus the three short stages
    n_scoring = 1 if (shared or n_layers == 1) else n_layers
    inferred = (ms_per_step - avg["score"] * n_scoring - avg["select"]) / n_layers - avg["compact"]
    traffic = ATTENTION_TRAFFIC.get((a.workload, L_B == Lc))
    roofline = {"kernel": "chunk_attention_kernel", "bound": "mfma", "achieved": attn_tflops,
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": attn_tflops / PEAK_BF16_TFLOPS,
                "traffic": traffic[0] if traffic else None,
                "traffic_source": (traffic[1] + " (separate rocprofv3 --pmc run, not re-measured here)") if traffic else None,
                "flops_per_launch": attn_flops, "avg_launch_ms": avg["attention"], "launches_timed": len(attn_ms),
                "how": "hipEventRecord before and after the attention launch inside the step entry point, on the launch "
                       "stream, over %d whole steps" % a.steps,
                "ms_per_step_with_stage_events": ms_with_events,
                "step_minus_short_stages_ms": inferred}

    # ---- CPU leg: the oracle as it stands on a bounded sample of the same workload, timed; its outputs are also the
    # parity reference for the device buffers of the last step that ran on input set 0 (teacher-forced like the tests:
    # the oracle selects on the device's fp32 scores, so indices and cache must match bit for bit)
    cpu, parity, parity_ok = None, None, True
    if not a.no_cpu_baseline and a.workload in ("C1", "C0", "C2", "C4") and not paper_head:
        from oracle import pafu_oracle as orc
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = len(os.sched_getaffinity(0))
        s0 = sets[0]
        got_scores = s0["scores"].cpu().numpy()
        # about 10-30 s of CPU work: every query row at the Wan-1.3B layer, a strided sample above that
        n_rows = Lc if Lc * (n_kept + Lc) * N <= 1.3e9 else max(96, int(1.3e9 / ((n_kept + Lc) * N)))
        rows = np.arange(Lc) if n_rows >= Lc else np.unique(np.linspace(0, Lc - 1, n_rows).astype(np.int64))
        # with shared indices layer 0's cache follows ANOTHER layer's scores: then the oracle is only timed, on its own
        cpu_only = shared
        c0 = time.perf_counter()
        s_ref = orc.smlp_score(np.concatenate([d["X_cache"], d["X_chunk"]]), d["W1"], None, d["W2"], None)
        c1 = time.perf_counter()
        sel_scores = s_ref[:n].astype(np.float32) if cpu_only else got_scores[:n]
        ids_ref = orc.select_topk(sel_scores, k, a.pinned)
        c2 = time.perf_counter()
        if fp8:     # the oracle carries codes through selection and compaction and attends on the dequantised values
            ek, ev = FP8_SCALES
            qz = lambda x_, e_: orc.quantise_e4m3(x_.reshape(x_.shape[0], N * D), e_)
            dq = lambda c_, e_: orc.dequantise_e4m3(c_, e_).reshape(c_.shape[0], N, D)
            Kc_codes, Vc_codes = qz(kvq["K_cache"], ek), qz(kvq["V_cache"], ev)
            Kn_codes, Vn_codes = qz(kvq["K_chunk"], ek), qz(kvq["V_chunk"], ev)
            c2 = time.perf_counter()        # (quantising the inputs is set-up, not part of the step)
            Kk, Vk, SLk = orc.compact_kv(Kc_codes, Vc_codes, sel_scores, ids_ref)
            c3 = time.perf_counter()
            O_ref = orc.chunk_attention(kvq["Q"], dq(Kk, ek), dq(Vk, ev), dq(Kn_codes, ek), dq(Vn_codes, ev),
                                        block_len=L_B, rows=rows)
        else:
            Kk, Vk, SLk = orc.compact_kv(kvq["K_cache"], kvq["V_cache"], sel_scores, ids_ref)
            c3 = time.perf_counter()
            O_ref = orc.chunk_attention(kvq["Q"], Kk, Vk, kvq["K_chunk"], kvq["V_chunk"], block_len=L_B, rows=rows)
        c4 = time.perf_counter()
        attn_full_ms = (c4 - c3) * 1e3 * (Lc / len(rows))
        total = (c1 - c0) * 1e3 + (c2 - c1) * 1e3 + (c3 - c2) * 1e3 + attn_full_ms
        cpu = {"value": total * n_layers, "unit": "ms per step (attention extrapolated from the sampled rows)",
               "cores": int(cores), "kind": "oracle",
               "sample": "full score/select/compact of one layer; attention on %d of %d query rows x all heads, "
                         "scaled by %d/%d%s" % (len(rows), Lc, Lc, len(rows), "; x30 layers" if n_layers > 1 else ""),
               "stages_ms": {"score": (c1 - c0) * 1e3, "select": (c2 - c1) * 1e3, "compact": (c3 - c2) * 1e3,
                             "attention_extrapolated": attn_full_ms}}
        if not cpu_only:
            f32 = lambda t_: t_.float().cpu().numpy()
            got_ids = s0["ids"].cpu().numpy()[:n_kept]
            got_O = f32(s0["O"]).astype(np.float64)[rows]
            if fp8:
                gK, gV = s0["K_out"].cpu().numpy(), s0["V_out"].cpu().numpy()
                cache_mism = int((gK != np.concatenate([Kk, Kn_codes])).sum() + (gV != np.concatenate([Vk, Vn_codes])).sum())
            else:
                cache_mism = 2 * int((f32(s0["K_out"])[:n_kept] != Kk).sum() + (f32(s0["V_out"])[:n_kept] != Vk).sum())
            cache_mism += 4 * int((s0["SL_out"].cpu().numpy()[:n_kept] != SLk).sum())
            parity = {
                "score_max_abs": float(np.abs(got_scores - s_ref).max()),
                "id_mismatches": int((got_ids != ids_ref).sum()),
                "cache_byte_mismatches": cache_mism,
                "attn_max_abs": float(np.abs(got_O - O_ref).max()),
                "attn_rel_fro": float(np.linalg.norm(got_O - O_ref) / np.linalg.norm(O_ref)),
                "attn_rows_checked": int(len(rows)),
                "how": "buffers of input set 0 after the last step (layer 0 of a multi-layer step); the oracle "
                       "selects on the device's fp32 scores",
                "tolerances": dict(TOL, id_mismatches=0, cache_byte_mismatches=0),
            }
            parity_ok = (parity["score_max_abs"] < TOL["score_max_abs"] and parity["id_mismatches"] == 0
                         and parity["cache_byte_mismatches"] == 0 and parity["attn_max_abs"] < TOL["attn_max_abs"]
                         and parity["attn_rel_fro"] < TOL["attn_rel_fro"])
            parity["ok"] = bool(parity_ok)

    out = {
        "metric": METRIC,
        "value": ms_per_step, "unit": "ms", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if is_bf16 else "f32", "data": "synthetic",
        "config": {"workload": "%s: %d layer(s), %d heads x %d, cache %d tokens, chunk %d queries, budget %d, "
                               "S-MLP %d->%d->%d, L_B=%d, salient=%s" % (a.workload, n_layers, N, D, n, Lc, k, F_in, M,
                                                                          12 if paper_head else cfg.n_out, L_B,
                                                                          a.structure),
                   "layers": n_layers, "input_sets": n_sets,
                   "indices": "shared (last layer's head)" if shared else "per layer",
                   "n_pinned": a.pinned, "kv_storage": a.kv},
        "wall_ms_per_step": wall_ms,
        "launch": "HIP graph replay" if a.graph else "eager",
        "first_window_ms_per_step": first_ms,
        "sustained_ms_per_step": sustained["ms_per_step"] if sustained else None,
        "sustained_steps": sustained["steps"] if sustained else None,
        "stages": stages, "roofline": roofline, "parity": parity, "cpu_baseline": cpu,
        "input_gen_s": gen_s,
    }
    print(json.dumps(out))
    if not parity_ok:
        print("bench.py: parity against the oracle is out of tolerance: %s" % json.dumps(parity), file=sys.stderr)
        sys.exit(1)


if __name__ == "__main__":
    main()
