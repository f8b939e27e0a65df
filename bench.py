#!/usr/bin/env python3
"""Benchmark of the PaFu-KV chunk step on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input: score all cached and
chunk tokens with the S-MLP, select the top-k cached tokens, compact K/V/SL, and attend from the chunk's
queries over the retained cache plus the chunk (pafu_step, SINGLE mode).  The default workload is the
Wan-1.3B-shaped single layer in bf16 (12 heads x 128, 32760 cached + 4680 chunk tokens, budget 16380).

Prints ONE JSON line: ms per step (inputs resident in HBM), a per-stage breakdown measured with events
on the launch stream, the roofline of the dominant kernel (attention, dense bf16 MFMA), and the fp64
oracle timed on this machine's host cores on a bounded sample of the same workload.
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

# HBM bytes per attention launch from rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE, scaled by a copy kernel);
# filled from the summaries under profiles/ (None = not measured for that workload).
MEASURED_ATTENTION_TRAFFIC_BYTES = {
    # profiles/step_C1_hbm_traffic_pmc.md: 107168.7 KiB x 1.98 fetched + 14042.1 KiB written
    ("C1", True): int((107168.7 * 1.98 + 14042.1) * 1024),
}


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


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="C1", choices=["C1", "C4", "C2", "C0", "C3", "SSE"])
    ap.add_argument("--budget", type=int, default=0, help="C3 only: cache budget k in tokens (default 8 frames = 12480)")
    ap.add_argument("--block-len", type=int, default=0, help="L_B (0 = chunk length, the paper's setting)")
    ap.add_argument("--structure", default="uniform", choices=["uniform", "coherent"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sets", type=int, default=3, help="input buffer sets rotated between steps")
    ap.add_argument("--shared-index", action="store_true",
                    help="C2 only: score + select once on the last layer, every layer reuses its indices (Sec. 3.3)")
    ap.add_argument("--head", default="benchmark", choices=["benchmark", "paper"],
                    help="S-MLP widths: the benchmark's (F = H, M from the config, 1 output) or App. A's "
                         "([Q|K|V] = 3H inputs, 1024 hidden, 12 outputs averaged)")
    ap.add_argument("--pinned", type=int, default=0, help="frame sink: cached tokens [0, pinned) are never evicted")
    return ap.parse_args()


def rollout(a, torch, np, B, wl):
    """C3: 60 sequential chunks at the Wan-1.3B layer shapes, fixed budget; steady-state ms per step."""
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
    slabs = [dict(K=torch.zeros(cap, N, D, device=dev, dtype=bf), V=torch.zeros(cap, N, D, device=dev, dtype=bf),
                  SL=torch.zeros(cap, device=dev)) for _ in range(2)]
    ids = torch.empty(max(k, 1), dtype=torch.int32, device=dev)
    O = torch.empty(Lc, N, D, device=dev, dtype=bf)
    times, sizes = [], []
    for rep in range(2):    # first pass warms up, second is timed
        n, cur = 0, 0
        times, sizes = [], []
        for step in range(n_chunks):
            c = pool[step % len(pool)]
            src, dst = slabs[cur], slabs[1 - cur]
            args = B.make_step_args(B.PAFU_MODE_ROLLOUT, N, D, n, Lc, k, Lc, None, c["X"], W1, None, W2, None, src["K"],
                                    src["V"], src["SL"], c["Q"], c["K"], c["V"], None, ids, dst["K"], dst["V"],
                                    dst["SL"], O, n_pinned=a.pinned)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            B.pafu_step(args)
            e1.record()
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1))
            n = min(k, n) + Lc
            sizes.append(n)
            cur = 1 - cur
    steady = times[5:]
    n_steady = sizes[-1]
    n_kept = min(k, n_steady)
    flops = 4.0 * Lc * (n_kept + Lc) * D * N
    peak_cache = 2 * (cap * N * D * 2 * 2 + cap * 4)
    out = {
        "metric": "ms per AR chunk step (score+select+compact+attn), MFMA util and HBM GB/s", "value": float(np.median(steady)), "unit": "ms",
        "n_gpus": 1, "steps": len(steady), "warmup": n_chunks + 5, "ms_per_step": float(np.median(steady)),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "C3: %d-chunk rollout, 12 heads x 128, chunk %d queries, budget %d tokens, steady cache "
                               "%d tokens, S-MLP %d->%d->1" % (n_chunks, Lc, k, n_steady, H, M)},
        "min_ms": float(np.min(steady)), "first_steps_ms": [float(x) for x in times[:5]], "cache_sizes_first_steps": sizes[:6],
        "peak_cache_bytes": peak_cache,
        "roofline": {"kernel": "chunk_attention_kernel", "bound": "mfma", "achieved": None, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": None, "traffic": None, "flops_per_launch": flops,
                     "note": "whole-step time only; per-kernel times come from the rocprofv3 summary"},
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
    B.library()
    dev = "cuda:0"
    torch.cuda.set_device(0)

    if a.workload == "C3":
        rollout(a, torch, np, B, wl)
        return
    if a.workload == "SSE":
        sse(a, torch, np, B, wl)
        return
    n_layers = wl.C2_LAYERS if a.workload == "C2" else 1
    cfg = wl.C1 if a.workload == "C2" else wl.CONFIGS[a.workload]
    N, D, n, Lc, k, H, M = cfg.N, cfg.D, cfg.n, cfg.Lc, cfg.k, cfg.H, cfg.M
    L_B = a.block_len or Lc
    n_kept = min(k, n)
    bf = torch.bfloat16
    x_dt = bf if cfg.dtype == "bf16" else torch.float32
    q = "bf16" if cfg.dtype == "bf16" else None

    def to_dev(arr, bf16=False):
        t = torch.from_numpy(np.ascontiguousarray(arr)).to(dev)
        return t.to(bf) if bf16 else t

    # ---- inputs: one generated layer; further layers / buffer sets are token-rolled copies (same
    # distribution, different addresses) so that no step re-reads what the previous one left in cache
    t0 = time.time()
    d = wl.make_layer_inputs(cfg, structure=a.structure)
    base = dict(
        X=to_dev(np.concatenate([d["X_cache"], d["X_chunk"]]), cfg.dtype == "bf16"),
        K=to_dev(d["K_cache"], True), V=to_dev(d["V_cache"], True),
        Q=to_dev(d["Q"], True), Kn=to_dev(d["K_chunk"], True), Vn=to_dev(d["V_chunk"], True),
    )
    W1 = to_dev(d["W1"], cfg.dtype == "bf16")
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
    sets = []
    for s in range(n_sets * n_layers):
        if s == 0:
            cur = base
        else:
            sh = 977 * s
            cur = dict(X=torch.cat([torch.roll(base["X"][:n], sh, 0), torch.roll(base["X"][n:], sh, 0)]),
                       K=torch.roll(base["K"], sh, 0), V=torch.roll(base["V"], sh, 0),
                       Q=torch.roll(base["Q"], sh, 0), Kn=torch.roll(base["Kn"], sh, 0),
                       Vn=torch.roll(base["Vn"], sh, 0))
        cur.update(scores=torch.empty(n + Lc, device=dev), ids=torch.empty(max(n_kept, 1), dtype=torch.int32, device=dev),
                   K_out=torch.empty(max(n_kept, 1), N, D, device=dev, dtype=bf),
                   V_out=torch.empty(max(n_kept, 1), N, D, device=dev, dtype=bf),
                   SL_out=torch.empty(max(n_kept, 1), device=dev), O=torch.empty(Lc, N, D, device=dev, dtype=bf))
        cur["x_cache"], cur["x_chunk"] = feature_segments(cur["X"])
        cur["x_all"] = tuple(torch.cat([c_, n_]) for c_, n_ in zip(cur["x_cache"], cur["x_chunk"])) if paper_head \
            else (cur["X"],)
        cur["ws"] = torch.empty(M + 64, device=dev)
        cur["args"] = B.make_step_args(B.PAFU_MODE_SINGLE, N, D, n, Lc, k, L_B, cur["x_cache"], cur["x_chunk"], W1, b1,
                                       W2, b2, cur["K"], cur["V"], None, cur["Q"], cur["Kn"], cur["Vn"], cur["scores"],
                                       cur["ids"], cur["K_out"], cur["V_out"], cur["SL_out"], cur["O"],
                                       workspace=cur["ws"], n_pinned=a.pinned)
        sets.append(cur)
    torch.cuda.synchronize()
    gen_s = time.time() - t0

    def run_step(i):
        if n_layers == 1:
            B.pafu_step(sets[i % n_sets]["args"])
        elif a.shared_index:
            B.pafu_step_layers_shared([s["args"] for s in sets], n_layers - 1)
        else:
            B.pafu_step_layers([s["args"] for s in sets])

    # ---- whole-step timing
    for i in range(a.warmup):
        run_step(i)
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for i in range(a.steps):
        run_step(i)
    ev1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t_start) * 1e3 / a.steps
    ms_per_step = ev0.elapsed_time(ev1) / a.steps

    # ---- per-stage timing (same buffers, stage entry points, events on the launch stream)
    stage_names = ("score", "select", "compact", "attention")
    stage_ms = {s: [] for s in stage_names}
    reps = max(a.steps, 10) if n_layers == 1 else 2

    def stage_calls(cur):
        return (
            lambda: B.pafu_score(cur["x_all"], W1, b1, W2, b2, cur["scores"], workspace=cur["ws"]),
            lambda: B.pafu_select_topk(cur["scores"], k, cur["ids"], n=n),
            lambda: B.pafu_compact_kv(cur["K"], cur["V"], cur["scores"], cur["ids"], n_kept, cur["K_out"], cur["V_out"],
                                      cur["SL_out"]),
            lambda: B.pafu_chunk_attention(cur["Q"], cur["K_out"], cur["V_out"], n_kept, cur["Kn"], cur["Vn"], L_B,
                                           cur["O"]),
        )

    # The repetitions are enqueued back to back, like the timed steps above, and read after one synchronisation at
    # the end, so that the stage durations are taken at the same sustained clocks as the whole-step figure.
    recorded = []
    for i in range(reps + 2):
        for cur in (sets if n_layers > 1 else [sets[i % n_sets]]):
            evs = [torch.cuda.Event(enable_timing=True) for _ in range(5)]
            calls = stage_calls(cur)
            evs[0].record()
            for j, c in enumerate(calls):
                c()
                evs[j + 1].record()
            if i >= 2:
                recorded.append(evs)
    torch.cuda.synchronize()
    for evs in recorded:
        for j, s in enumerate(stage_names):
            stage_ms[s].append(evs[j].elapsed_time(evs[j + 1]))
    avg = {s: float(np.mean(v)) for s, v in stage_ms.items()}
    mn = {s: float(np.min(v)) for s, v in stage_ms.items()}

    # ---- algorithmic work per launch (one layer)
    T = n + Lc
    eb = 2 if cfg.dtype == "bf16" else 4
    visible_pairs = Lc * n_kept + sum(min(Lc, (i // L_B + 1) * L_B) for i in range(Lc))
    attn_flops = 4.0 * visible_pairs * D * N
    F_in = n_seg * H
    bytes_score = T * F_in * eb + M * F_in * eb + T * 4
    bytes_select = n * 4 + n_kept * 4
    bytes_compact = 2 * (2 * n_kept * N * D * 2) + 2 * n_kept * 4 + n_kept * 4
    attn_tflops = attn_flops / (avg["attention"] * 1e-3) / 1e12
    stages = {
        "score": {"ms": avg["score"], "min_ms": mn["score"], "GB/s": bytes_score / avg["score"] / 1e6,
                  "frac_hbm": bytes_score / avg["score"] / 1e6 / PEAK_HBM_GBS,
                  "TFLOP/s": 2.0 * T * F_in * M / avg["score"] / 1e9},
        "select": {"ms": avg["select"], "min_ms": mn["select"], "GB/s": bytes_select / avg["select"] / 1e6},
        "compact": {"ms": avg["compact"], "min_ms": mn["compact"], "GB/s": bytes_compact / avg["compact"] / 1e6,
                    "frac_hbm": bytes_compact / avg["compact"] / 1e6 / PEAK_HBM_GBS},
        "attention": {"ms": avg["attention"], "min_ms": mn["attention"], "TFLOP/s": attn_tflops,
                      "frac_mfma": attn_tflops / PEAK_BF16_TFLOPS},
    }
    # The kernels of a step run back to back (no gaps in the kernel trace), so the attention launch's duration inside
    # the timed whole steps is the step time minus the three short stages.  It is a few percent longer than the
    # duration between the stage events above, where the event records leave the chip short rests; the roofline
    # figure uses the in-step duration, which is also what the rocprofv3 average over the same command shows.
    # (a multi-layer step selects for up to 32 layers in one launch, one workgroup per layer; with shared indices it
    # scores and selects once for all layers).  Never report less than the duration between the stage events.
    shared = a.shared_index and n_layers > 1
    score_share = avg["score"] / n_layers if shared else avg["score"]
    select_share = avg["select"] / n_layers if shared else avg["select"] * ((n_layers + 31) // 32) / n_layers
    attn_in_step_ms = max(ms_per_step / n_layers - (score_share + select_share + avg["compact"]), avg["attention"])
    attn_in_step_tflops = attn_flops / (attn_in_step_ms * 1e-3) / 1e12
    roofline = {"kernel": "chunk_attention_kernel", "bound": "mfma", "achieved": attn_in_step_tflops,
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": attn_in_step_tflops / PEAK_BF16_TFLOPS,
                "traffic": MEASURED_ATTENTION_TRAFFIC_BYTES.get((a.workload, L_B == Lc)),
                "flops_per_launch": attn_flops, "avg_launch_ms": attn_in_step_ms,
                "avg_launch_ms_between_stage_events": avg["attention"]}

    # ---- CPU baseline: the oracle as it stands, bounded sample of the same workload
    cpu = None
    if not a.no_cpu_baseline and a.workload in ("C1", "C0", "C2") and not paper_head:
        from oracle import pafu_oracle as orc
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = len(os.sched_getaffinity(0))
        # about 10-30 s of CPU work: every query row at the Wan-1.3B layer, a strided sample above that
        n_rows = Lc if Lc * (n_kept + Lc) * N <= 1.3e9 else max(96, int(1.3e9 / ((n_kept + Lc) * N)))
        rows = np.arange(Lc) if n_rows >= Lc else np.unique(np.linspace(0, Lc - 1, n_rows).astype(np.int64))
        c0 = time.perf_counter()
        s_ref = orc.smlp_score(np.concatenate([d["X_cache"], d["X_chunk"]]), d["W1"], None, d["W2"], None)
        c1 = time.perf_counter()
        ids_ref = orc.select_topk(s_ref[:n].astype(np.float32), k)
        c2 = time.perf_counter()
        Kk, Vk, _ = orc.compact_kv(d["K_cache"], d["V_cache"], s_ref[:n].astype(np.float32), ids_ref)
        c3 = time.perf_counter()
        orc.chunk_attention(d["Q"], Kk, Vk, d["K_chunk"], d["V_chunk"], block_len=L_B, rows=rows)
        c4 = time.perf_counter()
        attn_full_ms = (c4 - c3) * 1e3 * (Lc / len(rows))
        total = (c1 - c0) * 1e3 + (c2 - c1) * 1e3 + (c3 - c2) * 1e3 + attn_full_ms
        cpu = {"value": total * n_layers, "unit": "ms per step (attention extrapolated from the sampled rows)",
               "cores": int(cores), "kind": "oracle",
               "sample": "full score/select/compact of one layer; attention on %d of %d query rows x all heads, "
                         "scaled by %d/%d%s" % (len(rows), Lc, Lc, len(rows), "; x30 layers" if n_layers > 1 else ""),
               "stages_ms": {"score": (c1 - c0) * 1e3, "select": (c2 - c1) * 1e3, "compact": (c3 - c2) * 1e3,
                             "attention_extrapolated": attn_full_ms}}

    out = {
        "metric": "ms per AR chunk step (score+select+compact+attn), MFMA util and HBM GB/s",
        "value": ms_per_step, "unit": "ms", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": "%s: %d layer(s), %d heads x %d, cache %d tokens, chunk %d queries, budget %d, "
                               "S-MLP %d->%d->%d, L_B=%d, salient=%s" % (a.workload, n_layers, N, D, n, Lc, k, F_in, M,
                                                                          12 if paper_head else cfg.n_out, L_B,
                                                                          a.structure),
                   "layers": n_layers, "input_sets": n_sets,
                   "indices": "shared (last layer's head)" if (a.shared_index and n_layers > 1) else "per layer",
                   "n_pinned": a.pinned},
        "wall_ms_per_step": wall_ms, "stages": stages, "roofline": roofline, "cpu_baseline": cpu,
        "input_gen_s": gen_s,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
