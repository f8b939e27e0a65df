"""Tensors whose rows lie more than 4 GiB apart: every stage addresses rows as 64-bit base + row * stride, and a
32-bit slip would read the wrong row (the values differ per row, so parity against the oracle catches it).
Padded slabs stand in for what a 30-layer cache laid out token-major looks like to one layer."""
import numpy as np
import pytest
import torch

from oracle import pafu_oracle as orc
from paper_2601_21896_amd import binding as B
from paper_2601_21896_amd import workloads as wl
from tests.gpu_util import ATTN_MAX_ABS, ATTN_REL_FRO, DEV, SCORE_MAX_ABS, attn_errors, dev, host

pytestmark = pytest.mark.gpu

N, D = 2, 128
ROW = N * D
LD = 1 << 17            # elements between rows: 256 KiB in bf16
N_CACHE = 18000         # the last row starts 4.72e9 bytes behind the first
LC = 200


def _padded(rows, values):
    """[rows, ROW] float32 values -> bf16 slab with LD elements between rows, and the strided [rows, ROW] view."""
    slab = torch.zeros(rows * LD, dtype=torch.bfloat16, device=DEV)
    view = slab.view(rows, LD)[:, :ROW]
    view.copy_(torch.from_numpy(values).to(DEV))
    return slab, view


@pytest.fixture(scope="module")
def big():
    cfg = wl.scaled(wl.C1, N=N, D=D, M=256, frame_tokens=LC, chunk_frames=1, cache_frames=N_CACHE // LC, k=4000)
    assert cfg.n == N_CACHE and (N_CACHE - 1) * LD * 2 > 1 << 32
    d = wl.make_layer_inputs(cfg)
    keep = []
    out = dict(cfg=cfg, d=d, keep=keep)
    for name in ("X_cache", "K_cache", "V_cache"):
        slab, view = _padded(N_CACHE, d[name].reshape(N_CACHE, ROW))
        keep.append(slab)
        out[name] = view
    yield out
    keep.clear()
    torch.cuda.empty_cache()


def test_step_reads_features_and_cache_rows_beyond_4_gib(big):
    cfg, d = big["cfg"], big["d"]
    k = cfg.k
    slab_x, x_chunk = _padded(LC, d["X_chunk"])                   # same row stride as the cache features
    rb = wl.round_to_bf16
    kv = {x: rb(d[x]) for x in ("K_cache", "V_cache", "Q", "K_chunk", "V_chunk")}
    scores = torch.empty(N_CACHE + LC, device=DEV)
    ids = torch.full((k,), -1, dtype=torch.int32, device=DEV)
    K_out = torch.zeros(k, N, D, device=DEV, dtype=torch.bfloat16)
    V_out = torch.zeros_like(K_out)
    SL_out = torch.zeros(k, device=DEV)
    O = torch.empty(LC, N, D, device=DEV, dtype=torch.bfloat16)
    w = [dev(d["W1"], "bf16"), dev(d["b1"]), dev(d["W2"]), dev(d["b2"])]
    t = [dev(kv["Q"], "bf16"), dev(kv["K_chunk"], "bf16"), dev(kv["V_chunk"], "bf16")]
    args = B.make_step_args(B.PAFU_MODE_SINGLE, N, D, N_CACHE, LC, k, LC, big["X_cache"], x_chunk, w[0], w[1], w[2], w[3],
                            big["K_cache"], big["V_cache"], None, t[0], t[1], t[2], scores, ids, K_out, V_out, SL_out, O)
    assert args.ld_x == LD and args.ld_cache == LD
    B.pafu_step(args)
    torch.cuda.synchronize()
    got_s = host(scores)
    ref = orc.step_single(d["X_cache"], d["X_chunk"], d["W1"], d["b1"], d["W2"], d["b2"], kv["K_cache"], kv["V_cache"],
                          kv["Q"], kv["K_chunk"], kv["V_chunk"], k, LC, forced_scores_f32=got_s)
    assert np.abs(got_s - ref["scores"]).max() < SCORE_MAX_ABS
    # retained rows on both sides of the 4 GiB line
    assert int(ref["ids"].max()) * LD * 2 > 1 << 32 and int(ref["ids"].min()) * LD * 2 < 1 << 32
    assert np.array_equal(host(ids), ref["ids"])
    assert np.array_equal(host(K_out), ref["K_kept"]) and np.array_equal(host(V_out), ref["V_kept"])
    assert np.array_equal(host(SL_out), ref["SL_kept"])
    max_abs, rel = attn_errors(host(O), ref["O"])
    assert max_abs < ATTN_MAX_ABS and rel < ATTN_REL_FRO, (max_abs, rel)


def test_attention_reads_a_cache_whose_rows_lie_beyond_4_gib(big):
    d = big["d"]
    rb = wl.round_to_bf16
    Q, Kn, Vn = (dev(rb(d[x]), "bf16") for x in ("Q", "K_chunk", "V_chunk"))
    O = torch.empty(LC, N, D, device=DEV, dtype=torch.float32)
    Kc = big["K_cache"].view(N_CACHE, N, D)
    Vc = big["V_cache"].view(N_CACHE, N, D)
    assert Kc.stride(0) == LD
    B.pafu_chunk_attention(Q, Kc, Vc, N_CACHE, Kn, Vn, LC, O)
    torch.cuda.synchronize()
    want = orc.chunk_attention(rb(d["Q"]), rb(d["K_cache"]), rb(d["V_cache"]), rb(d["K_chunk"]), rb(d["V_chunk"]), LC)
    max_abs, rel = attn_errors(host(O), want)
    assert max_abs < ATTN_MAX_ABS and rel < ATTN_REL_FRO, (max_abs, rel)
    # the index-based variant addresses cache rows with 32-bit offsets and says so instead of reading a wrong row
    ids = torch.arange(N_CACHE, dtype=torch.int32, device=DEV)
    with pytest.raises(B.PafuError) as e:
        B.pafu_chunk_attention_gather(Q, Kc, Vc, ids, N_CACHE, Kn, Vn, LC, O)
    assert e.value.status == -2
