"""GPU parity of pafu_chunk_attention against the fp64 oracle (max-abs 2e-2, relative Frobenius 5e-3)."""
import numpy as np
import pytest
import torch

from oracle import pafu_oracle as orc
from paper_2601_21896_amd import binding as B
from paper_2601_21896_amd import workloads as wl
from tests.gpu_util import ATTN_MAX_ABS, ATTN_REL_FRO, DEV, attention_workspace, attn_errors, dev, host

pytestmark = pytest.mark.gpu


def _inputs(n, Lc, N, D, seed, q_gain=1.0):
    rng = np.random.Generator(np.random.PCG64(seed))
    c = rng.uniform(0.5, 2.0, size=(N * D,)).astype(np.float32)
    r = lambda rows, s=None: wl.round_to_bf16(
        (rng.standard_normal((rows, N * D), dtype=np.float32) * (1.0 if s is None else s[None, :]))).reshape(rows, N, D)
    Kc, Vc = r(n, c), r(n)
    Q = wl.round_to_bf16(r(Lc) * np.float32(q_gain))
    Kn, Vn = r(Lc, c), r(Lc)
    return Q, Kc, Vc, Kn, Vn


def _run(Q, Kc, Vc, Kn, Vn, L_B, out_dtype=torch.bfloat16, Lq=None, ws=None):
    Lq = Q.shape[0] if Lq is None else Lq
    N, D = Q.shape[1], Q.shape[2]
    n = Kc.shape[0]
    O = torch.full((Lq + 2, N, D), 55.0, device=DEV, dtype=out_dtype)
    dQ = dev(Q[:Lq], "bf16")
    dKc = dev(Kc, "bf16") if n else None
    dVc = dev(Vc, "bf16") if n else None
    B.pafu_chunk_attention(dQ, dKc, dVc, n, dev(Kn, "bf16"), dev(Vn, "bf16"), L_B, O[:Lq], workspace=ws)
    torch.cuda.synchronize()
    assert torch.all(O[Lq:] == 55.0)
    return host(O[:Lq])


@pytest.mark.parametrize("n,Lc,N,D,L_B", [
    (128, 64, 2, 64, 64),        # C0 shapes after budget 50%
    (128, 64, 2, 64, 16),
    (128, 64, 2, 64, 1),         # causal inside the chunk
    (0, 64, 2, 64, 64),          # first chunk: empty cache
    (0, 40, 1, 128, 7),
    (300, 200, 3, 128, 200),     # ragged query tile (200 = 128 + 72) and key tail (500 = 7*64 + 52)
    (300, 200, 3, 128, 50),
    (333, 130, 2, 128, 13),
    (1, 1, 1, 128, 1),
    (63, 129, 2, 64, 129),
    (1000, 520, 2, 128, 130),
])
def test_attention_matches_oracle(n, Lc, N, D, L_B):
    Q, Kc, Vc, Kn, Vn = _inputs(n, Lc, N, D, seed=n * 7 + Lc)
    got = _run(Q, Kc, Vc, Kn, Vn, L_B)
    want = orc.chunk_attention(Q, Kc, Vc, Kn, Vn, block_len=L_B)
    max_abs, rel = attn_errors(got, want)
    assert max_abs < ATTN_MAX_ABS and rel < ATTN_REL_FRO, (max_abs, rel)


def test_attention_peaked_softmax_and_fp32_output():
    # queries scaled x8: the softmax is peaked, |O| ~ 1, so the max-abs bound bites
    n, Lc, N, D = 500, 192, 2, 128
    Q, Kc, Vc, Kn, Vn = _inputs(n, Lc, N, D, seed=99, q_gain=8.0)
    want = orc.chunk_attention(Q, Kc, Vc, Kn, Vn, block_len=64)
    assert np.abs(want).max() > 0.5
    for odt in (torch.bfloat16, torch.float32):
        got = _run(Q, Kc, Vc, Kn, Vn, 64, out_dtype=odt)
        max_abs, rel = attn_errors(got, want)
        assert max_abs < ATTN_MAX_ABS and rel < ATTN_REL_FRO, (odt, max_abs, rel)


# With a workspace the launch cuts the flattened (head, query tile, key tiles) list into equal runs, one per CU, and
# merges the partial results of the query tiles that several workgroups worked on.  These shapes are long enough for
# that path to be taken (a few query tiles, hundreds of key tiles each), so a query tile is shared by many runs.
@pytest.mark.parametrize("n,Lc,N,D,L_B,odt,q_gain", [
    (16000, 600, 4, 128, 600, torch.bfloat16, 1.0),   # 12 items of 130 units each over 256 runs
    (9000, 1500, 3, 128, 500, torch.bfloat16, 1.0),   # block mask: the items have different lengths
    (9000, 1500, 3, 128, 500, torch.float32, 8.0),    # ... peaked softmax, fp32 output
    (20000, 300, 5, 64, 300, torch.bfloat16, 1.0),    # head dim 64
    (0, 9000, 2, 128, 1, torch.bfloat16, 1.0),        # no cache, strictly causal inside the chunk
    (12345, 777, 3, 128, 100, torch.bfloat16, 1.0),   # ragged everything
])
def test_attention_equal_runs_match_oracle(n, Lc, N, D, L_B, odt, q_gain):
    Q, Kc, Vc, Kn, Vn = _inputs(n, Lc, N, D, seed=n + Lc + N, q_gain=q_gain)
    ws = attention_workspace(D)
    got = _run(Q, Kc, Vc, Kn, Vn, L_B, out_dtype=odt, ws=ws)
    want = orc.chunk_attention(Q, Kc, Vc, Kn, Vn, block_len=L_B)
    max_abs, rel = attn_errors(got, want)
    assert max_abs < ATTN_MAX_ABS and rel < ATTN_REL_FRO, (max_abs, rel)
    # the same launch without the workspace (one workgroup per query tile) agrees to the rounding of the bf16
    # softmax weights (taken relative to different running maxima), and a second launch with the workspace (now
    # holding the first one's partial results) gives the same bits as the first
    plain = _run(Q, Kc, Vc, Kn, Vn, L_B, out_dtype=odt)
    assert np.abs(plain - got).max() < ATTN_MAX_ABS * max(1.0, np.abs(want).max())
    again = _run(Q, Kc, Vc, Kn, Vn, L_B, out_dtype=odt, ws=ws)
    assert np.array_equal(got, again)


def test_attention_workspace_too_small_falls_back_to_whole_query_tiles():
    n, Lc, N, D = 16000, 600, 4, 128
    Q, Kc, Vc, Kn, Vn = _inputs(n, Lc, N, D, seed=3)
    small = torch.empty(4096, dtype=torch.uint8, device=DEV)
    got = _run(Q, Kc, Vc, Kn, Vn, Lc, ws=small)
    plain = _run(Q, Kc, Vc, Kn, Vn, Lc)
    assert np.array_equal(got, plain)


def test_attention_large_key_offset_and_fewer_queries():
    # a large common vector on every key shifts logits by a per-row constant: exercises the running max
    n, Lc, N, D = 200, 100, 2, 128
    Q, Kc, Vc, Kn, Vn = _inputs(n, Lc, N, D, seed=5)
    shift = wl.round_to_bf16(np.full((1, N, D), 3.0, np.float32))
    Kc2, Kn2 = wl.round_to_bf16(Kc + shift), wl.round_to_bf16(Kn + shift)
    got = _run(Q, Kc2, Vc, Kn2, Vn, 25, Lq=70)
    want = orc.chunk_attention(Q[:70], Kc2, Vc, Kn2, Vn, block_len=25)
    max_abs, rel = attn_errors(got, want)
    assert max_abs < ATTN_MAX_ABS and rel < ATTN_REL_FRO, (max_abs, rel)


def test_attention_strided_slabs():
    # cache rows live in a slab with spare capacity and a wider token stride
    n, Lc, N, D = 150, 70, 2, 64
    Q, Kc, Vc, Kn, Vn = _inputs(n, Lc, N, D, seed=17)
    ld = N * D + 64
    slabK = torch.zeros(n + 10, ld, device=DEV, dtype=torch.bfloat16)
    slabV = torch.zeros(n + 10, ld, device=DEV, dtype=torch.bfloat16)
    slabK[:n, : N * D] = dev(Kc, "bf16").view(n, N * D)
    slabV[:n, : N * D] = dev(Vc, "bf16").view(n, N * D)
    Kv = slabK.as_strided((n, N, D), (ld, D, 1))
    Vv = slabV.as_strided((n, N, D), (ld, D, 1))
    O = torch.empty(Lc, N, D, device=DEV, dtype=torch.bfloat16)
    B.pafu_chunk_attention(dev(Q, "bf16"), Kv, Vv, n, dev(Kn, "bf16"), dev(Vn, "bf16"), 35, O)
    torch.cuda.synchronize()
    want = orc.chunk_attention(Q, Kc, Vc, Kn, Vn, block_len=35)
    max_abs, rel = attn_errors(host(O), want)
    assert max_abs < ATTN_MAX_ABS and rel < ATTN_REL_FRO, (max_abs, rel)


# ------------------------------------------------------------------ index-based Select (Sec. 3.4; Eq. 7)
@pytest.mark.parametrize("n_cache,n_kept,Lc,N,D,L_B,order", [
    (300, 128, 64, 2, 64, 64, "sorted"),       # retained rows = whole tiles
    (300, 100, 64, 2, 64, 16, "sorted"),       # last cache tile mixed with chunk rows
    (1000, 517, 200, 3, 128, 200, "sorted"),
    (1000, 517, 200, 3, 128, 50, "shuffled"),  # the list need not be ascending
    (500, 500, 130, 2, 128, 13, "sorted"),     # everything kept
    (400, 0, 40, 1, 128, 7, "sorted"),         # nothing kept
    (70, 1, 1, 1, 128, 1, "sorted"),
    (5000, 2560, 300, 2, 128, 300, "sorted"),  # many full tiles through the prefetched-id path
])
def test_gather_attention_matches_oracle_and_the_compacted_path(n_cache, n_kept, Lc, N, D, L_B, order):
    Q, Kc, Vc, Kn, Vn = _inputs(n_cache, Lc, N, D, seed=n_cache + n_kept)
    rng = np.random.default_rng(n_cache * 3 + n_kept)
    ids = np.sort(rng.permutation(n_cache)[:n_kept]).astype(np.int32)
    if order == "shuffled":
        ids = rng.permutation(ids).astype(np.int32)
    d_ids = torch.from_numpy(ids).to(DEV) if n_kept else torch.zeros(4, dtype=torch.int32, device=DEV)
    dQ, dKc, dVc, dKn, dVn = (dev(x, "bf16") for x in (Q, Kc, Vc, Kn, Vn))
    O = torch.full((Lc + 2, N, D), 55.0, device=DEV, dtype=torch.bfloat16)
    B.pafu_chunk_attention_gather(dQ, dKc, dVc, d_ids, n_kept, dKn, dVn, L_B, O[:Lc])
    torch.cuda.synchronize()
    assert torch.all(O[Lc:] == 55.0)
    got = host(O[:Lc])
    want = orc.chunk_attention(Q, Kc[ids], Vc[ids], Kn, Vn, block_len=L_B)
    max_abs, rel = attn_errors(got, want)
    assert max_abs < ATTN_MAX_ABS and rel < ATTN_REL_FRO, (max_abs, rel)
    # same arithmetic in the same order as the plain kernel on the compacted cache: identical bits
    plain = _run(Q, Kc[ids], Vc[ids], Kn, Vn, L_B)
    assert np.array_equal(got, plain)


def test_gather_attention_with_equal_runs():
    n_cache, n_kept, Lc, N, D, L_B = 30000, 17000, 600, 4, 128, 200
    Q, Kc, Vc, Kn, Vn = _inputs(n_cache, Lc, N, D, seed=41)
    ids = np.sort(np.random.default_rng(4).permutation(n_cache)[:n_kept]).astype(np.int32)
    ws = attention_workspace(D)
    O = torch.full((Lc + 2, N, D), 55.0, device=DEV, dtype=torch.bfloat16)
    B.pafu_chunk_attention_gather(dev(Q, "bf16"), dev(Kc, "bf16"), dev(Vc, "bf16"), torch.from_numpy(ids).to(DEV), n_kept,
                                  dev(Kn, "bf16"), dev(Vn, "bf16"), L_B, O[:Lc], workspace=ws)
    torch.cuda.synchronize()
    assert torch.all(O[Lc:] == 55.0)
    want = orc.chunk_attention(Q, Kc[ids], Vc[ids], Kn, Vn, block_len=L_B)
    max_abs, rel = attn_errors(host(O[:Lc]), want)
    assert max_abs < ATTN_MAX_ABS and rel < ATTN_REL_FRO, (max_abs, rel)
    # the plain kernel on the compacted cache with the same workspace cuts the work the same way: identical bits
    plain = _run(Q, Kc[ids], Vc[ids], Kn, Vn, L_B, ws=ws)
    assert np.array_equal(host(O[:Lc]), plain)


def test_gather_attention_clamps_out_of_range_ids():
    # ids outside the cache must not fault; rows are clamped into range (the result equals attention over those rows)
    n_cache, Lc, N, D = 200, 64, 2, 128
    Q, Kc, Vc, Kn, Vn = _inputs(n_cache, Lc, N, D, seed=5)
    ids = np.arange(128, dtype=np.int32)
    ids[3], ids[70] = -9, 10 ** 6
    eff = np.clip(ids, 0, n_cache - 1)
    O = torch.empty(Lc, N, D, device=DEV, dtype=torch.bfloat16)
    B.pafu_chunk_attention_gather(dev(Q, "bf16"), dev(Kc, "bf16"), dev(Vc, "bf16"), torch.from_numpy(ids).to(DEV), 128,
                                  dev(Kn, "bf16"), dev(Vn, "bf16"), Lc, O)
    torch.cuda.synchronize()
    want = orc.chunk_attention(Q, Kc[eff], Vc[eff], Kn, Vn, block_len=Lc)
    max_abs, rel = attn_errors(host(O), want)
    assert max_abs < ATTN_MAX_ABS and rel < ATTN_REL_FRO, (max_abs, rel)
