"""GPU parity of the 8-bit (E4M3) K/V cache path: quantisation and compaction bit for bit against the oracle's codes,
attention and the steps against the oracle on the dequantised values (same tolerances as the bf16 path: the kernel's
arithmetic is the bf16 kernel's, only the storage is narrower)."""
import numpy as np
import pytest
import torch

from oracle import pafu_oracle as orc
from paper_2601_21896_amd import binding as B
from paper_2601_21896_amd import workloads as wl
from tests.gpu_util import (ATTN_MAX_ABS, ATTN_REL_FRO, DEV, SCORE_MAX_ABS, attention_workspace, attn_errors, dev, host,
                            step_workspace)

pytestmark = pytest.mark.gpu
FP8 = B.PAFU_FP8_E4M3


def codes_dev(c):
    return torch.from_numpy(np.ascontiguousarray(c)).to(DEV)


def test_quantize_matches_the_oracle_bit_for_bit():
    rng = np.random.Generator(np.random.PCG64(7))
    rows, N, D, pad = 300, 3, 128, 32
    base = rng.standard_normal((rows, N * D), dtype=np.float32) * np.float32(3.0)
    special = np.array([0.0, -0.0, 448.0, -448.0, 449.0, 464.0, 1e9, -1e9, np.inf, -np.inf, np.nan, 2.0 ** -6, 2.0 ** -9,
                        2.0 ** -10, 7.5 * 2.0 ** -9, 1.0625, 1.1875, 2.0 ** -20, -2.0 ** -30, 432.0, 416.0], np.float32)
    base[0, : len(special)] = special
    base[1] *= np.float32(2.0 ** -8)            # a row in the subnormal range of the format
    base[2] *= np.float32(100.0)                # a row that saturates
    Kh, Vh = wl.round_to_bf16(base), wl.round_to_bf16(base[::-1].copy())
    for ek, ev in ((0, 0), (-5, -6), (3, -12)):
        slabK = torch.full((rows + 2, N * D + pad), 0xAB, dtype=torch.uint8, device=DEV)
        slabV = torch.full((rows + 2, N * D + pad), 0xAB, dtype=torch.uint8, device=DEV)
        Kq = slabK[1:rows + 1, : N * D]
        Vq = slabV[1:rows + 1, : N * D]
        B.pafu_quantize_kv(dev(Kh, "bf16").view(rows, N, D), dev(Vh, "bf16").view(rows, N, D), ek, ev, Kq, Vq)
        torch.cuda.synchronize()
        assert np.array_equal(Kq.cpu().numpy(), orc.quantise_e4m3(Kh, ek)), (ek, ev)
        assert np.array_equal(Vq.cpu().numpy(), orc.quantise_e4m3(Vh, ev)), (ek, ev)
        for slab in (slabK, slabV):             # guard rows and padding columns untouched
            assert torch.all(slab[0] == 0xAB) and torch.all(slab[-1] == 0xAB) and torch.all(slab[:, N * D:] == 0xAB)


def test_dequantize_is_exact_for_every_code():
    codes = np.tile(np.arange(256, dtype=np.uint8), (4, 1))           # [4, 256] = N * D with N = 2, D = 128
    for ek, ev in ((0, 0), (-7, 5), (-30, 30)):
        K = torch.zeros(4, 2, 128, device=DEV, dtype=torch.bfloat16)
        V = torch.zeros_like(K)
        B.pafu_dequantize_kv(codes_dev(codes), codes_dev(codes[:, ::-1].copy()), ek, ev, K, V)
        torch.cuda.synchronize()
        wantK = orc.dequantise_e4m3(codes, ek).reshape(4, 2, 128)
        wantV = orc.dequantise_e4m3(codes[:, ::-1], ev).reshape(4, 2, 128)
        for got, want in ((host(K), wantK), (host(V), wantV)):
            nan = np.isnan(want)
            assert np.array_equal(np.isnan(got), nan)
            assert np.array_equal(got[~nan].astype(np.float64), want[~nan])
            assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_compact_moves_codes():
    rng = np.random.default_rng(2)
    n, N, D, count = 500, 12, 128, 217
    K = torch.from_numpy(rng.integers(0, 256, (n, N * D), dtype=np.uint8)).to(DEV)
    V = torch.from_numpy(rng.integers(0, 256, (n, N * D), dtype=np.uint8)).to(DEV)
    SL = torch.randn(n, device=DEV)
    ids_np = np.sort(rng.permutation(n)[:count]).astype(np.int32)
    Ko = torch.zeros(count, N * D, dtype=torch.uint8, device=DEV)
    Vo = torch.zeros_like(Ko)
    SLo = torch.zeros(count, device=DEV)
    rc = B.library().pafu_compact_kv(torch.cuda.current_stream().cuda_stream, K.data_ptr(), V.data_ptr(), SL.data_ptr(),
                                     N * D, n, torch.from_numpy(ids_np).to(DEV).data_ptr(), count, N, D, FP8,
                                     Ko.data_ptr(), Vo.data_ptr(), SLo.data_ptr(), N * D)
    assert rc == 0
    torch.cuda.synchronize()
    Kw, Vw, SLw = orc.compact_kv(K.cpu().numpy(), V.cpu().numpy(), SL.cpu().numpy(), ids_np)
    assert np.array_equal(Ko.cpu().numpy(), Kw) and np.array_equal(Vo.cpu().numpy(), Vw)
    assert np.array_equal(SLo.cpu().numpy(), SLw)


def _inputs(n, Lc, N, D, seed, q_gain=1.0):
    rng = np.random.Generator(np.random.PCG64(seed))
    c = rng.uniform(0.5, 2.0, size=(N * D,)).astype(np.float32)
    r = lambda rows, s=None: wl.round_to_bf16(
        (rng.standard_normal((rows, N * D), dtype=np.float32) * (1.0 if s is None else s[None, :]))).reshape(rows, N, D)
    Kc, Vc = r(n, c), r(n)
    Q = wl.round_to_bf16(r(Lc) * np.float32(q_gain))
    Kn, Vn = r(Lc, c), r(Lc)
    return Q, Kc, Vc, Kn, Vn


@pytest.mark.parametrize("n,Lc,N,L_B,odt,ws,pad", [
    (128, 64, 2, 64, torch.bfloat16, False, 0),
    (300, 200, 3, 50, torch.bfloat16, False, 0),       # cache / chunk boundary inside a tile, block mask, ragged tiles
    (0, 130, 2, 13, torch.bfloat16, False, 0),         # empty cache
    (1, 1, 1, 1, torch.bfloat16, False, 0),
    (1000, 520, 2, 130, torch.float32, False, 64),     # padded strides, fp32 output
    (333, 129, 2, 129, torch.bfloat16, False, 16),
    (16000, 600, 4, 600, torch.bfloat16, True, 0),     # long key axis: equal runs + merge
    (9000, 1500, 3, 500, torch.bfloat16, True, 0),
])
def test_attention_fp8_matches_oracle_on_dequantised_values(n, Lc, N, L_B, odt, ws, pad):
    D, ek, ev = 128, -5, -6
    Q, Kc, Vc, Kn, Vn = _inputs(n, Lc, N, D, seed=n * 5 + Lc)
    q = lambda a, e: orc.quantise_e4m3(a.reshape(a.shape[0], N * D), e)
    Kcq, Vcq, Knq, Vnq = q(Kc, ek), q(Vc, ev), q(Kn, ek), q(Vn, ev)

    def slab(c):                                          # rows with a padded stride
        t = torch.zeros(max(c.shape[0], 1), N * D + pad, dtype=torch.uint8, device=DEV)
        t[: c.shape[0], : N * D] = codes_dev(c)
        return t[: c.shape[0], : N * D] if c.shape[0] else None
    O = torch.full((Lc + 2, N, D), 55.0, device=DEV, dtype=odt)
    B.pafu_chunk_attention_fp8(dev(Q, "bf16"), slab(Kcq), slab(Vcq), n, slab(Knq), slab(Vnq), L_B, ek, ev, O[:Lc],
                               workspace=attention_workspace(D) if ws else None)
    torch.cuda.synchronize()
    assert torch.all(O[Lc:] == 55.0)
    dq = lambda c, e: orc.dequantise_e4m3(c, e).reshape(c.shape[0], N, D)
    want = orc.chunk_attention(Q, dq(Kcq, ek), dq(Vcq, ev), dq(Knq, ek), dq(Vnq, ev), block_len=L_B)
    max_abs, rel = attn_errors(host(O[:Lc]), want)
    assert max_abs < ATTN_MAX_ABS and rel < ATTN_REL_FRO, (max_abs, rel)
    # against the oracle on the UNquantised tensors the difference is the storage format's, far above rounding
    full = orc.chunk_attention(Q, Kc, Vc, Kn, Vn, block_len=L_B)
    assert attn_errors(want, full)[1] > 2 * rel or n + Lc < 8


def _rollout_fp8(cfg, k, n_chunks, L_B, ek, ev, rows=None, n_pinned=0, workspace=False):
    N, D, Lc = cfg.N, cfg.D, cfg.Lc
    W1, b1, W2, b2 = wl.make_rollout_weights(cfg, bias=True)
    dW1, db1, dW2, db2 = dev(W1, "bf16"), dev(b1), dev(W2), dev(b2)
    cap = k + Lc
    slabs = [dict(K=torch.zeros(cap, N * D, device=DEV, dtype=torch.uint8),
                  V=torch.zeros(cap, N * D, device=DEV, dtype=torch.uint8),
                  SL=torch.zeros(cap, device=DEV)) for _ in range(2)]
    st = orc.RolloutState(N, D, np.uint8)
    st.K, st.V = st.K.reshape(0, N * D), st.V.reshape(0, N * D)
    ids = torch.empty(max(k, 1), dtype=torch.int32, device=DEV)
    O = torch.empty(Lc, N, D, device=DEV, dtype=torch.bfloat16)
    n, cur, sizes = 0, 0, []
    for t in range(n_chunks):
        c = wl.make_chunk_inputs(cfg, t)
        src, dst = slabs[cur], slabs[1 - cur]
        n_kept = min(k, n)
        args = B.make_step_args(B.PAFU_MODE_ROLLOUT, N, D, n, Lc, k, L_B, None, dev(c["X_chunk"], "bf16"), dW1, db1,
                                dW2, db2, src["K"], src["V"], src["SL"], dev(c["Q"], "bf16"), dev(c["K_chunk"], "bf16"),
                                dev(c["V_chunk"], "bf16"), None, ids, dst["K"], dst["V"], dst["SL"], O,
                                n_pinned=n_pinned, kv_dtype=FP8, k_scale_log2=ek, v_scale_log2=ev)
        if workspace:
            step_workspace(args)
        B.pafu_step(args)
        torch.cuda.synchronize()
        s_chunk = host(dst["SL"][n_kept:n_kept + Lc])
        # the oracle's state holds codes as [n, N * D]; its attention wants [n, N, D]
        st3 = orc.RolloutState(N, D, np.uint8)
        st3.K, st3.V, st3.SL = st.K.reshape(-1, N, D), st.V.reshape(-1, N, D), st.SL
        out = orc.rollout_step_fp8(st3, c["X_chunk"], W1, b1, W2, b2, c["Q"], c["K_chunk"], c["V_chunk"], k, L_B, ek, ev,
                                   forced_chunk_scores_f32=s_chunk, n_pinned=n_pinned, rows=rows)
        st.K, st.V, st.SL = st3.K.reshape(-1, N * D), st3.V.reshape(-1, N * D), st3.SL
        assert np.abs(s_chunk - out["s_chunk"]).max() < SCORE_MAX_ABS, t
        assert np.array_equal(host(ids)[:n_kept], out["ids"]), t
        n = n_kept + Lc
        assert n == st.n
        assert np.array_equal(dst["K"][:n].cpu().numpy(), st.K) and np.array_equal(dst["V"][:n].cpu().numpy(), st.V), t
        assert np.array_equal(host(dst["SL"][:n]), st.SL), t
        got = host(O) if rows is None else host(O)[rows]
        max_abs, rel = attn_errors(got, out["O"])
        assert max_abs < ATTN_MAX_ABS and rel < ATTN_REL_FRO, (t, max_abs, rel)
        sizes.append(n)
        cur = 1 - cur
    return sizes


def test_rollout_fp8_small():
    cfg = wl.scaled(wl.C1, N=2, frame_tokens=30, chunk_frames=3, cache_frames=0, k=240)     # Lc = 90
    sizes = _rollout_fp8(cfg, 240, 8, cfg.Lc, -5, -6)
    assert sizes == [90, 180, 270, 330, 330, 330, 330, 330]
    _rollout_fp8(cfg, 240, 6, 30, -4, -7, n_pinned=30)


def test_rollout_fp8_full_size_steps():
    # Wan-1.3B layer shapes, budget of 8 frames: the first evictions and two steady-state steps
    cfg = wl.C1
    rows = np.array(sorted(set(range(0, cfg.Lc, 37)) | {cfg.Lc - 1}))
    sizes = _rollout_fp8(cfg, wl.C3_K, 6, cfg.Lc, -5, -6, rows=rows, workspace=True)
    assert sizes == [4680, 9360, 14040, 17160, 17160, 17160]


def test_step_single_fp8():
    cfg = wl.scaled(wl.C1, N=2, frame_tokens=60, cache_frames=9, chunk_frames=3, k=270)     # n = 540, Lc = 180
    d = wl.make_layer_inputs(cfg)
    n, Lc, N, D, k, ek, ev = cfg.n, cfg.Lc, cfg.N, cfg.D, cfg.k, -5, -6
    Kq = orc.quantise_e4m3(d["K_cache"].reshape(n, N * D), ek)
    Vq = orc.quantise_e4m3(d["V_cache"].reshape(n, N * D), ev)
    X = dev(np.concatenate([d["X_cache"], d["X_chunk"]]), "bf16")
    scores = torch.empty(n + Lc, device=DEV)
    ids = torch.empty(k, dtype=torch.int32, device=DEV)
    K_out = torch.zeros(k + Lc, N * D, device=DEV, dtype=torch.uint8)
    V_out = torch.zeros_like(K_out)
    SL_out = torch.zeros(k, device=DEV)
    O = torch.empty(Lc, N, D, device=DEV, dtype=torch.bfloat16)
    args = B.make_step_args(B.PAFU_MODE_SINGLE, N, D, n, Lc, k, 60, X[:n], X[n:], dev(d["W1"], "bf16"), None,
                            dev(d["W2"]), None, codes_dev(Kq), codes_dev(Vq), None, dev(d["Q"], "bf16"),
                            dev(d["K_chunk"], "bf16"), dev(d["V_chunk"], "bf16"), scores, ids, K_out, V_out, SL_out, O,
                            kv_dtype=FP8, k_scale_log2=ek, v_scale_log2=ev)
    B.pafu_step(args)
    torch.cuda.synchronize()
    got_s = host(scores)
    want_ids = orc.select_topk(got_s[:n], k)
    assert np.array_equal(host(ids), want_ids)
    Kk, Vk, SLk = orc.compact_kv(Kq, Vq, got_s[:n], want_ids)
    Knq = orc.quantise_e4m3(d["K_chunk"].reshape(Lc, N * D), ek)
    Vnq = orc.quantise_e4m3(d["V_chunk"].reshape(Lc, N * D), ev)
    assert np.array_equal(K_out.cpu().numpy(), np.concatenate([Kk, Knq]))
    assert np.array_equal(V_out.cpu().numpy(), np.concatenate([Vk, Vnq]))
    assert np.array_equal(host(SL_out), SLk)
    dq = lambda c, e: orc.dequantise_e4m3(c, e).reshape(c.shape[0], N, D)
    want = orc.chunk_attention(d["Q"], dq(Kk, ek), dq(Vk, ev), dq(Knq, ek), dq(Vnq, ev), block_len=60)
    max_abs, rel = attn_errors(host(O), want)
    assert max_abs < ATTN_MAX_ABS and rel < ATTN_REL_FRO, (max_abs, rel)


def test_fp8_rejects_what_it_does_not_support():
    lib = B.library()
    A = 0x10000
    # head dim 64
    assert lib.pafu_chunk_attention_fp8(None, A, 64, A + 0x100000, A + 0x200000, 10, A + 0x300000, A + 0x400000, 64, 2,
                                        64, 128, 128, 128, 128, 64, 0.0, 0, 0, A + 0x500000, 0, None, 0) == -2
    # scale exponent out of range
    assert lib.pafu_chunk_attention_fp8(None, A, 64, A + 0x100000, A + 0x200000, 10, A + 0x300000, A + 0x400000, 64, 2,
                                        128, 256, 256, 256, 256, 64, 0.0, 100, 0, A + 0x500000, 0, None, 0) == -2
    assert lib.pafu_quantize_kv(None, A, A + 0x100000, 256, 10, 2, 128, 0, 0, A + 0x200000, A + 0x300000, 250) == -2
    assert lib.pafu_quantize_kv(None, A, A + 0x100000, 256, 10, 2, 128, 0, 0, A, A + 0x300000, 256) == -6
