"""GPU parity of pafu_compact_kv, pafu_select_topk and pafu_score against the fp64 oracle,
called through the C ABI.  Indices and the compacted cache must match bit for bit; scores
within max-abs 1e-3."""
import numpy as np
import pytest
import torch

from oracle import pafu_oracle as orc
from paper_2601_21896_amd import binding as B
from paper_2601_21896_amd import workloads as wl
from tests.gpu_util import DEV, SCORE_MAX_ABS, bits, dev, host

pytestmark = pytest.mark.gpu


# ------------------------------------------------------------------------------- compact
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("n,N,D,count,pad", [(256, 2, 64, 128, 0), (1000, 12, 128, 517, 0), (333, 3, 40, 100, 8),
                                             (64, 40, 128, 64, 0), (50, 1, 8, 7, 0), (40, 52, 128, 33, 0),
                                             (30, 1, 10, 11, 6)])
def test_compact_bit_exact(dtype, n, N, D, count, pad):
    rng = np.random.default_rng(n + count)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    ld_in = N * D + pad
    Kslab = torch.randn(n, ld_in, device=DEV).to(tdt)
    Vslab = torch.randn(n, ld_in, device=DEV).to(tdt)
    K = Kslab.as_strided((n, N, D), (ld_in, D, 1))
    V = Vslab.as_strided((n, N, D), (ld_in, D, 1))
    SL = torch.randn(n, device=DEV)
    ids_np = np.sort(rng.permutation(n)[:count]).astype(np.int32)
    ids = torch.from_numpy(ids_np).to(DEV)
    guard = 4
    sentinel = 7.0
    Ko = torch.full((count + 2 * guard, ld_in), sentinel, device=DEV).to(tdt)
    Vo = torch.full((count + 2 * guard, ld_in), sentinel, device=DEV).to(tdt)
    SLo = torch.full((count + 2 * guard,), sentinel, device=DEV)
    Ko_v = Ko.as_strided((count, N, D), (ld_in, D, 1), guard * ld_in)
    Vo_v = Vo.as_strided((count, N, D), (ld_in, D, 1), guard * ld_in)
    B.pafu_compact_kv(K, V, SL, ids, count, Ko_v, Vo_v, SLo[guard:guard + count])
    torch.cuda.synchronize()
    Kw, Vw, SLw = orc.compact_kv(bits(K), bits(V), bits(SL), ids_np)
    assert np.array_equal(bits(Ko_v), Kw) and np.array_equal(bits(Vo_v), Vw)
    assert np.array_equal(bits(SLo[guard:guard + count]), SLw)
    # guard rows, and the padding columns between rows, are untouched
    for t in (Ko, Vo):
        assert torch.all(t[:guard] == sentinel) and torch.all(t[guard + count:] == sentinel)
        if pad:
            assert torch.all(t[:, N * D:] == sentinel)
    assert torch.all(SLo[:guard] == sentinel) and torch.all(SLo[guard + count:] == sentinel)


def test_compact_skips_invalid_ids_and_optional_scores():
    n, N, D = 20, 2, 64
    K = torch.randn(n, N, D, device=DEV).to(torch.bfloat16)
    V = torch.randn(n, N, D, device=DEV).to(torch.bfloat16)
    ids = torch.tensor([3, -1, 19, 20, 5], dtype=torch.int32, device=DEV)
    Ko = torch.zeros(5, N, D, device=DEV, dtype=torch.bfloat16)
    Vo = torch.zeros(5, N, D, device=DEV, dtype=torch.bfloat16)
    B.pafu_compact_kv(K, V, None, ids, 5, Ko, Vo, None)
    torch.cuda.synchronize()
    for r, i in enumerate([3, None, 19, None, 5]):
        if i is None:
            assert torch.all(Ko[r] == 0) and torch.all(Vo[r] == 0)
        else:
            assert torch.equal(Ko[r], K[i]) and torch.equal(Vo[r], V[i])


def test_compact_with_the_count_on_the_device():
    # selection writes the count, compaction reads it there: no host round trip in between
    n, N, D, k = 3000, 4, 128, 1111
    g = torch.Generator(device=DEV)
    g.manual_seed(3)
    K = torch.randn(n, N, D, device=DEV, generator=g).to(torch.bfloat16)
    V = torch.randn(n, N, D, device=DEV, generator=g).to(torch.bfloat16)
    SL = torch.randn(n, device=DEV, generator=g)
    cap = 1500                                              # room for more rows than the budget keeps
    ids = torch.full((cap,), -1, dtype=torch.int32, device=DEV)
    cnt = torch.zeros(1, dtype=torch.int32, device=DEV)
    Ko = torch.full((cap, N, D), 7.0, device=DEV, dtype=torch.bfloat16)
    Vo = torch.full((cap, N, D), 7.0, device=DEV, dtype=torch.bfloat16)
    SLo = torch.full((cap,), 7.0, device=DEV)
    B.pafu_select_topk(SL, k, ids, cnt)
    B.pafu_compact_kv_counted(K, V, SL, ids, cnt, cap, Ko, Vo, SLo)
    torch.cuda.synchronize()
    want_ids = orc.select_topk(host(SL), k)
    Kw, Vw, SLw = orc.compact_kv(bits(K), bits(V), bits(SL), want_ids)
    assert int(cnt.item()) == k
    assert np.array_equal(bits(Ko[:k]), Kw) and np.array_equal(bits(Vo[:k]), Vw) and np.array_equal(bits(SLo[:k]), SLw)
    assert torch.all(Ko[k:] == 7.0) and torch.all(Vo[k:] == 7.0) and torch.all(SLo[k:] == 7.0)   # nothing past the count
    # a device count above the capacity is clamped to it, a negative one moves nothing
    cnt.fill_(10 ** 6)
    ids2 = torch.arange(cap, dtype=torch.int32, device=DEV)
    B.pafu_compact_kv_counted(K, V, SL, ids2, cnt, cap, Ko, Vo, SLo)
    cnt.fill_(-5)
    Ko2 = torch.full((cap, N, D), 3.0, device=DEV, dtype=torch.bfloat16)
    B.pafu_compact_kv_counted(K, V, None, ids2, cnt, cap, Ko2, Vo, None)
    torch.cuda.synchronize()
    assert torch.equal(Ko, K[:cap]) and torch.all(Ko2 == 3.0)


# ------------------------------------------------------------------------------- select
def _run_select(s_np, k):
    n = len(s_np)
    s = torch.from_numpy(s_np).to(DEV) if n else torch.zeros(4, device=DEV)
    m = min(k, n)
    out = torch.full((m + 8,), -7, dtype=torch.int32, device=DEV)
    cnt = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    B.pafu_select_topk(s, k, out, cnt, n=n)
    torch.cuda.synchronize()
    assert int(cnt.item()) == m
    assert torch.all(out[m:] == -7)                     # nothing written past min(k, n)
    return out[:m].cpu().numpy()


# sizes on both sides of every kernel choice: 1 x 256, 2 x 512, 2 x 1024, 3 x 1024 words x threads, then the fallback
@pytest.mark.parametrize("n", [1, 2, 63, 64, 255, 1000, 4095, 4096, 4097, 8192, 8193, 9001, 32760, 32768, 32769, 65536,
                               65537, 75600, 98304, 98305, 120000])
def test_select_matches_oracle_with_ties(n):
    rng = np.random.default_rng(n)
    coarse = (rng.integers(-4, 5, size=n) * 0.25).astype(np.float32)     # many ties at the threshold
    smooth = rng.standard_normal(n).astype(np.float32)
    for s in (coarse, smooth):
        for k in sorted({0, 1, n // 3, n // 2, n - 1, n, n + 5}):
            if k < 0:
                continue
            got = _run_select(s, k)
            assert np.array_equal(got, orc.select_topk(s, k)), (n, k)


@pytest.mark.parametrize("n,k,n_pinned", [(1000, 400, 100), (1000, 50, 100), (4097, 2000, 1560), (32760, 16380, 1560),
                                         (32760, 16380, 0), (60000, 20000, 4680), (75600, 22680, 1560),
                                         (300, 300, 10), (300, 10, 300), (64, 0, 5)])
def test_select_pinned_prefix_matches_oracle(n, k, n_pinned):
    rng = np.random.default_rng(n + k + n_pinned)
    s = (rng.integers(-50, 50, size=n) * 0.25).astype(np.float32)      # many ties at the threshold
    s[:n_pinned] -= 100.0                                              # the prefix would lose on its scores
    s[rng.integers(0, n, 3)] = np.inf
    m = min(k, n)
    out = torch.full((m + 8,), -7, dtype=torch.int32, device=DEV)
    cnt = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    B.pafu_select_topk_pinned(torch.from_numpy(s).to(DEV), k, n_pinned, out, cnt)
    torch.cuda.synchronize()
    assert int(cnt.item()) == m and torch.all(out[m:] == -7)
    assert np.array_equal(out[:m].cpu().numpy(), orc.select_topk(s, k, n_pinned))


def test_select_special_values_and_degenerate_inputs():
    s = np.array([np.nan, -np.inf, -0.0, 0.0, 1.0, np.inf, -1.0, np.nan, 0.0, -0.0, 3e-45, -3e-45], dtype=np.float32)
    for k in range(len(s) + 2):
        assert np.array_equal(_run_select(s, k), orc.select_topk(s, k)), k
    n = 5000
    for s in (np.zeros(n, np.float32), np.arange(n, dtype=np.float32), -np.arange(n, dtype=np.float32),
              np.full(n, np.nan, np.float32), np.full(n, -np.inf, np.float32)):
        for k in (1, 77, 2500, 4999):
            assert np.array_equal(_run_select(s, k), orc.select_topk(s, k))
    assert _run_select(np.zeros(0, np.float32), 3).shape == (0,)


@pytest.mark.parametrize("n", [3000, 20000, 40000, 70000, 90000, 110000])
def test_select_special_values_in_long_lists(n):
    # every kernel variant sees NaN, infinities, signed zeros, denormals and heavy ties, also in its ragged last word
    rng = np.random.default_rng(7 * n)
    s = (rng.integers(-3, 4, size=n) * 0.5).astype(np.float32)
    special = np.array([np.nan, -np.nan, np.inf, -np.inf, 0.0, -0.0, 1e-45, -1e-45, 3.4e38, -3.4e38], dtype=np.float32)
    where = rng.choice(n, size=n // 7, replace=False)
    s[where] = special[rng.integers(0, len(special), size=len(where))]
    s[-5:] = [np.nan, -0.0, np.inf, 0.0, -np.inf]
    for k in (1, n // 9, n // 2, n - 3):
        assert np.array_equal(_run_select(s, k), orc.select_topk(s, k)), (n, k)


def test_select_is_deterministic_across_runs():
    rng = np.random.default_rng(0)
    s = (rng.integers(0, 3, size=32760)).astype(np.float32)
    first = _run_select(s, 16380)
    for _ in range(10):
        assert np.array_equal(_run_select(s, 16380), first)


# ------------------------------------------------------------------------------- score
def _score_case(cfg, T, bias, n_out, act, seed, n_seg=1):
    rng = np.random.Generator(np.random.PCG64(seed))
    cfg = wl.scaled(cfg, n_out=n_out)
    F = cfg.H * n_seg
    W1, b1, W2, b2 = wl.make_head_weights(cfg, rng, F=F, bias=bias)
    q = wl.round_to_bf16 if cfg.dtype == "bf16" else (lambda a: a)
    segs = [q(rng.standard_normal((T, cfg.H), dtype=np.float32)) for _ in range(n_seg)]
    return segs, W1, b1, W2, b2


@pytest.mark.parametrize("name,T,bias,n_out,act,n_seg", [
    ("C0", 320, False, 1, "silu", 1),          # fp32 path at the tiny config's widths
    ("C0", 77, True, 12, "silu", 1),
    ("C0", 64, True, 3, "gelu_erf", 3),
    ("C1", 1000, False, 1, "silu", 1),         # MFMA path, ragged token tile
    ("C1", 129, True, 12, "silu", 1),
    ("C1", 300, True, 1, "gelu_erf", 1),
    ("C1", 200, True, 12, "silu", 3),          # paper-form input [Q|K|V] (F = 4608)
    ("C4", 200, True, 1, "silu", 1),           # M = 512: two hidden passes
    ("C1", 9601, True, 1, "silu", 1),          # streaming kernel with 2 token tiles per workgroup, ragged tail
    ("C1", 20011, False, 1, "silu", 1),        # ... with 3
    ("C1", 30000, True, 12, "silu", 3),        # ... with 4, three feature segments
])
def test_score_matches_oracle(name, T, bias, n_out, act, n_seg):
    cfg = wl.CONFIGS[name]
    segs, W1, b1, W2, b2 = _score_case(cfg, T, bias, n_out, act, seed=T + n_out)
    dt = cfg.dtype
    d_segs = tuple(dev(s, dt) for s in segs)
    out = torch.full((T + 4,), 123.0, device=DEV)
    ws = torch.empty(B.pafu_score_workspace_bytes(cfg.M) // 4 + 4, device=DEV)
    B.pafu_score(d_segs, dev(W1, dt), dev(b1) if bias else None, dev(W2), dev(b2) if bias else None, out,
                 act=B.PAFU_ACT_SILU if act == "silu" else B.PAFU_ACT_GELU_ERF, workspace=ws, T=T)
    torch.cuda.synchronize()
    want = orc.smlp_score(np.concatenate(segs, axis=1), W1, b1 if bias else None, W2, b2 if bias else None, act=act)
    got = host(out)
    assert np.all(got[T:] == 123.0)
    err = np.abs(got[:T] - want).max()
    assert err < SCORE_MAX_ABS, err
    # the scores are not trivially small: the tolerance must mean something
    assert np.abs(want).max() > 20 * err


def test_score_paper_true_width_mfma():
    # App. A widths: 4608 -> 1024 -> 12, mean over the 12 outputs
    cfg = wl.scaled(wl.C1, M=1024, n_out=12)
    rng = np.random.Generator(np.random.PCG64(5))
    W1, b1, W2, b2 = wl.make_head_weights(cfg, rng, F=3 * cfg.H, bias=True)
    T = 160
    segs = [wl.round_to_bf16(rng.standard_normal((T, cfg.H), dtype=np.float32)) for _ in range(3)]
    out = torch.empty(T, device=DEV)
    ws = torch.empty(B.pafu_score_workspace_bytes(cfg.M) // 4 + 4, device=DEV)
    B.pafu_score(tuple(dev(s, "bf16") for s in segs), dev(W1, "bf16"), dev(b1), dev(W2), dev(b2), out, workspace=ws)
    torch.cuda.synchronize()
    want = orc.smlp_score(np.concatenate(segs, axis=1), W1, b1, W2, b2)
    assert np.abs(host(out) - want).max() < SCORE_MAX_ABS


def test_score_mfma_path_with_hidden_width_not_a_multiple_of_256():
    # bf16, F % 64 == 0, M % 32 == 0 but M % 256 != 0: the one-tile MFMA kernel
    rng = np.random.default_rng(11)
    T, F, M = 301, 192, 96
    X = wl.round_to_bf16(rng.standard_normal((T, F)).astype(np.float32))
    W1 = wl.round_to_bf16((rng.standard_normal((M, F)) * 0.1).astype(np.float32))
    W2 = rng.standard_normal((3, M)).astype(np.float32)
    b1 = rng.standard_normal(M).astype(np.float32)
    b2 = rng.standard_normal(3).astype(np.float32)
    out = torch.empty(T, device=DEV)
    ws = torch.empty(M + 8, device=DEV)
    B.pafu_score(dev(X, "bf16"), dev(W1, "bf16"), dev(b1), dev(W2), dev(b2), out, workspace=ws)
    torch.cuda.synchronize()
    assert np.abs(host(out) - orc.smlp_score(X, W1, b1, W2, b2)).max() < SCORE_MAX_ABS


def test_score_generic_path_on_odd_shapes():
    # bf16 shapes the MFMA tiles do not divide fall back to the plain-FMA path
    rng = np.random.default_rng(3)
    T, F, M = 37, 72, 20
    X = wl.round_to_bf16(rng.standard_normal((T, F)).astype(np.float32))
    W1 = wl.round_to_bf16((rng.standard_normal((M, F)) * 0.1).astype(np.float32))
    W2 = rng.standard_normal((2, M)).astype(np.float32)
    b1 = rng.standard_normal(M).astype(np.float32)
    out = torch.empty(T, device=DEV)
    ws = torch.empty(M + 8, device=DEV)
    B.pafu_score(dev(X, "bf16"), dev(W1, "bf16"), dev(b1), dev(W2), None, out, workspace=ws)
    torch.cuda.synchronize()
    assert np.abs(host(out) - orc.smlp_score(X, W1, b1, W2, None)).max() < SCORE_MAX_ABS
