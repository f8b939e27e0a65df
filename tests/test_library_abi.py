"""The C-ABI library loads, exports every declared symbol, and rejects bad arguments on the host
(no GPU needed: validation happens before any HIP call)."""
import ctypes
import os
import re

import pytest

from paper_2601_21896_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "pafu.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pafu_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    lib = binding.library()
    names = _declared_symbols()
    assert set(names) == set(binding.SYMBOLS)
    for name in names:
        assert getattr(lib, name) is not None
    assert binding.pafu_version() >= 1
    assert binding.pafu_study_build() == 0          # the in-tree library is the product, not a study build
    assert binding.pafu_strerror(0) == "ok"
    assert "NULL" in binding.pafu_strerror(-1)


def test_workspace_queries():
    assert binding.pafu_score_workspace_bytes(256) >= 257 * 4
    assert binding.pafu_select_workspace_bytes(32760) >= 0
    # two partial-result slots (256 queries x (D + 2) floats) for each of at most 256 runs
    assert binding.pafu_attention_workspace_bytes(4680, 12, 128) == 2 * 256 * 256 * (128 + 2) * 4
    assert binding.pafu_attention_workspace_bytes(64, 2, 64) == 2 * 256 * 256 * (64 + 2) * 4
    assert binding.pafu_attention_workspace_bytes(64, 2, 96) == 0
    a = _fake_step(A)
    assert binding.pafu_step_workspace_bytes(a) == 0 + binding.pafu_attention_workspace_bytes(20, 2, 64)
    a.n_out = 5
    assert binding.pafu_step_workspace_bytes(a) == 256 + binding.pafu_attention_workspace_bytes(20, 2, 64)


A = 0x10000   # a fake, 16-byte aligned "device address": validation must fail before it is ever used


def test_select_rejects_bad_arguments():
    lib = binding.library()
    assert lib.pafu_select_topk(None, None, 10, 3, A, None, None, 0) == -1       # NULL scores
    assert lib.pafu_select_topk(None, A, -1, 3, A, None, None, 0) == -2          # n < 0
    assert lib.pafu_select_topk(None, A, 10, -3, A, None, None, 0) == -2         # k < 0
    assert lib.pafu_select_topk(None, A + 4, 10, 3, A, None, None, 0) == -4      # misaligned
    assert lib.pafu_select_topk(None, A, 10, 3, None, None, None, 0) == -1       # NULL out
    assert lib.pafu_select_topk_pinned(None, A, 10, 3, -1, A, None, None, 0) == -2   # n_pinned < 0
    assert lib.pafu_select_topk_pinned(None, None, 10, 3, 2, A, None, None, 0) == -1


def test_compact_rejects_bad_arguments():
    lib = binding.library()
    f = lib.pafu_compact_kv
    ok = dict(K=A, V=A + 0x100000, SL=None, ld=1536, n=100, ids=A + 0x200000, count=50, N=12, D=128, dt=0,
              Ko=A + 0x300000, Vo=A + 0x400000, SLo=None, ldo=1536)

    def call(**kw):
        a = dict(ok); a.update(kw)
        return f(None, a["K"], a["V"], a["SL"], a["ld"], a["n"], a["ids"], a["count"], a["N"], a["D"], a["dt"],
                 a["Ko"], a["Vo"], a["SLo"], a["ldo"])

    assert call(K=None) == -1
    assert call(ids=None) == -1
    assert call(count=101) == -2
    assert call(ld=1000) == -2                    # stride smaller than a row
    assert call(dt=7) == -3
    assert call(K=A + 8) == -4
    assert call(ld=1540) == -4                    # 3080 B stride not a multiple of 16
    assert call(Ko=A) == -6                       # in place is not allowed
    assert call(SL=A + 0x500000) == -1            # SL without SL_out
    assert call(count=0, K=None) == 0             # nothing to do


def test_attention_rejects_bad_arguments():
    lib = binding.library()
    f = lib.pafu_chunk_attention
    ok = dict(Q=A, Lq=64, Kc=A + 0x100000, Vc=A + 0x200000, nk=10, Kn=A + 0x300000, Vn=A + 0x400000, Lc=64, N=2,
              D=64, ldq=128, ldc=128, ldn=128, ldo=128, LB=64, sc=0.0, O=A + 0x500000, od=0)

    def call(**kw):
        a = dict(ok); a.update(kw)
        return f(None, a["Q"], a["Lq"], a["Kc"], a["Vc"], a["nk"], a["Kn"], a["Vn"], a["Lc"], a["N"], a["D"], a["ldq"],
                 a["ldc"], a["ldn"], a["ldo"], a["LB"], a["sc"], a["O"], a["od"], None, 0)

    assert call(D=96) == -2
    assert call(Lq=0) == -2
    assert call(LB=0) == -2
    assert call(Lq=65) == -2                      # more queries than chunk tokens
    assert call(Q=None) == -1
    assert call(Kc=None) == -1
    assert call(od=5) == -3
    assert call(ldq=132) == -4
    assert call(O=A) == -6
    g = lib.pafu_chunk_attention_gather

    def gcall(n_cache=100, ids=A + 0x600000, nk=10, **kw):
        a = dict(ok); a.update(kw)
        return g(None, a["Q"], a["Lq"], a["Kc"], a["Vc"], n_cache, ids, nk, a["Kn"], a["Vn"], a["Lc"], a["N"], a["D"],
                 a["ldq"], a["ldc"], a["ldn"], a["ldo"], a["LB"], a["sc"], a["O"], a["od"], None, 0)

    assert gcall(nk=101) == -2                    # more retained rows than the cache holds
    assert gcall(ids=None) == -1
    assert gcall(ids=A + 0x600004) == -4
    assert gcall(D=96) == -2
    assert gcall(O=A + 0x100000) == -6            # output over the cache


def test_score_rejects_bad_arguments():
    lib = binding.library()
    f = lib.pafu_score

    def call(x0=A, x1=None, x2=None, ns=1, T=10, Fs=128, ld=128, dt=0, W1=A + 0x100000, b1=None, W2=A + 0x200000,
             b2=None, M=32, no=1, act=0, out=A + 0x300000, ws=None, wsb=0):
        return f(None, x0, x1, x2, ns, T, Fs, ld, dt, W1, b1, W2, b2, M, no, act, out, ws, wsb)

    assert call(x0=None) == -1
    assert call(ns=2) == -1                       # second segment missing
    assert call(ns=4) == -2
    assert call(M=0) == -2
    assert call(act=9) == -2
    assert call(dt=3) == -3
    assert call(ld=100) == -2
    assert call(ld=132) == -4
    assert call(no=12) == -5                      # averaging several outputs needs the workspace
    assert call(T=0, x0=None) == 0


def test_step_rejects_bad_arguments():
    lib = binding.library()
    a = binding.pafu_step_args()
    assert lib.pafu_step(None, None) == -1
    a.mode = 5
    assert lib.pafu_step(None, ctypes.byref(a)) == -2
    assert lib.pafu_step_layers(None, None, 2) == -1
    assert lib.pafu_step_layers(None, None, 0) == 0
    assert lib.pafu_step_layers_shared(None, None, 2, 0) == -1
    assert lib.pafu_step_layers_shared(None, ctypes.byref(a), 0, 0) == -2        # no layers
    assert lib.pafu_step_layers_shared(None, ctypes.byref(a), 1, 1) == -2        # index layer out of range
    assert lib.pafu_step_layers_shared(None, ctypes.byref(a), 1, 0) == -2        # the index layer is validated in full
    a.mode = 0
    a.n_pinned = -1
    a.Lc = a.N = a.D = 1
    assert lib.pafu_step(None, ctypes.byref(a)) == -2                             # negative frame sink


def _fake_step(base, mode=0, n=100, Lc=20, k=50, N=2, D=64):
    """A pafu_step_args that passes every check, over fake device addresses 1 MiB apart from `base`."""
    a = binding.pafu_step_args()
    a.mode, a.N, a.D, a.n, a.Lc, a.k, a.block_len = mode, N, D, n, Lc, k, Lc
    a.M, a.n_out, a.act, a.n_seg, a.Fs, a.x_dtype, a.out_dtype = 32, 1, 0, 1, N * D, 0, 0
    a.ld_x = a.ld_cache = a.ld_out = a.ld_chunk = a.ld_o = N * D
    slot = iter(range(base, base + 64 * 0x100000, 0x100000))
    a.x_cache[0], a.x_chunk[0] = next(slot), next(slot)
    a.W1, a.W2 = next(slot), next(slot)
    a.K_cache, a.V_cache, a.SL_in = next(slot), next(slot), next(slot)
    a.Q, a.K_chunk, a.V_chunk = next(slot), next(slot), next(slot)
    a.scores, a.ids = next(slot), next(slot)
    a.K_out, a.V_out, a.SL_out, a.O = next(slot), next(slot), next(slot), next(slot)
    return a


def test_step_rejects_aliased_buffers():
    lib = binding.library()
    row = 2 * 64 * 2                                    # bytes per token of K / V
    # ROLLOUT appends the chunk behind the k retained rows: an input inside that region is an alias too
    a = _fake_step(A, mode=1)
    a.K_chunk = a.K_out + 50 * row
    assert lib.pafu_step(None, ctypes.byref(a)) == -6
    a = _fake_step(A, mode=1)
    a.SL_in = a.SL_out + 52 * 4                          # the appended scores would overwrite the stored list
    assert lib.pafu_step(None, ctypes.byref(a)) == -6
    a = _fake_step(A)
    a.O = a.V_chunk
    assert lib.pafu_step(None, ctypes.byref(a)) == -6
    a = _fake_step(A)
    a.V_out = a.K_out + 16                               # overlapping rows of the two output slabs
    assert lib.pafu_step(None, ctypes.byref(a)) == -6
    # multi-layer steps reorder the stages across layers: a buffer shared between layers is an error
    for field in ("scores", "ids", "SL_out", "K_out", "O"):
        pair = (binding.pafu_step_args * 2)(_fake_step(A), _fake_step(A + 0x8000000))
        setattr(pair[1], field, getattr(pair[0], field))
        assert lib.pafu_step_layers(None, pair, 2) == -6, field
    pair = (binding.pafu_step_args * 2)(_fake_step(A), _fake_step(A + 0x8000000))
    pair[1].K_cache = pair[0].K_out                      # one layer's output is another layer's input
    assert lib.pafu_step_layers(None, pair, 2) == -6
    assert lib.pafu_step_layers_shared(None, pair, 2, 1) == -6
    pair = (binding.pafu_step_args * 2)(_fake_step(A), _fake_step(A + 0x8000000))
    pair[0].O = pair[1].O
    assert lib.pafu_step_layers_shared(None, pair, 2, 1) == -6


def test_attention_rejects_row_strides_its_tile_offsets_cannot_hold():
    f = binding.library().pafu_chunk_attention

    def call(ld_c=256, ld_n=256, n_kept=100):
        return f(None, A, 64, A + 0x10000000, A + 0x20000000, n_kept, A + 0x30000000, A + 0x40000000, 64, 2, 128, 256,
                 ld_c, ld_n, 256, 64, 0.0, A + 0x50000000, 0, None, 0)
    assert call(ld_c=(1 << 25)) == -2
    assert call(ld_n=(1 << 25)) == -2
    assert call(ld_c=(1 << 25) - 8, n_kept=1) in (0, -7)       # accepted (a launch error without a GPU)


def test_new_entry_points_reject_bad_arguments():
    lib = binding.library()
    # pafu_score_static: same checks as pafu_score, plus the limit of its static scratch
    f = lib.pafu_score_static

    def call(x0=A, T=10, Fs=128, ld=128, dt=0, W1=A + 0x100000, W2=A + 0x200000, M=32, no=3, act=0, out=A + 0x300000):
        return f(None, x0, None, None, 1, T, Fs, ld, dt, W1, None, W2, None, M, no, act, out)
    assert call(x0=None) == -1
    assert call(M=0) == -2
    assert call(dt=2) == -3                        # the 8-bit format is for K/V tensors only
    assert call(ld=132) == -4
    assert call(M=8193) == -5                      # beyond the static scratch
    # pafu_compact_kv_counted
    g = lib.pafu_compact_kv_counted
    ok = dict(K=A, V=A + 0x100000, SL=None, ld=1536, n=100, ids=A + 0x200000, cnt=A + 0x600000, mx=50, N=12, D=128, dt=0,
              Ko=A + 0x300000, Vo=A + 0x400000, SLo=None, ldo=1536)

    def ccall(**kw):
        a = dict(ok); a.update(kw)
        return g(None, a["K"], a["V"], a["SL"], a["ld"], a["n"], a["ids"], a["cnt"], a["mx"], a["N"], a["D"], a["dt"],
                 a["Ko"], a["Vo"], a["SLo"], a["ldo"])
    assert ccall(cnt=None) == -1
    assert ccall(mx=101) == -2
    assert ccall(Ko=A) == -6
    assert ccall(dt=9) == -3
    assert ccall(mx=0, cnt=None, K=None) == 0
    # pafu_quantize_kv / pafu_dequantize_kv
    q = lib.pafu_quantize_kv
    assert q(None, None, A, 256, 10, 2, 128, 0, 0, A + 0x200000, A + 0x300000, 256) == -1
    assert q(None, A, A + 0x100000, 256, 10, 2, 127, 0, 0, A + 0x200000, A + 0x300000, 256) == -2     # N * D not a multiple of 8
    assert q(None, A, A + 0x100000, 256, 10, 2, 128, 65, 0, A + 0x200000, A + 0x300000, 256) == -2    # scale exponent
    assert q(None, A, A + 0x100000, 256, 10, 2, 128, 0, 0, A + 0x200000, A + 0x300000, 264) == -4     # byte stride % 16
    assert q(None, A, A + 0x100000, 256, 0, 2, 128, 0, 0, None, None, 256) == 0
    assert lib.pafu_dequantize_kv(None, A, A + 0x100000, 256, 10, 2, 128, 0, 0, A + 0x200000, A + 0x200100, 256) == -6
    # a step with the 8-bit cache: head dim 128 only, and the output slab counts with the chunk rows
    a = _fake_step(A, N=2, D=64)
    a.kv_dtype = 2
    assert lib.pafu_step(None, ctypes.byref(a)) == -2
    a = _fake_step(A, N=1, D=128)
    a.kv_dtype = 7
    assert lib.pafu_step(None, ctypes.byref(a)) == -3
    a = _fake_step(A, N=1, D=128)
    a.kv_dtype = 2
    a.Q = a.K_out + 50 * 128 + 16 * 128                  # inside the rows where the quantised chunk goes (SINGLE mode too)
    assert lib.pafu_step(None, ctypes.byref(a)) == -6
    assert lib.pafu_study_build() == 0


def test_sse_rejects_bad_arguments_and_reports_its_workspace():
    lib = binding.library()
    assert binding.pafu_sse_workspace_bytes(1000, 3) == 16 * 3 * 1000
    f = lib.pafu_sse_score
    ok = dict(Q=A, K=A + 0x100000, L=100, N=2, D=64, ldq=128, ldk=128, LB=10, sc=0.0, out=A + 0x200000,
              ws=A + 0x300000, wsb=16 * 2 * 100)

    def call(**kw):
        a = dict(ok); a.update(kw)
        return f(None, a["Q"], a["K"], a["L"], a["N"], a["D"], a["ldq"], a["ldk"], a["LB"], a["sc"], a["out"], a["ws"],
                 a["wsb"])

    assert call(D=96) == -2
    assert call(LB=0) == -2
    assert call(L=-1) == -2
    assert call(L=0) == 0                          # nothing to do
    assert call(Q=None) == -1
    assert call(out=None) == -1
    assert call(ldq=100) == -2                     # stride shorter than a token
    assert call(ldq=132) == -4
    assert call(wsb=100) == -5
    assert call(ws=None) == -5
    assert call(out=A + 0x300000) == -6            # output inside the workspace
