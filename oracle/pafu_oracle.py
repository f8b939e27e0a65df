"""fp64 CPU oracle for the PaFu-KV chunk step: score -> select -> compact -> attention.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain statement of what the
hot path computes.  It shares no code with the HIP library, imports nothing from
the product package, and must never be called from a product code path: only the
tests, the smoke check and the benchmark's CPU-baseline leg may use it.

Every function is the definition written out (none of the four stages is an
approximation of something else), in float64, with NumPy matmul / sort as the
only library steps.  There is no tiling, no online softmax and no fusion.

Inputs are whatever values the device path sees, widened exactly: a bf16 tensor
arrives here as float32/float64 values that are exactly representable in bf16.

Pins (tests/test_oracle_*.py): every function below is pinned by closed forms, value tables of the number format,
brute force on tiny inputs, invariants, or reduction to an independent library
routine.  The paper prints no worked numeric example for any stage, so no pin
is a printed value.

Notation follows the paper: N heads, D head dim, L_B block length, k budget,
SL salience score list, KV cache.  Layouts are token-major: Q/K/V `[tokens, N, D]`.
"""

from __future__ import annotations

import math

import numpy as np
from scipy.special import erf as _erf

__all__ = [
    "smlp_score",
    "select_topk",
    "compact_kv",
    "chunk_attention",
    "step_single",
    "RolloutState",
    "rollout_step",
    "step_single_shared",
    "rollout_step_shared",
    "sse_score",
    "quantise_e4m3",
    "dequantise_e4m3",
    "rollout_step_fp8",
]


# --------------------------------------------------------------------------------------
# Salience Estimation Head (S-MLP)
# --------------------------------------------------------------------------------------
def smlp_score(X, W1, b1, W2, b2, act: str = "silu") -> np.ndarray:
    """Per-token salience score of the S-MLP.

    Appendix A ("S-MLP"): two linear layers with a SiLU in between, then the mean
    over the output dimension; Sec. 3.3 / 3.4: the head maps per-token features to
    one scalar per token.

    X  [T, F]      per-token features (the caller concatenates Q|K|V when the
                   paper-form input is wanted)
    W1 [M, F], b1 [M] or None      first linear layer, out-features x in-features
    W2 [n_out, M], b2 [n_out] or None
    act: "silu" (the paper's) or "gelu_erf" (exact erf GELU, the benchmark
         description's fallback wording)
    returns s [T] float64
    """
    X = np.asarray(X, dtype=np.float64)
    W1 = np.asarray(W1, dtype=np.float64)
    W2 = np.asarray(W2, dtype=np.float64)
    T, F = X.shape
    M = W1.shape[0]
    n_out = W2.shape[0]
    assert W1.shape == (M, F) and W2.shape == (n_out, M)
    h = X @ W1.T
    if b1 is not None:
        h = h + np.asarray(b1, dtype=np.float64)[None, :]
    if act == "silu":
        a = h * (1.0 / (1.0 + np.exp(-h)))
    elif act == "gelu_erf":
        a = 0.5 * h * (1.0 + _erf(h / math.sqrt(2.0)))
    else:
        raise ValueError(act)
    y = a @ W2.T
    if b2 is not None:
        y = y + np.asarray(b2, dtype=np.float64)[None, :]
    return y.sum(axis=1) / float(n_out)


# --------------------------------------------------------------------------------------
# Top-k retention
# --------------------------------------------------------------------------------------
def select_topk(scores_f32, k: int, n_pinned: int = 0) -> np.ndarray:
    """Indices of the k most salient tokens, ascending.

    Sec. 3.4 (inference paragraph) and Alg. 2: keep the top-k of the score list.
    Total order used: higher score first; equal scores -> lower token index first;
    -0.0 equals +0.0; NaN ranks below -inf.  k >= n keeps everything (eviction only
    happens once the cache exceeds its budget).  The decision is taken on the fp32
    score values exactly as given.

    n_pinned (frame sink, Sec. 4 "Experimental Implementation" and the frame-sink
    ablation): the first n_pinned tokens of the cache are never evicted and count
    towards the budget.  The retained set is that prefix plus the k - n_pinned most
    salient of the other tokens; a budget smaller than the prefix keeps the first k
    tokens of it.  The paper takes the mechanism from prior work without describing
    it; this is the reading taken here.

    returns int32 [min(k, n)], sorted ascending.
    """
    s = np.asarray(scores_f32, dtype=np.float32)
    assert s.ndim == 1
    n = s.shape[0]
    k = int(k)
    n_pinned = max(0, min(int(n_pinned), n))
    assert k >= 0
    if k >= n:
        return np.arange(n, dtype=np.int32)
    if n_pinned >= k:
        return np.arange(k, dtype=np.int32)
    if n_pinned > 0:
        rest = select_topk(s[n_pinned:], k - n_pinned) + n_pinned
        return np.concatenate([np.arange(n_pinned, dtype=np.int32), rest.astype(np.int32)])
    isnan = np.isnan(s)
    val = s.astype(np.float64)
    val = np.where(isnan, 0.0, val) + 0.0  # x + 0.0 turns -0.0 into +0.0
    idx = np.arange(n)
    # lexsort: last key is the primary one.  NaN last, then value descending, then index.
    order = np.lexsort((idx, -val, isnan.astype(np.int8)))
    keep = order[:k]
    return np.sort(keep).astype(np.int32)


# --------------------------------------------------------------------------------------
# Cache update: Select(KV; ids), Select(SL; ids)
# --------------------------------------------------------------------------------------
def compact_kv(K, V, SL, ids):
    """Alg. 2, cache update: the retained rows of K, V and of the score list, in
    the order ids gives (bit copies; dtype preserved)."""
    ids = np.asarray(ids, dtype=np.int64)
    K = np.asarray(K)
    V = np.asarray(V)
    SL = np.asarray(SL)
    return K[ids].copy(), V[ids].copy(), SL[ids].copy()


# --------------------------------------------------------------------------------------
# Attention of the chunk's queries over retained cache + chunk
# --------------------------------------------------------------------------------------
def chunk_attention(Q, Kc, Vc, Kn, Vn, block_len: int, scale: float | None = None,
                    rows=None, return_P: bool = False):
    """O = softmax(Q [Kc;Kn]^T / sqrt(D) + mask) [Vc;Vn]   per head.

    Sec. 3.2: P = softmax(Q K^T / sqrt(D)); blocks of length L_B with
    b(i) = floor(i / L_B).  Every retained cache key is visible to every chunk
    query; chunk key j is visible to chunk query i iff b(j) <= b(i) (block-causal;
    L_B >= chunk length means no mask, the paper's setting, App. A).

    Q  [Lq, N, D]   chunk queries        Kn, Vn [Lc, N, D]  the chunk's own keys/values
    Kc, Vc [n, N, D] retained cache (n may be 0)
    rows: optional 1-D array of query indices to compute (others are not returned)
    returns O [len(rows) or Lq, N, D] float64  (and P [N, rows, n+Lc] if return_P)
    """
    Q = np.asarray(Q, dtype=np.float64)
    Kc = np.asarray(Kc, dtype=np.float64)
    Vc = np.asarray(Vc, dtype=np.float64)
    Kn = np.asarray(Kn, dtype=np.float64)
    Vn = np.asarray(Vn, dtype=np.float64)
    Lq, N, D = Q.shape
    n = Kc.shape[0]
    Lc = Kn.shape[0]
    assert block_len >= 1
    if scale is None:
        scale = 1.0 / math.sqrt(D)
    if rows is None:
        rows = np.arange(Lq)
    rows = np.asarray(rows, dtype=np.int64)
    K_all = np.concatenate([Kc.reshape(n, N, D), Kn], axis=0)
    V_all = np.concatenate([Vc.reshape(n, N, D), Vn], axis=0)
    # visibility[i, j] for chunk keys
    bq = rows // block_len
    bk = np.arange(Lc) // block_len
    vis_chunk = bk[None, :] <= bq[:, None]
    vis = np.concatenate([np.ones((rows.shape[0], n), dtype=bool), vis_chunk], axis=1)
    O = np.empty((rows.shape[0], N, D), dtype=np.float64)
    P_all = np.empty((N, rows.shape[0], n + Lc), dtype=np.float64) if return_P else None
    for h in range(N):
        z = (Q[rows, h, :] @ K_all[:, h, :].T) * scale
        z = np.where(vis, z, -np.inf)
        m = z.max(axis=1, keepdims=True)
        p = np.exp(z - m)
        p = p / p.sum(axis=1, keepdims=True)
        O[:, h, :] = p @ V_all[:, h, :]
        if return_P:
            P_all[h] = p
    if return_P:
        return O, P_all
    return O


# --------------------------------------------------------------------------------------
# One chunk step
# --------------------------------------------------------------------------------------
def step_single(X_cache, X_chunk, W1, b1, W2, b2, K_cache, V_cache, Q, K_chunk, V_chunk,
                k: int, block_len: int, act: str = "silu", forced_scores_f32=None, n_pinned: int = 0):
    """One step in SINGLE mode: score cached and new tokens, select the top-k cached
    tokens on the fresh cache scores, compact, attend (Alg. 2 order of operations;
    Sec. 3.4).

    forced_scores_f32: optional fp32 [n + Lc] vector used for selection instead of
    the oracle's own rounded scores (teacher-forced parity: the device's scores are
    fed in so that select/compact/attention can be compared exactly).

    returns dict(scores [n+Lc] f64, ids, K_kept, V_kept, SL_kept, O)
    """
    n = X_cache.shape[0]
    s_cache = smlp_score(X_cache, W1, b1, W2, b2, act) if n else np.zeros(0)
    s_chunk = smlp_score(X_chunk, W1, b1, W2, b2, act)
    s = np.concatenate([s_cache, s_chunk])
    s32 = s.astype(np.float32) if forced_scores_f32 is None else np.asarray(forced_scores_f32, np.float32)
    ids = select_topk(s32[:n], k, n_pinned)
    Kk, Vk, SLk = compact_kv(K_cache, V_cache, s32[:n], ids)
    O = chunk_attention(Q, Kk, Vk, K_chunk, V_chunk, block_len)
    return dict(scores=s, ids=ids, K_kept=Kk, V_kept=Vk, SL_kept=SLk, O=O)


class RolloutState:
    """Cache state between chunks: K, V [n, N, D], SL [n] fp32, all caller-visible."""

    def __init__(self, N: int, D: int, kv_dtype=np.float32):
        self.K = np.zeros((0, N, D), dtype=kv_dtype)
        self.V = np.zeros((0, N, D), dtype=kv_dtype)
        self.SL = np.zeros((0,), dtype=np.float32)

    @property
    def n(self) -> int:
        return self.K.shape[0]

    def copy(self) -> "RolloutState":
        c = RolloutState.__new__(RolloutState)
        c.K, c.V, c.SL = self.K.copy(), self.V.copy(), self.SL.copy()
        return c


def rollout_step(state: RolloutState, X_chunk, W1, b1, W2, b2, Q, K_chunk, V_chunk,
                 k: int, block_len: int, act: str = "silu", forced_chunk_scores_f32=None, n_pinned: int = 0,
                 rows=None):
    """One chunk of a rollout (Sec. 3.4 inference paragraph; Alg. 2).

    The chunk's scores join the stored ones after its step, so the next step's
    top-k runs over retained + that chunk and old and new tokens compete; stored
    scores are never refreshed.  Order: score the chunk; select on the stored SL;
    compact; attend over retained + chunk; append chunk K/V and its scores.

    rows: optional query rows of the attention output to compute (full-size checks sample them; the
    cache update does not depend on it).

    returns dict(s_chunk f64, ids, O); mutates state.
    """
    s_chunk = smlp_score(X_chunk, W1, b1, W2, b2, act)
    s32 = (s_chunk.astype(np.float32) if forced_chunk_scores_f32 is None
           else np.asarray(forced_chunk_scores_f32, np.float32))
    ids = select_topk(state.SL, k, n_pinned)
    Kk, Vk, SLk = compact_kv(state.K, state.V, state.SL, ids)
    O = chunk_attention(Q, Kk, Vk, K_chunk, V_chunk, block_len, rows=rows)
    state.K = np.concatenate([Kk, np.asarray(K_chunk, dtype=Kk.dtype)], axis=0)
    state.V = np.concatenate([Vk, np.asarray(V_chunk, dtype=Vk.dtype)], axis=0)
    state.SL = np.concatenate([SLk, s32]).astype(np.float32)
    return dict(s_chunk=s_chunk, ids=ids, O=O)


# --------------------------------------------------------------------------------------
# 8-bit storage of the K/V cache (beyond the paper: App. A states no storage precision)
# --------------------------------------------------------------------------------------
E4M3_MAX = 448.0          # largest finite magnitude: 1.75 * 2^8
E4M3_MIN_NORMAL = 2.0 ** -6
E4M3_SUBNORMAL_STEP = 2.0 ** -9


def quantise_e4m3(x, scale_log2: int = 0) -> np.ndarray:
    """Codes of x / 2^scale_log2 in the 8-bit floating-point format E4M3 (1 sign, 4 exponent bits with bias 7,
    3 mantissa bits; no infinities; exponent 15 with mantissa 7 is NaN; the "fn" variant of the OCP 8-bit
    floating-point specification).  Reading taken for the cache (the paper gives none): one power-of-two scale per
    tensor chosen by the caller, round to nearest with ties to the even mantissa, magnitudes beyond 448 saturate
    to 448, NaN stays NaN, the sign of zero is kept.

    The value grid: for exponent field E >= 1, 2^(E-7) (1 + M/8); for E = 0, 2^-6 (M/8).  Rounding is done by
    scaling to the grid's local step and rounding to the nearest integer (ties to even), which is exact in
    float64 for every finite input.

    returns uint8 codes, same shape as x.
    """
    v = np.asarray(x, dtype=np.float64) / (2.0 ** int(scale_log2))
    sign = np.signbit(v)
    a = np.minimum(np.abs(v), E4M3_MAX)
    nan = np.isnan(v)
    a = np.where(nan, 0.0, a)
    # local step of the grid: 2^(floor(log2 a) - 3) for normals, 2^-9 below the smallest normal
    with np.errstate(divide="ignore"):
        ex = np.floor(np.log2(np.where(a > 0, a, 1.0)))
    ex = np.maximum(ex, -6.0)
    step = 2.0 ** (ex - 3.0)
    q = np.rint(a / step) * step              # np.rint rounds halves to even; a / step is exact (power-of-two step)
    # q may have moved up to the next binade (mantissa 8/8): recompute exponent and mantissa from q itself
    with np.errstate(divide="ignore"):
        eq = np.floor(np.log2(np.where(q > 0, q, 1.0)))
    normal = q >= E4M3_MIN_NORMAL
    E = np.where(normal, eq + 7.0, 0.0)
    M = np.where(normal, q / 2.0 ** eq * 8.0 - 8.0, q / E4M3_SUBNORMAL_STEP)
    code = (E.astype(np.int64) << 3) | M.astype(np.int64)
    code = np.where(nan, 0x7F, code)
    code = code | (sign.astype(np.int64) << 7)
    return code.astype(np.uint8)


def dequantise_e4m3(codes, scale_log2: int = 0) -> np.ndarray:
    """Values of E4M3 codes times 2^scale_log2, float64 (exact)."""
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    E = (c >> 3) & 0xF
    M = c & 7
    mag = np.where(E > 0, 2.0 ** (E - 7.0) * (1.0 + M / 8.0), E4M3_MIN_NORMAL * (M / 8.0))
    mag = np.where((E == 15) & (M == 7), np.nan, mag)
    return np.where((c >> 7) == 1, -mag, mag) * (2.0 ** int(scale_log2))


def rollout_step_fp8(state: RolloutState, X_chunk, W1, b1, W2, b2, Q, K_chunk, V_chunk, k: int, block_len: int,
                     k_scale_log2: int, v_scale_log2: int, act: str = "silu", forced_chunk_scores_f32=None,
                     n_pinned: int = 0, rows=None):
    """rollout_step with the cache held as E4M3 codes (state.K / state.V are uint8 arrays).

    The chunk's K/V are quantised when they enter the step, so the chunk's queries attend over exactly the values
    that later steps will find in the cache; selection and compaction move codes; attention runs on the
    dequantised values.  returns dict(s_chunk f64, ids, O, K_codes, V_codes of the chunk); mutates state.
    """
    s_chunk = smlp_score(X_chunk, W1, b1, W2, b2, act)
    s32 = (s_chunk.astype(np.float32) if forced_chunk_scores_f32 is None
           else np.asarray(forced_chunk_scores_f32, np.float32))
    ids = select_topk(state.SL, k, n_pinned)
    Kk, Vk, SLk = compact_kv(state.K, state.V, state.SL, ids)
    Kq = quantise_e4m3(K_chunk, k_scale_log2)
    Vq = quantise_e4m3(V_chunk, v_scale_log2)
    O = chunk_attention(Q, dequantise_e4m3(Kk, k_scale_log2), dequantise_e4m3(Vk, v_scale_log2),
                        dequantise_e4m3(Kq, k_scale_log2), dequantise_e4m3(Vq, v_scale_log2), block_len, rows=rows)
    state.K = np.concatenate([Kk, Kq], axis=0)
    state.V = np.concatenate([Vk, Vq], axis=0)
    state.SL = np.concatenate([SLk, s32]).astype(np.float32)
    return dict(s_chunk=s_chunk, ids=ids, O=O, K_codes=Kq, V_codes=Vq)


# --------------------------------------------------------------------------------------
# Final-layer head, indices shared by all layers (Sec. 3.3)
# --------------------------------------------------------------------------------------
def step_single_shared(X_cache, X_chunk, W1, b1, W2, b2, layers, k: int, block_len: int, act: str = "silu",
                       forced_scores_f32=None, n_pinned: int = 0, rows=None):
    """SINGLE-mode step of several layers with ONE index list (Sec. 3.3: the head reads the final layer only and
    its top-k indices update the caches of all layers).

    X_cache / X_chunk are the index layer's features; `layers` is a list of dicts with K_cache, V_cache, Q,
    K_chunk, V_chunk (one per layer, same token counts); rows: optional query rows of O to compute.

    returns dict(scores f64 [n+Lc], ids, SL_kept, layers=[dict(K_kept, V_kept, O)])
    """
    n = X_cache.shape[0]
    s_cache = smlp_score(X_cache, W1, b1, W2, b2, act) if n else np.zeros(0)
    s = np.concatenate([s_cache, smlp_score(X_chunk, W1, b1, W2, b2, act)])
    s32 = s.astype(np.float32) if forced_scores_f32 is None else np.asarray(forced_scores_f32, np.float32)
    ids = select_topk(s32[:n], k, n_pinned)
    outs = []
    SLk = s32[:n][ids]
    for L in layers:
        assert L["K_cache"].shape[0] == n
        Kk, Vk, _ = compact_kv(L["K_cache"], L["V_cache"], s32[:n], ids)
        outs.append(dict(K_kept=Kk, V_kept=Vk,
                         O=chunk_attention(L["Q"], Kk, Vk, L["K_chunk"], L["V_chunk"], block_len, rows=rows)))
    return dict(scores=s, ids=ids, SL_kept=SLk, layers=outs)


def rollout_step_shared(states, index_layer: int, X_chunk, W1, b1, W2, b2, chunks, k: int, block_len: int,
                        act: str = "silu", forced_chunk_scores_f32=None, n_pinned: int = 0):
    """One chunk of a multi-layer rollout with shared indices (Sec. 3.3; Alg. 2): the stored score list lives with
    the index layer; its top-k decides which rows every layer keeps; each layer attends over its own retained rows
    plus its own chunk rows and appends them; the chunk's scores (from the index layer's features) join the list.

    states: one RolloutState per layer (only states[index_layer].SL is used); chunks: per layer dict(Q, K_chunk,
    V_chunk).  returns dict(s_chunk f64, ids, O=[per layer]); mutates the states.
    """
    s_chunk = smlp_score(X_chunk, W1, b1, W2, b2, act)
    s32 = (s_chunk.astype(np.float32) if forced_chunk_scores_f32 is None
           else np.asarray(forced_chunk_scores_f32, np.float32))
    SL = states[index_layer].SL
    ids = select_topk(SL, k, n_pinned)
    Os = []
    for st, c in zip(states, chunks):
        assert st.K.shape[0] == SL.shape[0]
        Kk, Vk = st.K[ids].copy(), st.V[ids].copy()
        Os.append(chunk_attention(c["Q"], Kk, Vk, c["K_chunk"], c["V_chunk"], block_len))
        st.K = np.concatenate([Kk, np.asarray(c["K_chunk"], dtype=Kk.dtype)], axis=0)
        st.V = np.concatenate([Vk, np.asarray(c["V_chunk"], dtype=Vk.dtype)], axis=0)
    states[index_layer].SL = np.concatenate([SL[ids], s32]).astype(np.float32)
    return dict(s_chunk=s_chunk, ids=ids, O=Os)


# --------------------------------------------------------------------------------------
# Spatialtemporal-balanced Salience Estimation (teacher-side score), Sec. 3.2, Eq. 4-5
# --------------------------------------------------------------------------------------
def sse_score(Q, K, block_len: int, scale: float | None = None, return_parts: bool = False):
    """Salience score of every key from the attention weights of a bidirectional pass.

    Sec. 3.2: P = softmax(Q K^T / sqrt(D)) over the FULL key axis, per head.  With blocks of
    L_B tokens, b(i) = floor(i / L_B), the queries of key j fall into three sets: those in a
    later block than j ("low": j < l(i)), in j's own block ("diag") and in an earlier block
    ("up": j >= h(i)).  Eq. 4: per set, the maximum of P[h, i, j] over its queries, then the
    mean over heads.  Eq. 5: the score is the mean of the parts that exist for the key -
    (diag + low) / 2 in the first block, (up + diag + low) / 3 in the middle, (diag + up) / 2
    in the last block.

    Readings: the sum in Eq. 4 runs over heads; the block-wise listing in the appendix differs
    from Eq. 4-5 (no softmax, mean over heads before the maximum) and is not followed; a part
    "exists" for key j iff its query set is non-empty, which is Eq. 5 whenever the sequence is a
    whole number (>= 2) of blocks and extends it to a single block (score = diag) and to a
    ragged last block.

    Q, K: [L, N, D].  returns s [L] float64 (and low, diag, up [L] with return_parts; a part
    whose query set is empty is 0 there).
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    L, N, D = Q.shape
    assert K.shape == (L, N, D) and block_len >= 1
    scale = 1.0 / math.sqrt(D) if scale is None else float(scale)
    blk = np.arange(L) // int(block_len)
    later = blk[:, None] > blk[None, :]      # [i, j]: query i sits in a later block than key j
    same = blk[:, None] == blk[None, :]
    earlier = blk[:, None] < blk[None, :]
    low = np.zeros(L)
    diag = np.zeros(L)
    up = np.zeros(L)
    for h in range(N):
        z = (Q[:, h, :] @ K[:, h, :].T) * scale            # [i, j]
        z -= z.max(axis=1, keepdims=True)
        P = np.exp(z)
        P /= P.sum(axis=1, keepdims=True)
        low += np.where(later, P, 0.0).max(axis=0)          # P > 0, so an empty set gives 0
        diag += np.where(same, P, 0.0).max(axis=0)
        up += np.where(earlier, P, 0.0).max(axis=0)
    low /= N
    diag /= N
    up /= N
    has_low = blk < blk[-1]
    has_up = blk > 0
    s = (diag + np.where(has_low, low, 0.0) + np.where(has_up, up, 0.0)) / (1.0 + has_low + has_up)
    if return_parts:
        return s, low, diag, up
    return s
