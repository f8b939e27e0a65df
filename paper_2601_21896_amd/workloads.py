"""Seeded synthetic inputs for the PaFu-KV chunk step.

This module only draws numbers and lays them out; it holds none of the method's
arithmetic (no scoring, selection, gathering or attention), so both the device
path and the CPU checker may be fed from it.

Shapes follow the paper's Appendix A (1560 latent tokens per frame, chunks of 3
frames = 4680 tokens, a 21-frame cache = 32760 tokens, 12 heads x 128).  The
synthetic tensors stand in for real Wan2.1 activations, which need the model's
weights.  Value distributions: N(0,1) features / Q / K / V, a per-channel key
scale drawn from U[0.5, 2], N(0, 0.02^2) head weights, zero biases, and a +2
offset on every feature channel of 10% of the cached tokens so that salience is
structured.

All tensors are returned as float32 NumPy arrays.  For a bf16 workload every
value is first rounded to the nearest bf16 (ties to even), so a later cast to
bf16 on the device is exact and the CPU checker sees the same numbers.
"""

from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

BASE_SEED = 260121896


@dataclass(frozen=True)
class LayerConfig:
    name: str
    config_id: int
    N: int                 # attention heads
    D: int                 # head dim
    frame_tokens: int      # latent tokens per frame
    chunk_frames: int
    cache_frames: int
    k: int                 # budget: cached tokens kept
    M: int                 # S-MLP hidden width
    n_out: int             # S-MLP outputs (averaged)
    dtype: str             # "bf16" or "f32"
    salient_frac: float

    @property
    def H(self) -> int:
        return self.N * self.D

    @property
    def Lc(self) -> int:
        return self.frame_tokens * self.chunk_frames

    @property
    def n(self) -> int:
        return self.frame_tokens * self.cache_frames


C0 = LayerConfig("C0-tiny", 0, N=2, D=64, frame_tokens=64, chunk_frames=1, cache_frames=4,
                 k=128, M=32, n_out=1, dtype="f32", salient_frac=0.0)
C1 = LayerConfig("C1-wan1.3b-layer", 1, N=12, D=128, frame_tokens=1560, chunk_frames=3,
                 cache_frames=21, k=16380, M=256, n_out=1, dtype="bf16", salient_frac=0.1)
C4 = LayerConfig("C4-wan14b-720p-layer", 4, N=40, D=128, frame_tokens=3600, chunk_frames=3,
                 cache_frames=21, k=22680, M=512, n_out=1, dtype="bf16", salient_frac=0.1)
# C2 = 30 independent layers at C1 shapes (layer l uses seed + 1000 l);
# C3 = 60-chunk rollout at C1 shapes with k = 8 frames (chunk t uses seed + 1000 t).
C2_LAYERS = 30
C3_CHUNKS = 60
C3_K = 8 * 1560
C3_K_SWEEP = (8190, 16380, 32760)

CONFIGS = {"C0": C0, "C1": C1, "C4": C4}


def scaled(cfg: LayerConfig, **kw) -> LayerConfig:
    """A copy of cfg with some fields replaced (reduced sizes for parity tests)."""
    return replace(cfg, **kw)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result stays float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    out = ((u + r) & np.uint32(0xFFFF0000)).view(np.float32)
    return out


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of bf16-representable float32 values."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def _q(cfg: LayerConfig, a: np.ndarray) -> np.ndarray:
    return round_to_bf16(a) if cfg.dtype == "bf16" else np.ascontiguousarray(a, dtype=np.float32)


def _normal(rng, shape, scale=1.0):
    a = rng.standard_normal(size=shape, dtype=np.float32)
    if scale != 1.0:
        a *= np.float32(scale)
    return a


def make_head_weights(cfg: LayerConfig, rng, F: int | None = None, bias: bool = False):
    """S-MLP weights: W1 [M, F], W2 [n_out, M] ~ N(0, 0.02^2); biases zero unless bias=True
    (then ~ N(0, 0.02^2) as well).  b1, b2 and W2 stay fp32; W1 takes the config's dtype."""
    F = cfg.H if F is None else F
    W1 = _q(cfg, _normal(rng, (cfg.M, F), 0.02))
    W2 = _normal(rng, (cfg.n_out, cfg.M), 0.02)
    if bias:
        b1 = _normal(rng, (cfg.M,), 0.02)
        b2 = _normal(rng, (cfg.n_out,), 0.02)
    else:
        b1 = np.zeros((cfg.M,), np.float32)
        b2 = np.zeros((cfg.n_out,), np.float32)
    return W1, b1, W2, b2


def salient_mask(cfg: LayerConfig, rng, n: int, structure: str = "uniform") -> np.ndarray:
    """Boolean [n]: which cached tokens get the feature offset.

    "uniform": exactly floor(frac*n) tokens anywhere (worst case for gather locality).
    "coherent": the same floor(frac*frame_tokens) patch positions in every cached frame
                (video salience is spatially persistent)."""
    mask = np.zeros(n, dtype=bool)
    if cfg.salient_frac <= 0.0 or n == 0:
        return mask
    if structure == "uniform":
        m = int(np.floor(cfg.salient_frac * n))
        mask[rng.permutation(n)[:m]] = True
    elif structure == "coherent":
        ft = cfg.frame_tokens
        m = int(np.floor(cfg.salient_frac * ft))
        pos = rng.permutation(ft)[:m]
        for f in range((n + ft - 1) // ft):
            p = pos + f * ft
            mask[p[p < n]] = True
    else:
        raise ValueError(structure)
    return mask


def make_layer_inputs(cfg: LayerConfig, seed: int | None = None, structure: str = "uniform",
                      bias: bool = False, n_cache: int | None = None, weights: bool = True,
                      features: bool = True) -> dict:
    """All tensors of one layer's chunk step, drawn in a fixed order from one seed.

    Order: W1, b1, W2, b2, X_cache, X_chunk, salient mask, channel scale, K_cache, V_cache,
    Q, K_chunk, V_chunk.  `weights=False` / `features=False` skip (and do not draw) those
    groups - used by the rollout, whose weights come from the base seed.
    """
    seed = BASE_SEED + cfg.config_id if seed is None else seed
    rng = np.random.Generator(np.random.PCG64(seed))
    n = cfg.n if n_cache is None else n_cache
    N, D, H, Lc = cfg.N, cfg.D, cfg.H, cfg.Lc
    out: dict = {"cfg": cfg, "seed": seed, "n": n}
    if weights:
        out["W1"], out["b1"], out["W2"], out["b2"] = make_head_weights(cfg, rng, bias=bias)
    if features:
        Xc = _normal(rng, (n, H))
        Xn = _normal(rng, (Lc, H))
        mask = salient_mask(cfg, rng, n, structure)
        Xc[mask] += np.float32(2.0)
        out["X_cache"], out["X_chunk"], out["salient"] = _q(cfg, Xc), _q(cfg, Xn), mask
    c = rng.uniform(0.5, 2.0, size=(H,)).astype(np.float32)
    out["k_scale"] = c
    out["K_cache"] = _q(cfg, _normal(rng, (n, H)) * c[None, :]).reshape(n, N, D)
    out["V_cache"] = _q(cfg, _normal(rng, (n, H))).reshape(n, N, D)
    out["Q"] = _q(cfg, _normal(rng, (Lc, H))).reshape(Lc, N, D)
    out["K_chunk"] = _q(cfg, _normal(rng, (Lc, H)) * c[None, :]).reshape(Lc, N, D)
    out["V_chunk"] = _q(cfg, _normal(rng, (Lc, H))).reshape(Lc, N, D)
    return out


def make_chunk_inputs(cfg: LayerConfig, t: int, base_seed: int | None = None) -> dict:
    """Chunk t of a rollout: features, Q, K, V of the new chunk only (seed + 1000 t)."""
    base = BASE_SEED + 3 if base_seed is None else base_seed
    d = make_layer_inputs(cfg, seed=base + 1000 * t, n_cache=0, weights=False)
    return {k_: d[k_] for k_ in ("X_chunk", "Q", "K_chunk", "V_chunk", "seed")}


def make_rollout_weights(cfg: LayerConfig, base_seed: int | None = None, bias: bool = False):
    base = BASE_SEED + 3 if base_seed is None else base_seed
    rng = np.random.Generator(np.random.PCG64(base))
    return make_head_weights(cfg, rng, bias=bias)
