"""Seeded synthetic KV / window-query generators for the five benchmark shapes.

This module holds no arithmetic of the compression method itself: it only
draws random tensors with the structure the paper reports for real models
(concentrated attention in deep layers, many near-parallel key/value vectors
in shallow layers; Sec. "Preliminary Experiment") at Llama-3-8B / Mistral-7B
head shapes (Sec. "Experimental Setup": 32 query heads; 8 KV heads, 4 query
heads per KV head).  Both the CPU oracle's tests and the GPU path read the
same bit patterns produced here.

Every tensor is returned in its *device representation*:
  f32  -> numpy float32
  f16  -> numpy float16
  bf16 -> numpy uint16 (upper half of the float32 pattern, round-to-nearest-even)
``to_f64`` converts a device representation exactly to float64.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Iterator, Optional

import numpy as np

HEAD_DIM = 128

# Hyper-parameter table of the paper (Table "Hyper-parameters Used in Experiments").
THETA_K = 0.98
THETA_V = 0.95


def _rng(*key: int) -> np.random.Generator:
    """Counter-based generator keyed by a tuple of small integers."""
    ss = np.random.SeedSequence([int(k) & 0xFFFFFFFF for k in key])
    return np.random.Generator(np.random.Philox(ss))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest even); returns the uint16 patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def cast(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round a float64/float32 array to the device representation of `dtype`."""
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f16":
        return np.ascontiguousarray(x.astype(np.float16))
    if dtype == "bf16":
        return f32_to_bf16_bits(x.astype(np.float32))
    raise ValueError(dtype)


def to_f64(bits: np.ndarray, dtype: str) -> np.ndarray:
    """Exact float64 value of a device representation."""
    if dtype in ("f32", "f16"):
        return bits.astype(np.float64)
    if dtype == "bf16":
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError(dtype)


@dataclass
class Layer:
    """One layer's inputs: K, V [B, Hkv, l, d]; Qw [B, Hkv*h_n, l_w, d]."""
    dtype: str
    K: np.ndarray
    V: np.ndarray
    Qw: np.ndarray
    group_size: int
    window: int
    pool: int
    budget: int            # deep: total kept tokens, window included
    max_codes: int         # shallow: codebook cap
    theta_k: float = THETA_K
    theta_v: float = THETA_V
    name: str = ""
    paths: tuple = ("deep", "shallow")
    meta: Dict = field(default_factory=dict)

    @property
    def batch(self) -> int:
        return self.K.shape[0]

    @property
    def n_kv_heads(self) -> int:
        return self.K.shape[1]

    @property
    def seq_len(self) -> int:
        return self.K.shape[2]

    @property
    def head_dim(self) -> int:
        return self.K.shape[3]


# --------------------------------------------------------------------------
# building blocks
# --------------------------------------------------------------------------

def clustered(rng: np.random.Generator, B: int, H: int, l: int, d: int,
              n_centroids: int, sigma: float, heavy_frac: float = 0.0,
              heavy_scale: float = 4.0, drift_sigma: float = 0.0,
              centroids: Optional[np.ndarray] = None):
    """Tokens = per-head centroid + N(0, sigma^2) (+ a random walk along the
    sequence when drift_sigma > 0); a fraction is scaled to `heavy_scale` x norm.
    Returns (x [B,H,l,d] float32, centroids [B,H,C,d], assignment [B,H,l])."""
    if centroids is None:
        centroids = rng.standard_normal((B, H, n_centroids, d), dtype=np.float32)
    assign = rng.integers(0, n_centroids, size=(B, H, l))
    x = np.take_along_axis(centroids, assign[..., None], axis=2)
    x = x + np.float32(sigma) * rng.standard_normal((B, H, l, d), dtype=np.float32)
    if drift_sigma > 0.0:
        step = np.float32(drift_sigma) * rng.standard_normal((B, H, l, d), dtype=np.float32)
        x = x + np.cumsum(step, axis=2, dtype=np.float32)
    if heavy_frac > 0.0:
        heavy = rng.random((B, H, l)) < heavy_frac
        x = np.where(heavy[..., None], np.float32(heavy_scale) * x, x)
    return x.astype(np.float32), centroids, assign


def window_queries(rng: np.random.Generator, centroids: np.ndarray, group_size: int,
                   window: int, sigma: float) -> np.ndarray:
    """Each window query of each query head sits near a random centroid of its
    KV head, so its logits are large on one cluster and near N(0,1)*|q| elsewhere."""
    B, H, C, d = centroids.shape
    pick = rng.integers(0, C, size=(B, H, group_size * window))
    q = np.take_along_axis(centroids, pick[..., None], axis=2)
    q = q + np.float32(sigma) * rng.standard_normal(q.shape, dtype=np.float32)
    return q.reshape(B, H * group_size, window, d).astype(np.float32)


# --------------------------------------------------------------------------
# the five configurations
# --------------------------------------------------------------------------

def config1(seed: int = 0) -> Layer:
    """1 KV head, 4 query heads, l=512, fp32 N(0,1) K/V, 25 % of the tokens planted
    as near-duplicates (cosine in [0.985, 0.999]) of an earlier non-planted token."""
    l, d, hn, lw = 512, HEAD_DIM, 4, 32
    rng = _rng(1, seed)
    planted = np.zeros(l, dtype=bool)
    cand = rng.permutation(np.arange(1, l))[: l // 4]
    planted[cand] = True
    src = np.zeros(l, dtype=np.int64)
    free = np.flatnonzero(~planted)
    for t in np.flatnonzero(planted):
        earlier = free[free < t]
        src[t] = earlier[rng.integers(0, len(earlier))]

    def tensor(r):
        x = r.standard_normal((l, d))
        cosv = r.uniform(0.985, 0.999, size=l)
        for t in np.flatnonzero(planted):
            b = x[src[t]]
            u = r.standard_normal(d)
            bh = b / np.linalg.norm(b)
            u = u - (u @ bh) * bh
            u /= np.linalg.norm(u)
            x[t] = b + np.tan(np.arccos(cosv[t])) * np.linalg.norm(b) * u
        return x

    K = tensor(_rng(1, seed, 1))[None, None]
    V = tensor(_rng(1, seed, 2))[None, None]
    Q = _rng(1, seed, 3).standard_normal((1, hn, lw, d))
    return Layer("f32", cast(K, "f32"), cast(V, "f32"), cast(Q, "f32"), hn, lw, 7, 128, 128,
                 name="config1", meta={"planted": planted, "src": src})


def _clustered_layer(key, dtype, B, H, l, hn, lw, pool, budget, cap, n_centroids,
                     heavy_frac=0.05, drift_sigma=0.0, noise_frac=0.0, name="", paths=("deep", "shallow")):
    d = HEAD_DIM
    rk = _rng(*key, 1)
    K, cen_k, assign = clustered(rk, B, H, l, d, n_centroids, 0.1, heavy_frac, 4.0, drift_sigma)
    rv = _rng(*key, 2)
    cen_v = rv.standard_normal((B, H, n_centroids, d), dtype=np.float32)
    V = np.take_along_axis(cen_v, assign[..., None], axis=2)
    V = V + np.float32(0.1) * rv.standard_normal((B, H, l, d), dtype=np.float32)
    if drift_sigma > 0.0:
        V = V + np.cumsum(np.float32(drift_sigma) * rv.standard_normal((B, H, l, d), dtype=np.float32),
                          axis=2, dtype=np.float32)
    if noise_frac > 0.0:
        rn = _rng(*key, 4)
        noise = rn.random((B, H, l)) < noise_frac
        s3 = np.float32(np.sqrt(3.0))
        K = np.where(noise[..., None], rn.uniform(-s3, s3, size=K.shape).astype(np.float32), K)
        V = np.where(noise[..., None], rn.uniform(-s3, s3, size=V.shape).astype(np.float32), V)
    Q = window_queries(_rng(*key, 3), cen_k, hn, lw, 0.1)
    return Layer(dtype, cast(K, dtype), cast(V, dtype), cast(Q, dtype), hn, lw, pool, budget, cap,
                 name=name, paths=paths, meta={"assign": assign})


def config2(seed: int = 0) -> Layer:
    """Llama-3-8B-shaped layer, l=4096, fp16, 64 Gaussian clusters per head (sigma 0.1),
    5 % heavy hitters with 4x norm; window 32, pool 7, budget 1024, cap 1024."""
    return _clustered_layer((2, seed), "f16", 1, 8, 4096, 4, 32, 7, 1024, 1024, 64, name="config2")


def config3_budget(layer: int) -> int:
    """Deep-layer budgets taper linearly from 2048 (layer 8) to 256 (layer 31)."""
    return int(np.floor(2048 + (256 - 2048) * (layer - 8) / 23.0 + 0.5))


def config3_layer(layer: int, seed: int = 0, seq_len: int = 8192) -> Layer:
    """Layer `layer` of the 32-layer stack at l=8192: layers 0-7 shallow (cap 512),
    layers 8-31 deep with the tapering budget."""
    if layer < 8:
        return _clustered_layer((3, seed, layer), "f16", 1, 8, seq_len, 4, 32, 7, seq_len, 512, 64,
                                name=f"config3/layer{layer}", paths=("shallow",))
    return _clustered_layer((3, seed, layer), "f16", 1, 8, seq_len, 4, 32, 7, config3_budget(layer), 512, 64,
                            name=f"config3/layer{layer}", paths=("deep",))


CONFIG4_DRIFT_SIGMA = 0.0026


def config4(seed: int = 0, seq_len: int = 32768, n_kv_heads: int = 8) -> Layer:
    """Mistral-7B-shaped layer at l=32768, fp16, 256 clusters with a random-walk drift
    along the sequence (same-cluster cosine falls through theta_K over a few thousand
    positions); window 64, pool 7, budget 2048, cap 2048."""
    return _clustered_layer((4, seed), "f16", 1, n_kv_heads, seq_len, 4, 64, 7, 2048, 2048, 256,
                            drift_sigma=CONFIG4_DRIFT_SIGMA, name="config4")


def config5_layer(layer: int, budget: int, seed: int = 0, batch: int = 4, seq_len: int = 32768,
                  n_kv_heads: int = 8) -> Layer:
    """One layer of the batched bf16 stress stack: half the tokens clustered
    (256 centroids), half uniform noise of unit variance; window 64, pool 15."""
    return _clustered_layer((5, seed, layer), "bf16", batch, n_kv_heads, seq_len, 4, 64, 15, budget, budget,
                            256, noise_frac=0.5, name=f"config5/layer{layer}/b{budget}")


def small_random(seed: int, dtype: str = "f16", B: int = 1, H: int = 2, l: int = 300, hn: int = 4,
                 lw: int = 16, pool: int = 7, budget: int = 64, cap: int = 64,
                 n_centroids: int = 12, noise_frac: float = 0.2, drift_sigma: float = 0.0) -> Layer:
    """Small ragged-size layer for parity tests (sizes need not be tile multiples)."""
    return _clustered_layer((99, seed, l), dtype, B, H, l, hn, lw, pool, budget, cap, n_centroids,
                            noise_frac=noise_frac, drift_sigma=drift_sigma, name=f"small/{seed}/{l}")


def decode_case(seed: int, dtype: str = "f16", B: int = 1, H: int = 2, n_prefill: int = 600, m: int = 128,
                n_centroids: int = 24, novel_frac: float = 0.25, novel_centroids: int = 5,
                sigma: float = 0.1, d: int = 128):
    """Decode-time stand-in: `n_prefill` clustered tokens per head (the codebook is built from
    them) and `m` later tokens, of which a fraction `novel_frac` comes from `novel_centroids`
    directions the prefill never saw (they find no entry and need new ones) and the rest from
    the prefill's own centroids.  Returns (prefill [B,H,n_prefill,d], new [B,H,m,d]) in the
    device representation of `dtype`."""
    rng = _rng(77, seed, n_prefill, m)
    x, cent, _ = clustered(rng, B, H, n_prefill + m, d, n_centroids, sigma, heavy_frac=0.05)
    fresh, _, _ = clustered(rng, B, H, m, d, max(novel_centroids, 1), sigma)
    novel = rng.random((B, H, m)) < novel_frac
    new = np.where(novel[..., None], fresh, x[:, :, n_prefill:])
    return cast(x[:, :, :n_prefill], dtype), cast(new, dtype)
