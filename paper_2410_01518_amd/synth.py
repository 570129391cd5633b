"""Seeded synthetic KV-cache inputs shaped like the benchmark configurations.

This module only draws random tensors (and rounds them to bf16 storage); it
holds none of the method's arithmetic, so both the tests' CPU checker and the
HIP path can be fed from it.  bf16 tensors are returned as uint16 bit patterns.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class CCDConfig:
    name: str
    B: int
    L: int
    Hq: int
    Hkv: int
    d: int
    N: int          # tokens in the (full) pot when compression fires
    k: int          # |C|: entries kept
    P: int          # |P|: catalyst-prompt query tokens
    T: int          # NuC slots (alpha * |C|, alpha = 50 % in the paper's experiments)
    w: int          # pooling window (1 = none)
    dtype: str      # "fp32" | "bf16"
    keys: str       # "normal" | "outlier1pct" | "zipf"
    seed: int

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def units(self) -> int:
        return self.B * self.L * self.Hkv


CONFIGS = {
    # tiny CCD step
    "c1": CCDConfig("c1", 1, 1, 4, 4, 64, 512, 256, 16, 128, 1, "fp32", "normal", 1),
    # single layer, Llama-style GQA, 1 % outlier tokens
    "c2": CCDConfig("c2", 1, 1, 32, 8, 128, 2048, 1024, 32, 512, 7, "bf16", "outlier1pct", 2),
    # full 32-layer Llama-3-8B-shaped cache (headline)
    "c3": CCDConfig("c3", 1, 32, 32, 8, 128, 4096, 2048, 64, 1024, 7, "bf16", "normal", 3),
    # one call of the streaming Mistral-7B-shaped run (same shape as c3)
    "c4": CCDConfig("c4", 1, 32, 32, 8, 128, 4096, 2048, 64, 1024, 7, "bf16", "normal", 4),
    # large pot, heavy compression, Zipf-skewed key norms, batch of 4
    "c5": CCDConfig("c5", 4, 80, 64, 8, 128, 32768, 4096, 128, 2048, 7, "bf16", "zipf", 5),
    # not a benchmark configuration: the headline's layer / head / pot shape with an fp32 cache of head dimension 64
    "c3f": CCDConfig("c3f", 1, 32, 32, 8, 64, 4096, 2048, 64, 1024, 7, "fp32", "normal", 6),
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16 storage bits (uint16)."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(u: np.ndarray) -> np.ndarray:
    return (np.asarray(u, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    return x if dtype == "fp32" else f32_to_bf16_bits(x)


def make_inputs(cfg: CCDConfig, *, per_head_novelty: bool = False, seed: int | None = None):
    """Q_cat [B,L,Hq,P,d], K, V [B,L,Hkv,N,d], novelty [B,N] (or [B,L,Hkv,N]) for one full pot."""
    rng = np.random.Generator(np.random.Philox(cfg.seed if seed is None else seed))
    B, L, Hq, Hkv, d, N, P = cfg.B, cfg.L, cfg.Hq, cfg.Hkv, cfg.d, cfg.N, cfg.P
    Q = rng.standard_normal((B, L, Hq, P, d), dtype=np.float32)
    K = rng.standard_normal((B, L, Hkv, N, d), dtype=np.float32)
    V = rng.standard_normal((B, L, Hkv, N, d), dtype=np.float32)
    if cfg.keys == "outlier1pct":
        # 1 % of the token positions, drawn once per sequence, carry keys scaled x4 in every head
        n_out = max(1, N // 100)
        for b in range(B):
            pos = rng.choice(N, size=n_out, replace=False)
            K[b, :, :, pos, :] *= np.float32(4.0)
    elif cfg.keys == "zipf":
        # key row t scaled by sqrt(min(z_t, 64)), z_t ~ Zipf(1.1), one draw per (sequence, token)
        z = np.minimum(rng.zipf(1.1, size=(B, N)), 64).astype(np.float32)
        K *= np.sqrt(z)[:, None, None, :, None]
    nov_shape = (B, L, Hkv, N) if per_head_novelty else (B, N)
    novelty = rng.random(nov_shape, dtype=np.float32)
    return {"Q_cat": _store(Q, cfg.dtype), "K": _store(K, cfg.dtype), "V": _store(V, cfg.dtype),
            "novelty": novelty}


def cap_keys(cfg: CCDConfig, *, seed: int | None = None, gain: float = 1.0) -> np.ndarray:
    """K_cap [B,L,Hkv,P,d]: the CaP tokens' own keys (standard normal like the cached keys, times `gain`), in the
    cache's storage type.  A stream of its own, so that make_inputs stays as it is."""
    rng = np.random.Generator(np.random.Philox((cfg.seed if seed is None else seed) + 7919))
    Kc = rng.standard_normal((cfg.B, cfg.L, cfg.Hkv, cfg.P, cfg.d), dtype=np.float32) * np.float32(gain)
    return _store(Kc, cfg.dtype)


def scaled(cfg: CCDConfig, **kw) -> CCDConfig:
    """A copy of a configuration with some fields replaced (test-sized variants)."""
    return replace(cfg, **kw)


def rope_tables(n_pos: int, d: int, base: float = 10000.0):
    """Input tables of the rotary embedding: cos, sin [n_pos, d/2] fp32 of the angles p * base**(-2i/d)."""
    i = np.arange(d // 2, dtype=np.float64)
    ang = np.arange(n_pos, dtype=np.float64)[:, None] * base ** (-2.0 * i / d)[None, :]
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)
