"""Seeded synthetic inputs shaped like the KV caches the method is evaluated on.

This module only draws random numbers.  It holds none of the method's
arithmetic (no ranges, thresholds, codes or attention), so both the CPU oracle's
tests and the GPU path's tests can feed from it without sharing anything else.

The paper measures on LLaMA-2 caches built from public benchmark prompts; those
are not available here, so these draws stand in for them: LLaMA-2-7B head shape
(32 heads x 128 channels), heavy tails at both ends of the value distribution
and a handful of high-importance tokens are the only things taken over.
All arrays are produced on the host with numpy's default_rng and cast to fp16
with round-to-nearest-even.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional, Tuple

import numpy as np

BASE_SEED = 20240304


@dataclass(frozen=True)
class Shape:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    context: int

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def token_heads(self) -> int:
        return self.batch * self.n_kv_heads * self.context


CONFIGS = {
    1: Shape("cfg1-small", 1, 8, 8, 64, 512),
    2: Shape("cfg2-llama7b-layer", 8, 32, 32, 128, 4096),
    3: Shape("cfg3-llama7b-stack", 8, 32, 32, 128, 4096),
    4: Shape("cfg4-long-context", 1, 32, 32, 128, 32768),
    5: Shape("cfg5-gqa70b-layer", 16, 64, 8, 128, 8192),
}


def shape(config: int, **override) -> Shape:
    return replace(CONFIGS[config], **override)


def _to_f16(a: np.ndarray) -> np.ndarray:
    return np.clip(a, -65504.0, 65504.0).astype(np.float16)


def _channel_std(rng, n_heads: int, D: int) -> np.ndarray:
    """Per (head, channel) standard deviation, log-uniform in [0.5, 4]."""
    return np.exp(rng.uniform(np.log(0.5), np.log(4.0), size=(n_heads, D))).astype(np.float32)


def kv_spiky(rng, sh: Shape, n_tokens: int, p: float = 0.01, gain: float = 15.0) -> np.ndarray:
    """N(0,1) entries, a Bernoulli(p) subset multiplied by `gain` (configs 1, 5
    use it on top of different per-channel scales)."""
    x = rng.standard_normal((sh.batch, sh.n_kv_heads, n_tokens, sh.head_dim), dtype=np.float32)
    m = rng.random(x.shape, dtype=np.float32) < p
    x[m] *= gain
    return x


def make_kv(config: int, sh: Optional[Shape] = None, n_tokens: Optional[int] = None,
            seed_offset: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """fp16 K and V of shape [B, Hkv, n_tokens, D] for the given workload."""
    sh = sh or CONFIGS[config]
    T = sh.context if n_tokens is None else n_tokens
    rng = np.random.default_rng(BASE_SEED + config + 1000 * seed_offset)
    out = []
    for side in range(2):
        if config == 1:
            x = kv_spiky(rng, sh, T, 0.01, 15.0)
        elif config == 5:
            std = _channel_std(rng, sh.n_kv_heads, sh.head_dim)
            x = kv_spiky(rng, sh, T, 0.01, 15.0) * std[None, :, None, :]
        else:
            # configs 2, 3, 4: per-channel std, 0.5% of the (head, channel) pairs heavy tailed
            std = _channel_std(rng, sh.n_kv_heads, sh.head_dim)
            heavy = rng.random((sh.n_kv_heads, sh.head_dim)) < 0.005
            x = rng.standard_normal((sh.batch, sh.n_kv_heads, T, sh.head_dim), dtype=np.float32)
            hh, cc = np.nonzero(heavy)
            for h, c in zip(hh, cc):
                x[:, h, :, c] = rng.standard_t(3.0, size=(sh.batch, T)).astype(np.float32)
            x *= std[None, :, None, :]
        out.append(_to_f16(x))
    return out[0], out[1]


def make_queries(config: int, sh: Optional[Shape] = None, n: int = 1, seed_offset: int = 0) -> np.ndarray:
    """fp16 queries [n, B, Hq, D].  Config 1: N(0,1); others: N(0, std = 1/sqrt(D))."""
    sh = sh or CONFIGS[config]
    rng = np.random.default_rng(BASE_SEED + 77 + config + 1000 * seed_offset)
    std = 1.0 if config == 1 else 1.0 / np.sqrt(sh.head_dim)
    q = rng.standard_normal((n, sh.batch, sh.n_q_heads, sh.head_dim), dtype=np.float32) * np.float32(std)
    return _to_f16(q)


def make_new_token(config: int, sh: Optional[Shape] = None, step: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """One appended token per sequence, drawn like the cache rows: fp16 [B, Hkv, D] each."""
    k, v = make_kv(config, sh, n_tokens=1, seed_offset=500 + step)
    return k[:, :, 0, :].copy(), v[:, :, 0, :].copy()


def zipf_score_rows(sh: Shape, T: int, exponent: float = 1.1, seed_offset: int = 0) -> np.ndarray:
    """Config 4: a normalised key-importance profile S_t ~ rank^-exponent under a
    seeded permutation of the positions; fp32 [B, Hq, T] (the same profile per
    head up to its own permutation)."""
    rng = np.random.default_rng(BASE_SEED + 4444 + 1000 * seed_offset)
    base = np.arange(1, T + 1, dtype=np.float64) ** (-exponent)
    base /= base.sum()
    out = np.empty((sh.batch, sh.n_q_heads, T), dtype=np.float32)
    for b in range(sh.batch):
        for h in range(sh.n_q_heads):
            out[b, h, rng.permutation(T)] = base
    return out


def random_score_rows(sh: Shape, T: int, n: int, seed: int, peaky: float = 2.0) -> np.ndarray:
    """n normalised score rows [n, B, Hq, T] from a seeded softmax of Gaussian
    logits; a plain way to get positive rows that sum to one for unit tests."""
    rng = np.random.default_rng(seed)
    a = rng.standard_normal((n, sh.batch, sh.n_q_heads, T)) * peaky
    a -= a.max(axis=-1, keepdims=True)
    e = np.exp(a)
    return (e / e.sum(axis=-1, keepdims=True)).astype(np.float32)
