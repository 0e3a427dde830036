"""Seeded synthetic inputs shaped like the paper's workloads.

Only shapes and value distributions live here -- none of the method's arithmetic -- so that the
CPU oracle and the GPU library can be fed identical tensors.  Shapes follow the paper's test
configurations (section "Experimental Setup", Table 1: about 600 / 1,851 / 7,194 context tokens,
3 to 15 agents; SmolLM2-1.7B with 24 layers x 32 heads x head_dim 64, Llama-3-8B with 32 layers,
8 KV heads, 32 query heads, head_dim 128).  The paper's real KV tensors need model weights and
texts that are not available, so the values are random:

  K[l,h,t,c] = z * g[l,h,c]   g = exp(0.5 z'), each channel independently an outlier (x8) with
                              probability 0.01      (config 1: g = 1 and two x10 channels per head)
  V[l,h,t,:] = z * exp(0.3 z'') per token           (config 1: plain N(0,1))
  Q ~ N(0,1)

everything drawn in float32 from numpy's PCG64 seeded with 1000*config + layer and rounded to
float16.  Tensors are produced layer by layer so that the big configurations can be streamed.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class PoolConfig:
    cid: int
    name: str
    layers: int
    kv_heads: int
    q_heads: int
    head_dim: int
    tokens: int
    agents: int
    q_per_agent: int
    max_tail: int = 0

    @property
    def group(self) -> int:
        return self.q_heads // self.kv_heads

    @property
    def rows_per_kv_head(self) -> int:
        return self.agents * self.q_per_agent * self.group

    def scaled(self, **kw) -> "PoolConfig":
        d = dict(self.__dict__)
        d.update(kw)
        return PoolConfig(**d)


CONFIGS = {
    1: PoolConfig(1, "tiny", 1, 4, 4, 64, 600, 3, 1),
    2: PoolConfig(2, "smollm2-1.7b-shape", 24, 32, 32, 64, 1851, 5, 1),
    3: PoolConfig(3, "llama3-8b-shape-4096", 32, 8, 32, 128, 4096, 15, 1),
    4: PoolConfig(4, "llama3-8b-shape-7194-tails", 32, 8, 32, 128, 7194, 15, 1, max_tail=64),
    5: PoolConfig(5, "llama3-8b-shape-7194-stress", 32, 8, 32, 128, 7194, 64, 4),
    # not one of the paper's workloads: a head_dim-256 shape (16 query heads over 8 KV heads) for the extra
    # kernel instantiations
    6: PoolConfig(6, "head-dim-256-shape-4096", 26, 8, 16, 256, 4096, 15, 1),
}


def _rng(cfg: PoolConfig, layer: int, stream: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([1000 * cfg.cid + layer, stream]))


def kv_layer(cfg: PoolConfig, layer: int, tokens: int | None = None, stream: int = 0):
    """K, V float16 [kv_heads, tokens, head_dim] of one layer."""
    T = cfg.tokens if tokens is None else tokens
    H, d = cfg.kv_heads, cfg.head_dim
    rng = _rng(cfg, layer, stream)
    k = rng.standard_normal((H, T, d), dtype=np.float32)
    v = rng.standard_normal((H, T, d), dtype=np.float32)
    if cfg.cid == 1:
        for h in range(H):
            ch = rng.choice(d, size=2, replace=False)
            k[h, :, ch] *= np.float32(10.0)
    else:
        g = np.exp(np.float32(0.5) * rng.standard_normal((H, 1, d), dtype=np.float32))
        outlier = rng.random((H, 1, d)) < 0.01
        g = np.where(outlier, g * np.float32(8.0), g).astype(np.float32)
        k *= g
        v *= np.exp(np.float32(0.3) * rng.standard_normal((H, T, 1), dtype=np.float32))
    return k.astype(np.float16), v.astype(np.float16)


def bf16_round(x):
    """float32 array rounded to the nearest bfloat16 (ties to even), returned as float32: how the tests
    and the benchmark make bfloat16 tensors (numpy has no such dtype)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32)


def bf16_bits(x):
    """The 16-bit patterns (uint16) of a float32 array holding bfloat16 values."""
    return (np.ascontiguousarray(x, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)


def kv_pool(cfg: PoolConfig):
    """K, V float16 [layers, kv_heads, tokens, head_dim]."""
    K = np.empty((cfg.layers, cfg.kv_heads, cfg.tokens, cfg.head_dim), dtype=np.float16)
    V = np.empty_like(K)
    for l in range(cfg.layers):
        K[l], V[l] = kv_layer(cfg, l)
    return K, V


def queries(cfg: PoolConfig, step: int = 0):
    """Q float16 [layers, agents, q_per_agent, q_heads, head_dim]."""
    rng = np.random.Generator(np.random.PCG64([1000 * cfg.cid + 500, step]))
    q = rng.standard_normal((cfg.layers, cfg.agents, cfg.q_per_agent, cfg.q_heads, cfg.head_dim),
                            dtype=np.float32)
    return q.astype(np.float16)


def tails(cfg: PoolConfig, lengths):
    """Per-agent private continuation: list of (K, V) float16 [layers, kv_heads, len_a, head_dim],
    drawn from the same distributions as the pool with a per-agent stream."""
    out = []
    for a, n in enumerate(lengths):
        K = np.empty((cfg.layers, cfg.kv_heads, n, cfg.head_dim), dtype=np.float16)
        V = np.empty_like(K)
        for l in range(cfg.layers):
            if n:
                K[l], V[l] = kv_layer(cfg, l, tokens=n, stream=100 + a)
        out.append((K, V))
    return out
