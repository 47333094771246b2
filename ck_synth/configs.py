"""Shapes of the five synthetic benchmark configurations.

The shapes follow a Llama-3-8B attention layer (32 query heads, 8 KV heads,
head_dim 128) and the hyper-parameters the paper states in Section III-B
(C0 = L/80, i.e. 400 clusters at a 32k context; incremental clustering of every
m = 320 generated tokens into C+ = 4 new clusters) and Section V (budgets from
256 to 2048 tokens).
"""
from __future__ import annotations

from dataclasses import dataclass


@dataclass(frozen=True)
class Config:
    name: str
    layers: int          # independent seeded KV sets
    S: int               # sequences in the batch
    Hkv: int             # KV heads
    Hq: int              # query heads (Hq / Hkv = GQA group size)
    d: int               # head dimension
    N: int               # prefill context length per sequence
    M: int               # mixture centers per head-problem
    C: int               # clusters per head-problem at prefill
    n_iter: int          # K-means iterations
    B: int               # token budget
    seed: int
    decode_steps: int = 1
    m_incr: int = 0      # cluster the generated tokens every m_incr steps (0 = never)
    c_incr: int = 0      # clusters added per incremental clustering

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def head_problems(self) -> int:
        return self.layers * self.S * self.Hkv


CONFIGS = (
    Config("tiny", layers=1, S=1, Hkv=2, Hq=2, d=128, N=2048, M=64, C=32,
           n_iter=10, B=256, seed=0),
    Config("llama3_8b_layer_32k", layers=1, S=1, Hkv=8, Hq=32, d=128, N=32768, M=512,
           C=400, n_iter=10, B=1024, seed=1),
    Config("full_depth_32layers_b8", layers=32, S=8, Hkv=8, Hq=32, d=128, N=32768,
           M=512, C=400, n_iter=10, B=2048, seed=2),
    Config("long_context_128k", layers=1, S=1, Hkv=8, Hq=32, d=128, N=131072, M=2048,
           C=1600, n_iter=10, B=2048, seed=3),
    Config("incremental_decode_b16", layers=1, S=16, Hkv=8, Hq=32, d=128, N=32768,
           M=512, C=400, n_iter=10, B=1024, seed=4, decode_steps=1024, m_incr=320,
           c_incr=4),
)


def get_config(which) -> Config:
    if isinstance(which, int):
        return CONFIGS[which]
    for c in CONFIGS:
        if c.name == which:
            return c
    raise KeyError(which)
