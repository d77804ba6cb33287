"""The five synthetic workloads the build is measured and tested on.

Shapes follow the models and hyper-parameters of the paper's experiments
(LLaMA-3-8B: 32 query / 8 KV heads, d = 128; Qwen2.5-7B: 28 / 4; default
r = 32, k = 2048, 64 lite tokens at 128K context; r = 16..32, k = 256, 16 lite
tokens at 4K).  The prompts, weights and activations of those experiments are
not available, so every tensor is drawn from a seeded generator instead.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    B: int
    Hq: int
    Hkv: int
    l: int
    r: int
    k: int
    w: int
    C: int
    d: int = 128
    layers: int = 1
    kv_dtype: str = "bf16"       # "bf16" or "f32"
    # heavy-token recipe
    n_heavy: int = 64            # tokens per query head inside the heavy window
    pool_mult: int = 8           # pool size = pool_mult * n_heavy tokens on the phase circle
    phase_spread: float = 1.0    # 0: every pool token aligned with the query (config 1)
    drift: float = 0.1           # fraction of the heavy window the query phase moves per step
    redraw_every: int = 0        # >0: jump to a fresh phase every this many steps
    beta: float = 4.0            # size of the planted component in factor space
    gamma: float = math.sqrt(128.0)  # size of the planted component of the query
    rho: float = 0.95            # AR(1) correlation of the background query across steps
    noise: float = 0.05          # full-rank residual added to A_K B
    group_share: float = 0.0     # how much the query heads of a KV group want the same tokens:
                                 # shared fraction of the heavy-token pools and of the
                                 # background query (see gen/workload.py)
    prefill: str = "warm"        # "identity": slot i holds token i (needs C == l); "warm": run steps
    seed: int = 20251023

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def pool(self) -> int:
        return self.n_heavy * self.pool_mult

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.d)

    def with_(self, **kw) -> "WorkloadConfig":
        return replace(self, **kw)


CONFIGS = {
    # 1: small, all hits (cache holds every token), one fixed query.
    "c1": WorkloadConfig(name="c1", B=1, Hq=32, Hkv=8, l=4096, r=32, k=256, w=16, C=4096,
                         n_heavy=64, pool_mult=1, phase_spread=0.0, drift=0.0,
                         prefill="identity"),
    # 2: LLaMA-3-8B-shaped single layer at 32K, ~90 % hits.
    "c2": WorkloadConfig(name="c2", B=1, Hq=32, Hkv=8, l=32768, r=32, k=1024, w=64, C=2048,
                         n_heavy=256, drift=0.1, rho=0.97),
    # 3: LLaMA-3-8B-shaped full decode step at 128K, 32 layers, rank sweep via with_(r=...).
    "c3": WorkloadConfig(name="c3", B=1, Hq=32, Hkv=8, l=131072, r=32, k=2048, w=64, C=4096,
                         layers=32, n_heavy=256, drift=0.1, rho=0.97),
    # 4: Qwen2.5-7B-shaped single layer, batch 8, 1 % heavy tokens, ~85 % hits.
    "c4": WorkloadConfig(name="c4", B=8, Hq=28, Hkv=4, l=65536, r=32, k=1024, w=64, C=2048,
                         n_heavy=655, pool_mult=4, drift=0.1, rho=0.96),
    # 5: miss-heavy stress, batch 16 at 128K, heavy set re-drawn every 4 steps.
    #    The cache size is not stated for this workload; 4096 slots as in config 3.
    "c5": WorkloadConfig(name="c5", B=16, Hq=32, Hkv=8, l=131072, r=32, k=2048, w=64, C=4096,
                         n_heavy=256, drift=0.1, redraw_every=4, rho=0.8),
}


def get_config(name: str, **overrides) -> WorkloadConfig:
    cfg = CONFIGS[name]
    return cfg.with_(**overrides) if overrides else cfg
