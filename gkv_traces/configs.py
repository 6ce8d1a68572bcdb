"""The five workload configurations (shapes, hyper-parameters, value recipe).

Notation follows the paper's Preliminary section: h_q query heads, h_kv KV
heads, d head dim, b budget, w observation window, s compression interval,
alpha memory-decay rate.  b=512, w=16, s=128 and alpha=0.8 with the max form
are the paper's own experimental settings (Experiment section,
"Implementation Details" and "Main Results").
"""
from __future__ import annotations

from dataclasses import dataclass, replace


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    n_layers: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str          # "f32" or "bf16"
    budget: int         # b
    window: int         # w
    interval: int       # s
    n_steps: int        # length T of the decode trace
    recipe: str         # "gauss_sink" | "recurring" | "heavy_tail"
    seed: int = 0
    alpha: float = 0.8
    combine: str = "max"   # "max" | "avg" | "sum"

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def capacity(self) -> int:
        """Rows allocated per KV head: b + s rounded up to a multiple of 32."""
        return (self.budget + self.interval + 31) // 32 * 32

    @property
    def n_units(self) -> int:
        return self.n_layers * self.batch * self.n_kv_heads

    def with_(self, **kw) -> "WorkloadConfig":
        return replace(self, **kw)


_CFG3 = WorkloadConfig(
    name="cfg3_28layer_b512", n_layers=28, batch=8, n_q_heads=28, n_kv_heads=4,
    head_dim=128, dtype="bf16", budget=512, window=16, interval=128,
    n_steps=16384, recipe="recurring", seed=3)

CONFIGS = {
    # 1 Tiny
    "cfg1_tiny": WorkloadConfig(
        name="cfg1_tiny", n_layers=1, batch=1, n_q_heads=8, n_kv_heads=2,
        head_dim=64, dtype="f32", budget=64, window=8, interval=16,
        n_steps=256, recipe="gauss_sink", seed=0),
    # 2 single layer at the real head shape
    "cfg2_single_layer": WorkloadConfig(
        name="cfg2_single_layer", n_layers=1, batch=1, n_q_heads=28, n_kv_heads=4,
        head_dim=128, dtype="bf16", budget=512, window=16, interval=128,
        n_steps=4096, recipe="recurring", seed=2),
    # 3 full 28-layer decode, the headline
    "cfg3_28layer_b512": _CFG3,
    # 4 budget sweep at batch 16 (+ local-only leg)
    "cfg4_b512": _CFG3.with_(name="cfg4_b512", batch=16, n_steps=32768, seed=4),
    "cfg4_b1024": _CFG3.with_(name="cfg4_b1024", batch=16, n_steps=32768, seed=4, budget=1024),
    "cfg4_b2048": _CFG3.with_(name="cfg4_b2048", batch=16, n_steps=32768, seed=4, budget=2048),
    "cfg4_b512_local": _CFG3.with_(name="cfg4_b512_local", batch=16, n_steps=32768, seed=4,
                                   alpha=0.0),
    # 5 large-batch throughput
    "cfg5_large_batch": WorkloadConfig(
        name="cfg5_large_batch", n_layers=36, batch=64, n_q_heads=40, n_kv_heads=8,
        head_dim=128, dtype="bf16", budget=1024, window=32, interval=64,
        n_steps=32768, recipe="heavy_tail", seed=5),
}


def get_config(name: str) -> WorkloadConfig:
    return CONFIGS[name]
