"""Seeded synthetic decode traces and the five workload configurations.

This package only draws random numbers and lays them out; it contains none of
the eviction method's arithmetic.  Both the CPU oracle's tests and the GPU
path's tests/benchmark take their inputs from here, so the two sides always
see the same bytes.
"""
from .configs import CONFIGS, WorkloadConfig, get_config
from .gen import Trace, bf16_round, to_bf16_bits, from_bf16_bits

__all__ = [
    "CONFIGS",
    "WorkloadConfig",
    "get_config",
    "Trace",
    "bf16_round",
    "to_bf16_bits",
    "from_bf16_bits",
]
