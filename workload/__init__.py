"""Seeded synthetic MoE-decode workloads (inputs only).

This package produces *data*: router and expert weights, hidden states,
per-sequence preferred-expert sets and logit biases.  It contains none of the
MoE layer's or the cache policy's arithmetic; the CPU oracle and the HIP path
each consume the same arrays and compute everything on their own.
"""
from .configs import MoEConfig, CONFIGS, get_config
from .gen import (Workload, f32_to_bf16_bits, bf16_bits_to_f32, widen, quantize_int4)

__all__ = ["MoEConfig", "CONFIGS", "get_config", "Workload",
           "f32_to_bf16_bits", "bf16_bits_to_f32", "widen", "quantize_int4"]
