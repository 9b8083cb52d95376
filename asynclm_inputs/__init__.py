"""Seeded synthetic inputs: model shapes, weights, token streams, interrupt schedules.

This module produces *inputs only*. It holds none of the decoder's arithmetic and is
the one piece of code that both the CPU oracle's tests and the HIP path's callers use,
so that both sides see bit-identical weights and token ids.
"""
from .configs import ModelConfig, Workload, PRESETS, preset, truncated
from .generator import (
    MASTER_SEED,
    splitmix64_draws_py,
    tensor_key,
    gaussian_tensor,
    make_weights,
    weights_to_numpy,
    uniform_tokens,
    build_workload,
)

__all__ = [
    "ModelConfig", "Workload", "PRESETS", "preset", "truncated", "MASTER_SEED",
    "splitmix64_draws_py", "tensor_key", "gaussian_tensor", "make_weights",
    "weights_to_numpy", "uniform_tokens", "build_workload",
]
