"""Seeded synthetic inputs for the POET-X hot path.

Shared by the tests, the benchmark and the smoke check.  Holds none of the
method's arithmetic: only shapes, seeds, random draws and dtype rounding.
"""
from .configs import CONFIGS, Projection, LayerConfig, get_config
from .gen import (draw_projection, round_bf16, round_f32, tensor_seed,
                  theta_shape, draw_permutation)

__all__ = ["CONFIGS", "Projection", "LayerConfig", "get_config", "draw_projection",
           "round_bf16", "round_f32", "tensor_seed", "theta_shape", "draw_permutation"]
