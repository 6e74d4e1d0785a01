"""The five benchmark configurations: shapes, block size, series length, dtype
and value scales.  Weight shapes are out x in (n x m)."""
from __future__ import annotations

from dataclasses import dataclass
from typing import Tuple


@dataclass(frozen=True)
class Projection:
    name: str
    d_out: int  # n
    d_in: int   # m


@dataclass(frozen=True)
class LayerConfig:
    index: int
    name: str
    n_tokens: int
    block: int
    neumann_k: int
    dtype: str            # "f32" or "bf16": storage type of X, W, Z, gradients
    sigma_w: float
    sigma_theta: float
    projections: Tuple[Projection, ...]
    fresh_perms: bool = False


def _llama(d: int, ffn: int, kv: int) -> Tuple[Projection, ...]:
    return (Projection("q", d, d), Projection("k", kv, d), Projection("v", kv, d),
            Projection("o", d, d), Projection("gate", ffn, d), Projection("up", ffn, d),
            Projection("down", d, ffn))


CONFIGS = {
    1: LayerConfig(1, "single-256-f32", 512, 32, 4, "f32", 0.02, 0.01,
                   (Projection("lin", 256, 256),)),
    2: LayerConfig(2, "llama60m", 4 * 256, 64, 4, "bf16", 0.02, 0.01, _llama(512, 1376, 512)),
    3: LayerConfig(3, "llama1b", 8 * 2048, 256, 4, "bf16", 0.02, 0.005, _llama(2048, 5632, 2048)),
    4: LayerConfig(4, "llama3b", 8 * 2048, 256, 5, "bf16", 0.02, 0.005, _llama(3072, 8192, 1024),
                   fresh_perms=True),
    5: LayerConfig(5, "llama8b-b256", 4 * 4096, 256, 5, "bf16", 0.02, 0.005,
                   _llama(4096, 14336, 1024)),
    6: LayerConfig(5, "llama8b-b512", 4 * 4096, 512, 5, "bf16", 0.02, 0.005,
                   _llama(4096, 14336, 1024)),
}


def get_config(key) -> LayerConfig:
    """Look a configuration up by key (1..6) or by name."""
    if isinstance(key, str) and not key.isdigit():
        for c in CONFIGS.values():
            if c.name == key:
                return c
        raise KeyError(key)
    return CONFIGS[int(key)]
