"""Seeded draws of one projection's tensors.

Values are drawn in float64 with numpy's PCG64, scaled, then rounded once to
the storage dtype; the rounded values are returned as float64 arrays so that
the CPU check and the GPU path consume exactly the same numbers.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 20260305
# tensor ids inside one projection
T_X, T_DZ, T_W, T_THETA_R, T_THETA_P, T_PI_R, T_PI_P = range(7)


def tensor_seed(config_index: int, proj_index: int, tensor_id: int, step: int = 0) -> int:
    return BASE_SEED + 1000 * config_index + 10 * proj_index + tensor_id + 100000 * step


def round_f32(a: np.ndarray) -> np.ndarray:
    return np.asarray(a, dtype=np.float64).astype(np.float32).astype(np.float64)


def round_bf16(a: np.ndarray) -> np.ndarray:
    """Round to bfloat16 (nearest even on the float32 bit pattern), returned as float64."""
    f = np.ascontiguousarray(np.asarray(a, dtype=np.float64).astype(np.float32))
    u = f.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = ((u + bias) & np.uint32(0xFFFF0000)).view(np.float32)
    return r.astype(np.float64)


def theta_shape(d: int, b: int):
    return (-(-d // b), b * (b - 1) // 2)


def draw_permutation(d: int, seed: int) -> np.ndarray:
    return np.random.Generator(np.random.PCG64(seed)).permutation(d).astype(np.int32)


def _normal(shape, sigma, seed):
    g = np.random.Generator(np.random.PCG64(seed))
    return g.standard_normal(shape) * sigma


def draw_theta(d: int, b: int, sigma: float, seed: int, zero_dead: bool = True) -> np.ndarray:
    """Packed skew parameters, fp32-rounded.  The unused slots of a ragged tail block are zero
    unless zero_dead is False (they must be ignored either way; the non-zero draw checks that)."""
    nb, L = theta_shape(d, b)
    th = round_f32(_normal((nb, L), sigma, seed))
    r = d - b * (nb - 1)
    if r < b and zero_dead:
        iu, ju = np.triu_indices(b, k=1)
        th[nb - 1, (iu >= r) | (ju >= r)] = 0.0
    return th


def draw_projection(cfg, proj_index: int, n_tokens: int | None = None, step: int = 0,
                    want=("X", "dZ", "W", "theta_R", "theta_P", "pi_R", "pi_P"), zero_dead: bool = True) -> dict:
    """All tensors of one projection of `cfg` (feature-major: X is m x N, dZ is n x N)."""
    p = cfg.projections[proj_index]
    N = cfg.n_tokens if n_tokens is None else n_tokens
    m, n, b = p.d_in, p.d_out, cfg.block
    rnd = round_f32 if cfg.dtype == "f32" else round_bf16
    ci = cfg.index if cfg.block != 512 else cfg.index + 1
    out = {"m": m, "n": n, "N": N, "b": b, "k": cfg.neumann_k}
    if "X" in want:
        out["X"] = rnd(_normal((m, N), 1.0, tensor_seed(ci, proj_index, T_X)))
    if "dZ" in want:
        out["dZ"] = rnd(_normal((n, N), 1.0, tensor_seed(ci, proj_index, T_DZ)))
    if "W" in want:
        out["W"] = rnd(_normal((n, m), cfg.sigma_w, tensor_seed(ci, proj_index, T_W)))
    if "theta_R" in want:
        out["theta_R"] = draw_theta(m, b, cfg.sigma_theta, tensor_seed(ci, proj_index, T_THETA_R), zero_dead)
    if "theta_P" in want:
        out["theta_P"] = draw_theta(n, b, cfg.sigma_theta, tensor_seed(ci, proj_index, T_THETA_P), zero_dead)
    if "pi_R" in want:
        out["pi_R"] = draw_permutation(m, tensor_seed(ci, proj_index, T_PI_R, step))
    if "pi_P" in want:
        out["pi_P"] = draw_permutation(n, tensor_seed(ci, proj_index, T_PI_P, step))
    return out
