"""Shared helpers for the GPU parity tests: move seeded inputs to the device,
run the library through its Python binding, bring results back as float64."""
from __future__ import annotations

import numpy as np
import torch

import paper_2603_05500_amd as px

TOL = {"f32": 1e-4, "bf16": 2e-2}


def tdtype(name):
    return torch.float32 if name == "f32" else torch.bfloat16


def to_dev(a: np.ndarray, dtype) -> torch.Tensor:
    """Values are already representable in `dtype`, so the conversion is exact."""
    return torch.from_numpy(np.ascontiguousarray(a)).to(dtype).cuda()


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max |got - ref| / max |ref| over the tensor (the tolerance's metric)."""
    denom = np.max(np.abs(ref))
    if denom == 0:
        return float(np.max(np.abs(got)))
    return float(np.max(np.abs(got - ref)) / denom)


def row_rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """Scale-aware companion of rel_err: the worst row, each row measured on its own scale
    (max |got_row - ref_row| / max |ref_row|).  A row (a feature across tokens, a block of
    packed parameters) that is wrong as a whole cannot hide behind larger rows."""
    got2 = got.reshape(got.shape[0], -1)
    ref2 = ref.reshape(ref.shape[0], -1)
    den = np.max(np.abs(ref2), axis=1)
    num = np.max(np.abs(got2 - ref2), axis=1)
    ok = den > 0
    if not ok.any():
        return float(np.max(num))
    return float(np.max(num[ok] / den[ok]))


def p999_err(got: np.ndarray, ref: np.ndarray) -> float:
    """99.9th percentile of the element-wise relative error, with the denominator floored at
    1e-3 of the tensor's largest magnitude (reported next to the tolerance's metric)."""
    floor = 1e-3 * np.max(np.abs(ref))
    if floor == 0:
        return 0.0
    e = np.abs(got - ref) / np.maximum(np.abs(ref), floor)
    return float(np.quantile(e.ravel(), 0.999))


def ws_tensor(nbytes: int) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device="cuda")


def build_blocks(theta: np.ndarray, d: int, b: int, k: int, dtype_name: str, precision=None):
    """cnp_build on the device; returns (blocks tensor for the apply calls, G as float64 numpy)."""
    nb = theta.shape[0]
    th = to_dev(theta, torch.float32)
    ws = ws_tensor(px.poetx_cnp_workspace_bytes(d, b))
    G = torch.empty((nb, b, b), dtype=torch.float32, device="cuda")
    if precision is None:
        precision = px.CNP_FP32 if dtype_name == "f32" else px.CNP_BF16
    if dtype_name == "f32":
        px.poetx_cnp_build(th, d, b, k, precision, G_f32=G, E_bf16=None, ws=ws)
        torch.cuda.synchronize()
        return G, to_np(G)
    E = torch.empty((nb, 2, b, b), dtype=torch.bfloat16, device="cuda")
    px.poetx_cnp_build(th, d, b, k, precision, G_f32=G, E_bf16=E, ws=ws)
    torch.cuda.synchronize()
    return E, to_np(G)


def run_layer(data: dict, dtype_name: str, cnp_precision=None) -> dict:
    """Whole hot path (cnp_build x2, fwd, bwd_input, bwd_skew) for one projection."""
    m, n, N, b, k = data["m"], data["n"], data["N"], data["b"], data["k"]
    dt = tdtype(dtype_name)
    code = px.F32 if dtype_name == "f32" else px.BF16
    desc = px.make_desc(m, n, b, k, N, code, cnp_precision)
    X, dZ, W = to_dev(data["X"], dt), to_dev(data["dZ"], dt), to_dev(data["W"], dt)
    pi_R = torch.from_numpy(data["pi_R"].astype(np.int32)).cuda()
    pi_P = torch.from_numpy(data["pi_P"].astype(np.int32)).cuda()
    th_R, th_P = to_dev(data["theta_R"], torch.float32), to_dev(data["theta_P"], torch.float32)
    blk_R, G_R = build_blocks(data["theta_R"], m, b, k, dtype_name, desc.cnp_precision)
    blk_P, G_P = build_blocks(data["theta_P"], n, b, k, dtype_name, desc.cnp_precision)
    ws = ws_tensor(px.poetx_linear_workspace_bytes(desc))
    Z = torch.empty((n, N), dtype=dt, device="cuda")
    B = torch.empty((n, N), dtype=dt, device="cuda")
    dX = torch.empty((m, N), dtype=dt, device="cuda")
    dA = torch.empty((m, N), dtype=dt, device="cuda")
    dth_R = torch.full_like(th_R, float("nan"))
    dth_P = torch.full_like(th_P, float("nan"))
    px.poetx_linear_fwd(desc, X, W, pi_R, pi_P, blk_R, blk_P, Z, B, ws)
    px.poetx_linear_bwd_input(desc, dZ, W, pi_R, pi_P, blk_R, blk_P, dX, dA, ws)
    px.poetx_linear_bwd_skew(desc, X, dZ, B, dA, pi_R, pi_P, th_R, th_P, dth_R, dth_P, False, ws)
    # the whole backward pass in one call, on a workspace of its own poisoned with NaNs
    ws1 = torch.full((ws.numel() // 4,), float("nan"), dtype=torch.float32, device="cuda").view(torch.uint8)
    dX1 = torch.full_like(dX, float("nan"))
    dth_R1 = torch.full_like(th_R, float("nan"))
    dth_P1 = torch.full_like(th_P, float("nan"))
    px.poetx_linear_bwd(desc, X, dZ, B, W, pi_R, pi_P, blk_R, blk_P, th_R, th_P, dX1, dth_R1, dth_P1, False, ws1)
    torch.cuda.synchronize()
    return {"G_R": G_R, "G_P": G_P, "Z": to_np(Z), "B": to_np(B), "dX": to_np(dX), "dA": to_np(dA),
            "dtheta_R": to_np(dth_R), "dtheta_P": to_np(dth_P),
            "one_call": {"dX": to_np(dX1), "dtheta_R": to_np(dth_R1), "dtheta_P": to_np(dth_P1)},
            "dev": {"X": X, "dZ": dZ, "W": W, "pi_R": pi_R, "pi_P": pi_P, "blk_R": blk_R, "blk_P": blk_P,
                    "Z": Z, "B": B, "dX": dX, "dA": dA, "th_R": th_R, "th_P": th_P, "desc": desc, "ws": ws}}
