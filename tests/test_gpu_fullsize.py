"""GPU parity at the full benchmark sizes (Llama-1B / 3B / 8B shaped projections,
N = 16384 tokens), in exactly the launch configuration bench.py times.

The fp64 oracle cannot run whole layers of this size in seconds, so it computes
what it can one piece at a time, each piece exact for the entries it covers:
  * the forward and input-gradient chains are independent per token, so a sample of
    token columns of Z, B and dX is computed by the oracle's own chain on those columns;
  * the parameter gradient of one block needs the reduction over all tokens but only
    b rows of B' (resp. dA'), so sampled blocks of each side are computed in full."""
import numpy as np
import pytest
import torch

from oracle import poetx_oracle as orc
from workloads import draw_projection, get_config
from tests.harness import TOL, rel_err, run_layer

pytestmark = pytest.mark.gpu

CASES = [  # (config key, projection index)
    (3, 1), (3, 6),            # llama1b: k 2048x2048, down 2048x5632
    (4, 2),                    # llama3b: v 1024x3072 (k = 5)
    (5, 1), (5, 4), (5, 6),    # llama8b b=256: k 1024x4096, gate 14336x4096, down 4096x14336
    (6, 2), (6, 6),            # llama8b b=512: v, down
]


@pytest.mark.parametrize("cfg_key,proj", CASES)
def test_fullsize_sampled(lib, cfg_key, proj):
    cfg = get_config(cfg_key)
    data = draw_projection(cfg, proj)
    m, n, N, b, k = data["m"], data["n"], data["N"], data["b"], data["k"]
    print(f"case {cfg.name} {cfg.projections[proj].name} n={n} m={m} N={N} b={b} k={k}", flush=True)
    res = run_layer(data, "bf16")
    tol = TOL["bf16"]
    W, X, dZ, pi_R, pi_P = data["W"], data["X"], data["dZ"], data["pi_R"], data["pi_P"]
    G_R = orc.cnp(orc.skew_from_packed(data["theta_R"], b, m), k)
    G_P = orc.cnp(orc.skew_from_packed(data["theta_P"], b, n), k)
    assert rel_err(res["G_R"], G_R) <= tol and rel_err(res["G_P"], G_P) <= tol
    eye = np.eye(b)
    assert rel_err(res["G_R"] - eye, G_R - eye) <= tol and rel_err(res["G_P"] - eye, G_P - eye) <= tol

    # --- sampled token columns: forward, saved activation, input gradient
    rng = np.random.Generator(np.random.PCG64(99 + cfg_key * 10 + proj))
    T = np.sort(rng.choice(N, size=48, replace=False))
    T[0], T[-1] = 0, N - 1
    f = orc.linear_fwd(X[:, T], W, pi_R, pi_P, G_R, G_P)
    g = orc.linear_bwd(dZ[:, T], f, pi_R, pi_P, G_R, G_P)
    B_ref = np.empty_like(f["Bp"])
    B_ref[pi_P, :] = f["Bp"]
    errs = {"Z": rel_err(res["Z"][:, T], f["Z"]), "B": rel_err(res["B"][:, T], B_ref),
            "dX": rel_err(res["dX"][:, T], g["dX"])}

    # --- sampled blocks: packed-parameter gradients (reduction over all N tokens)
    A_phys = orc.apply_left(X, pi_R, G_R, True)       # A = R^T X
    dB_phys = orc.apply_left(dZ, pi_P, G_P, False)    # dB = P dZ
    nbR, nbP = orc.n_blocks(m, b), orc.n_blocks(n, b)
    for side, nb in (("P", nbP), ("R", nbR)):
        for j in sorted({0, nb - 1, int(rng.integers(0, nb))}):
            rows = slice(j * b, (j + 1) * b)
            if side == "P":   # dG_P^j = B'_j dZ'_j^T,  B'_j = W[pi_P[rows], :] A
                dG = (W[pi_P[rows], :] @ A_phys) @ dZ[pi_P[rows], :].T
                Q = orc.skew_from_packed(data["theta_P"][j:j + 1], b)
                got = res["dtheta_P"][j]
            else:             # dG_R^j = X'_j dA'_j^T,  dA'_j = W[:, pi_R[rows]]^T dB
                dG = X[pi_R[rows], :] @ (W[:, pi_R[rows]].T @ dB_phys).T
                Q = orc.skew_from_packed(data["theta_R"][j:j + 1], b)
                got = res["dtheta_R"][j]
            ref = orc.packed_from_skew_grad(orc.cnp_bwd(Q, dG[None], k), b)[0]
            errs[f"dtheta_{side}[{j}]"] = rel_err(got, ref)
    bad = {key: v for key, v in errs.items() if not v <= tol}
    print({key: float(f"{v:.3e}") for key, v in errs.items()}, flush=True)
    assert not bad, f"over tolerance {tol}: {bad}"
    assert np.isfinite(res["dtheta_R"]).all() and np.isfinite(res["dtheta_P"]).all()
