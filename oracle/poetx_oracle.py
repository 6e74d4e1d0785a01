"""fp64 CPU oracle for the POET-X linear-layer hot path.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain statement of what the
HIP library must compute.  Only the tests, the smoke check and the benchmark's
CPU-baseline leg may import it; the product path never does, and this module
imports nothing from the product (numpy only).

Every routine works in float64 and follows the paper's own order of operations
and notation; there is no tiling, fusion or reordering beyond what the cited
passage states.  ``numpy.matmul`` is the only library primitive used as a step.

Conventions (the paper mixes several; one reading is fixed here)
---------------------------------------------------------------
* ``m = d_in``, ``n = d_out``.  The paper's ``W0`` is m x n (Sec. 2, Eq. 1); the
  *stored* weight is ``W = W0^T`` (n x m, out x in), the ``W`` of Eq. 4.
* Activations are column form, features x tokens: ``X`` is m x N and
  ``Z = P^T W R^T X`` is n x N  (Eq. 1 with Eq. 3's input-centric grouping).
* A permutation ``pi`` is a 0-based bijection; its matrix ``Psi`` has
  ``Psi[i, pi[i]] = 1`` so ``(Psi V)[i, :] = V[pi[i], :]`` (row gather) and
  ``(Psi^T V)[pi[i], :] = V[i, :]`` (row scatter)  (Eq. 5).
* ``R = Psi_R^T Diag(G_R^0 ... G_R^{nb-1}) Psi_R`` (Eq. 2), i.e.
  ``R[pi[i], pi[j]] = D[i, j]``; ``P`` likewise with ``pi_P``, ``G_P``.
* ``Q = skew(theta)``: theta is the packed strict upper triangle in row-major
  order, ``Q[i, j] = +theta`` for ``i < j``, ``Q[j, i] = -theta`` (Sec. 3.4).
* ``G = CNP_k(Q) = (I + Q)(I + sum_{i=1..k} Q^i)`` (Eq. 8 is k = 3).
* Ragged tail (d not a multiple of b): ``nb = ceil(d / b)``; the last block has
  side ``r = d - b (nb - 1)``.  Its theta row still has ``b(b-1)/2`` slots, only
  those with ``i < j < r`` are used; the others are ignored and get zero
  gradient.  Equivalent to padding the last block with identity.

Pin status (see tests/test_oracle_pins.py): every function below is pinned by
dense materialisation, closed forms of the Cayley transform, the orthogonality
defect identity, singular-value preservation, or central finite differences.
The paper prints no worked numerical example, so no stored paper values exist.
``weight_quantize_q8`` / ``weight_dequantize_q8`` (Sec. 3.6): the paper does not
state its quantisation scheme, so the scheme is this build's reading and is
"parity unpinned" against the paper; the routines are pinned to that reading's
own definition (error bound, code range, exact round trips, idempotence).
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------
# skew_symmetric  (Sec. 3.4: packed upper triangle -> Q = -Q^T)
# --------------------------------------------------------------------------
def packed_index(i: int, j: int, b: int) -> int:
    """Slot of entry (i, j), i < j, in the row-major strict upper triangle."""
    assert 0 <= i < j < b
    return i * b - i * (i + 1) // 2 + (j - i - 1)


def n_blocks(d: int, b: int) -> int:
    return -(-d // b)


def tail_side(d: int, b: int) -> int:
    """Side of the last block (== b when b divides d)."""
    return d - b * (n_blocks(d, b) - 1)


def skew_from_packed(theta: np.ndarray, b: int, d: int | None = None) -> np.ndarray:
    """theta [nb, b(b-1)/2] -> Q [nb, b, b], skew-symmetric (Sec. 3.4).

    If ``d`` is given and b does not divide it, entries of the last block with
    row or column index >= tail side are zero whatever theta holds there.
    """
    theta = np.asarray(theta, dtype=F64)
    nb = theta.shape[0]
    assert theta.shape[1] == b * (b - 1) // 2
    Q = np.zeros((nb, b, b), dtype=F64)
    iu, ju = np.triu_indices(b, k=1)  # row-major strict upper triangle
    Q[:, iu, ju] = theta
    Q[:, ju, iu] = -theta
    if d is not None:
        assert nb == n_blocks(d, b)
        r = tail_side(d, b)
        Q[nb - 1, r:, :] = 0.0
        Q[nb - 1, :, r:] = 0.0
    return Q


def packed_from_skew_grad(dQ: np.ndarray, b: int, d: int | None = None) -> np.ndarray:
    """Gradient on the packed parameters from the gradient on the full Q.

    Q = U - U^T with U the strict upper triangle holding theta, hence
    d/dtheta[i,j] = dQ[i,j] - dQ[j,i] for i < j (Sec. 3.4: gradients live on
    the packed form).  Unused tail slots get exactly zero.
    """
    dQ = np.asarray(dQ, dtype=F64)
    nb = dQ.shape[0]
    iu, ju = np.triu_indices(b, k=1)
    dtheta = dQ[:, iu, ju] - dQ[:, ju, iu]
    if d is not None:
        r = tail_side(d, b)
        dead = (iu >= r) | (ju >= r)
        dtheta[nb - 1, dead] = 0.0
    return dtheta


# --------------------------------------------------------------------------
# cayley_neumann  (Sec. 3.4, Eq. 8)
# --------------------------------------------------------------------------
def cnp(Q: np.ndarray, k: int) -> np.ndarray:
    """G = (I + Q)(I + Q + Q^2 + ... + Q^k), batched over the leading axis."""
    Q = np.asarray(Q, dtype=F64)
    assert k >= 1
    b = Q.shape[-1]
    eye = np.broadcast_to(np.eye(b, dtype=F64), Q.shape)
    series = eye.copy()
    power = eye.copy()
    for _ in range(k):
        power = power @ Q
        series = series + power
    return (eye + Q) @ series


def cayley_exact(Q: np.ndarray) -> np.ndarray:
    """The exact Cayley transform (I + Q)(I - Q)^{-1} the series truncates."""
    Q = np.asarray(Q, dtype=F64)
    b = Q.shape[-1]
    eye = np.eye(b, dtype=F64)
    # (I+Q)(I-Q)^{-1}: the factors commute, so solve (I-Q) C = (I+Q).
    return np.linalg.solve(eye - Q, eye + Q)


def cnp_bwd(Q: np.ndarray, dG: np.ndarray, k: int) -> np.ndarray:
    """dL/dQ (unconstrained, full b x b) from dL/dG for G = CNP_k(Q).

    Expanding Eq. 8 for general k gives G = I + 2 sum_{p=1..k} Q^p + Q^{k+1}.
    With d(Q^p) = sum_{j=0..p-1} Q^j dQ Q^{p-1-j} the chain rule yields
        dQ = sum_p c_p sum_{j=0..p-1} (Q^T)^j dG (Q^T)^{p-1-j},
    c_p = 2 for p <= k and c_{k+1} = 1.  At k = 3 this is the paper's
    2 grad_1 + 2 grad_2 + 2 grad_3 + grad_4 (Sec. 3.4, backward display).
    """
    Q = np.asarray(Q, dtype=F64)
    dG = np.asarray(dG, dtype=F64)
    b = Q.shape[-1]
    Qt = np.swapaxes(Q, -1, -2)
    pw = [np.broadcast_to(np.eye(b, dtype=F64), Q.shape).copy()]
    for _ in range(k):
        pw.append(pw[-1] @ Qt)  # pw[j] = (Q^T)^j
    out = np.zeros_like(Q)
    for p in range(1, k + 2):
        c = 2.0 if p <= k else 1.0
        for j in range(p):
            out += c * (pw[j] @ dG @ pw[p - 1 - j])
    return out


# --------------------------------------------------------------------------
# dense materialisation  (Eq. 2, Eq. 5, Eq. 7)
# --------------------------------------------------------------------------
def perm_matrix(pi: np.ndarray) -> np.ndarray:
    """Psi with Psi[i, pi[i]] = 1  (Eq. 5, first identity)."""
    pi = np.asarray(pi)
    d = pi.shape[0]
    Psi = np.zeros((d, d), dtype=F64)
    Psi[np.arange(d), pi] = 1.0
    return Psi


def block_diag(G: np.ndarray, d: int) -> np.ndarray:
    """Diag(G^0, ..., G^{nb-1}) as a dense d x d matrix (Eq. 7); the last block
    contributes only its leading r x r part when b does not divide d."""
    nb, b, _ = G.shape
    assert nb == n_blocks(d, b)
    D = np.zeros((d, d), dtype=F64)
    for j in range(nb):
        lo = j * b
        s = min(b, d - lo)
        D[lo:lo + s, lo:lo + s] = G[j, :s, :s]
    return D


def dense_orthogonal(G: np.ndarray, pi: np.ndarray, d: int) -> np.ndarray:
    """R = Psi^T Diag(G) Psi  (Eq. 2)."""
    Psi = perm_matrix(pi)
    return Psi.T @ block_diag(G, d) @ Psi


def linear_fwd_dense(X, W, pi_R, pi_P, G_R, G_P):
    """Z = (R W0 P)^T X with W0 = W^T, everything materialised (Eq. 1).
    Returns (Z, W_eff) with W_eff = R W0 P (m x n)."""
    X = np.asarray(X, dtype=F64)
    W = np.asarray(W, dtype=F64)
    n, m = W.shape
    R = dense_orthogonal(G_R, pi_R, m)
    P = dense_orthogonal(G_P, pi_P, n)
    W_eff = R @ W.T @ P
    return W_eff.T @ X, W_eff


# --------------------------------------------------------------------------
# matrix-free structured apply  (Eq. 2 + Eq. 5 + Eq. 7, no dense R)
# --------------------------------------------------------------------------
def _blockdiag_mul_rows(G, V, d, transpose):
    """Diag(op(G)) @ V for V with d rows, block by block (Eq. 7)."""
    nb, b, _ = G.shape
    out = np.empty_like(V)
    for j in range(nb):
        lo = j * b
        s = min(b, d - lo)
        Gj = G[j, :s, :s]
        out[lo:lo + s] = (Gj.T if transpose else Gj) @ V[lo:lo + s]
    return out


def apply_left(V, pi, G, transpose: bool):
    """Psi^T Diag(op(G)) Psi V for V of shape d x cols.

    op(G) = G^T if transpose else G, so this is R V or R^T V of Eq. 2 without
    forming R: gather rows by pi (Eq. 5, first identity), one small product per
    block (Eq. 7), scatter rows by pi (Eq. 5, second identity)."""
    V = np.asarray(V, dtype=F64)
    pi = np.asarray(pi)
    d = V.shape[0]
    Vp = V[pi, :]
    Yp = _blockdiag_mul_rows(np.asarray(G, dtype=F64), Vp, d, transpose)
    out = np.empty_like(Yp)
    out[pi, :] = Yp
    return out


def apply_right(V, pi, G, transpose: bool):
    """V Psi^T Diag(op(G)) Psi for V of shape rows x d  (W0 P, X^T R, ...).

    (V Psi^T)[:, i] = V[:, pi[i]] (Eq. 5, fourth identity); the block product
    acts on column groups; (Y Psi)[:, pi[i]] = Y[:, i] (third identity)."""
    V = np.asarray(V, dtype=F64)
    pi = np.asarray(pi)
    G = np.asarray(G, dtype=F64)
    d = V.shape[1]
    nb, b, _ = G.shape
    Vp = V[:, pi]
    Yp = np.empty_like(Vp)
    for j in range(nb):
        lo = j * b
        s = min(b, d - lo)
        Gj = G[j, :s, :s]
        Yp[:, lo:lo + s] = Vp[:, lo:lo + s] @ (Gj.T if transpose else Gj)
    out = np.empty_like(Yp)
    out[:, pi] = Yp
    return out


# --------------------------------------------------------------------------
# the POET-X linear layer, input-centric  (Eq. 3, Eq. 4, Eq. 6, Eq. 10)
# --------------------------------------------------------------------------
def permuted_weight(W, pi_R, pi_P):
    """W' = Psi_P W Psi_R^T, i.e. W'[i, j] = W[pi_P[i], pi_R[j]]  (Eq. 6)."""
    W = np.asarray(W, dtype=F64)
    return W[np.asarray(pi_P), :][:, np.asarray(pi_R)]


def linear_fwd(X, W, pi_R, pi_P, G_R, G_P):
    """Forward chain in the permuted frame (Eq. 6 then Eq. 10):

        X' = Psi_R X;  mm1: A' = D_R^T X';  mm2: B' = W' A';
        mm3: Z' = D_P^T B';  Z = Psi_P^T Z'.

    Returns dict with Z (physical row order) and the permuted-frame
    intermediates Xp, Ap, Bp (Bp is the one activation the fast variant saves).
    """
    X = np.asarray(X, dtype=F64)
    W = np.asarray(W, dtype=F64)
    n, m = W.shape
    G_R = np.asarray(G_R, dtype=F64)
    G_P = np.asarray(G_P, dtype=F64)
    Xp = X[np.asarray(pi_R), :]
    Ap = _blockdiag_mul_rows(G_R, Xp, m, transpose=True)
    Wp = permuted_weight(W, pi_R, pi_P)
    Bp = Wp @ Ap
    Zp = _blockdiag_mul_rows(G_P, Bp, n, transpose=True)
    Z = np.empty_like(Zp)
    Z[np.asarray(pi_P), :] = Zp
    return {"Z": Z, "Xp": Xp, "Ap": Ap, "Bp": Bp, "Wp": Wp}


def _block_outer(U, V, d, b):
    """Per-block U_j V_j^T (b x b each, reduction over tokens); rows/cols past
    the tail side of the last block stay zero."""
    nb = n_blocks(d, b)
    out = np.zeros((nb, b, b), dtype=F64)
    for j in range(nb):
        lo = j * b
        s = min(b, d - lo)
        out[j, :s, :s] = U[lo:lo + s] @ V[lo:lo + s].T
    return out


def linear_bwd(dZ, fwd, pi_R, pi_P, G_R, G_P):
    """Backward of the chain (Sec. 3.5, the three bullet items):

        dZ' = Psi_P dZ
        mm3: dG_P^j = B'_j dZ'_j^T,   dB' = D_P dZ'
        mm2: dA' = W'^T dB'            (no weight gradient: W is frozen)
        mm1: dG_R^j = X'_j dA'_j^T,   dX' = D_R dA';   dX = Psi_R^T dX'.

    Returns dict with dX (physical order), dG_R, dG_P ([nb, b, b]) and the
    permuted-frame dBp, dAp.
    """
    dZ = np.asarray(dZ, dtype=F64)
    G_R = np.asarray(G_R, dtype=F64)
    G_P = np.asarray(G_P, dtype=F64)
    n, m = fwd["Wp"].shape
    b = G_R.shape[-1]
    dZp = dZ[np.asarray(pi_P), :]
    dG_P = _block_outer(fwd["Bp"], dZp, n, b)
    dBp = _blockdiag_mul_rows(G_P, dZp, n, transpose=False)
    dAp = fwd["Wp"].T @ dBp
    dG_R = _block_outer(fwd["Xp"], dAp, m, b)
    dXp = _blockdiag_mul_rows(G_R, dAp, m, transpose=False)
    dX = np.empty_like(dXp)
    dX[np.asarray(pi_R), :] = dXp
    return {"dX": dX, "dG_R": dG_R, "dG_P": dG_P, "dBp": dBp, "dAp": dAp}


def linear_fwd_bwd_from_theta(X, dZ, W, pi_R, pi_P, theta_R, theta_P, b, k):
    """Whole hot path from the packed parameters: skew -> CNP -> forward ->
    backward -> CNP backward -> packed gradient.  Returns a dict with
    G_R, G_P, Z, Bp, dX, dG_R, dG_P, dtheta_R, dtheta_P."""
    W = np.asarray(W, dtype=F64)
    n, m = W.shape
    Q_R = skew_from_packed(theta_R, b, m)
    Q_P = skew_from_packed(theta_P, b, n)
    G_R = cnp(Q_R, k)
    G_P = cnp(Q_P, k)
    f = linear_fwd(X, W, pi_R, pi_P, G_R, G_P)
    g = linear_bwd(dZ, f, pi_R, pi_P, G_R, G_P)
    dth_R = packed_from_skew_grad(cnp_bwd(Q_R, g["dG_R"], k), b, m)
    dth_P = packed_from_skew_grad(cnp_bwd(Q_P, g["dG_P"], k), b, n)
    return {"G_R": G_R, "G_P": G_P, "Z": f["Z"], "Bp": f["Bp"], "Ap": f["Ap"],
            "dX": g["dX"], "dG_R": g["dG_R"], "dG_P": g["dG_P"], "dAp": g["dAp"],
            "dBp": g["dBp"], "dtheta_R": dth_R, "dtheta_P": dth_P}


# --------------------------------------------------------------------------
# POET-XQ  (Sec. 3.6: the frozen base weight is stored in INT8 and dequantised
# whenever it is needed).  The paper does not give the scheme; this reading:
# symmetric absmax per output row,  s_i = max_k |W[i,k]| / 127  (1 for a zero
# row),  q[i,k] = round-half-even(W[i,k] / s_i) clamped to [-127, 127],
# W[i,k] ~ s_i q[i,k].  The scale and the rounding decision are taken in fp32,
# the precision the device uses, so that the integer codes are comparable bit
# for bit; everything downstream of the codes is fp64.
# --------------------------------------------------------------------------
def weight_quantize_q8(W: np.ndarray):
    """W (n x m, values already in the storage dtype) -> (q int8 n x m, scale float32 n)."""
    W32 = np.asarray(W, dtype=np.float32)
    amax = np.max(np.abs(W32), axis=1)
    scale = np.where(amax > 0, amax / np.float32(127.0), np.float32(1.0)).astype(np.float32)
    q = np.rint(W32 / scale[:, None])          # fp32 division, round half to even
    q = np.clip(q, -127.0, 127.0).astype(np.int8)
    return q, scale


def weight_dequantize_q8(q: np.ndarray, scale: np.ndarray) -> np.ndarray:
    """(q, scale) -> the weight the layer multiplies by, fp64 n x m: s_i * q[i,k] exactly."""
    return np.asarray(scale, dtype=F64)[:, None] * np.asarray(q, dtype=F64)
