"""Pins for the fp64 oracle: each checks it against something the paper or the
mathematics fixes independently of the oracle's own code path."""
import numpy as np
import pytest

from oracle import poetx_oracle as orc

RNG = lambda s: np.random.Generator(np.random.PCG64(s))


def rand_theta(rng, d, b, sigma):
    nb = orc.n_blocks(d, b)
    return rng.standard_normal((nb, b * (b - 1) // 2)) * sigma


# ---------------------------------------------------------------- skew / packing
def test_skew_layout_explicit_loops():
    b, rng = 5, RNG(1)
    th = rng.standard_normal((2, 10))
    Q = orc.skew_from_packed(th, b)
    for blk in range(2):
        s = 0
        for i in range(b):
            for j in range(i + 1, b):
                assert orc.packed_index(i, j, b) == s
                assert Q[blk, i, j] == th[blk, s] and Q[blk, j, i] == -th[blk, s]
                s += 1
        assert np.all(np.diag(Q[blk]) == 0)
    assert np.array_equal(Q, -np.swapaxes(Q, 1, 2))


def test_skew_tail_masks_unused_slots():
    b, d = 4, 6  # tail side 2
    th = np.ones((2, 6))
    Q = orc.skew_from_packed(th, b, d)
    assert np.all(Q[1, 2:, :] == 0) and np.all(Q[1, :, 2:] == 0) and Q[1, 0, 1] == 1
    G = orc.cnp(Q, 3)
    assert np.array_equal(G[1, 2:, 2:], np.eye(2))  # identity padding


# ---------------------------------------------------------------- Eq. 5 identities
def test_permutation_identities():
    rng = RNG(2)
    m, n = 7, 5
    W = rng.standard_normal((m, n))
    pp, pq = rng.permutation(m), rng.permutation(n)
    Pm, Pn = orc.perm_matrix(pp), orc.perm_matrix(pq)
    inv_p, inv_q = np.argsort(pp), np.argsort(pq)
    assert np.array_equal(Pm @ W, W[pp, :])
    assert np.array_equal(Pm.T @ W, W[inv_p, :])
    assert np.array_equal(W @ Pn, W[:, inv_q])
    assert np.array_equal(W @ Pn.T, W[:, pq])
    assert np.array_equal(Pm @ Pm.T, np.eye(m))


# ---------------------------------------------------------------- (b) CNP vs exact Cayley
@pytest.mark.parametrize("t", [0.3, -0.05, 0.7])
def test_cnp_b2_closed_form(t):
    Q = np.array([[[0.0, t], [-t, 0.0]]])
    C = np.array([[1 - t * t, 2 * t], [-2 * t, 1 - t * t]]) / (1 + t * t)
    assert np.allclose(orc.cayley_exact(Q[0]), C, atol=1e-15)
    assert np.allclose(orc.cnp(Q, 3)[0], (1 - t ** 4) * C, atol=1e-15)
    # general k: Q^2 = -t^2 I so Q^{k+1} is known in closed form
    for k in (1, 2, 4, 5):
        Qk1 = np.linalg.matrix_power(Q[0], k + 1)
        assert np.allclose(orc.cnp(Q, k)[0], C @ (np.eye(2) - Qk1), atol=1e-15)


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_cnp_truncation_error_is_norm_power(k):
    rng = RNG(3)
    b = 16
    Q = orc.skew_from_packed(rand_theta(rng, 3 * b, b, 0.05), b)
    G = orc.cnp(Q, k)
    for j in range(3):
        C = orc.cayley_exact(Q[j])
        assert np.allclose(C.T @ C, np.eye(b), atol=1e-13)
        q = np.linalg.norm(Q[j], 2)
        assert q < 1
        err = np.linalg.norm(G[j] - C, 2)
        assert err == pytest.approx(q ** (k + 1), rel=1e-9)


def test_cnp_k3_expansion_and_regrouping():
    rng = RNG(4)
    Q = orc.skew_from_packed(rand_theta(rng, 12, 12, 0.1), 12)[0]
    Q2 = Q @ Q
    I = np.eye(12)
    eq8 = I + 2 * Q + 2 * Q2 + 2 * Q2 @ Q + Q2 @ Q2
    eq9 = 2 * (Q + Q2 + Q2 @ Q) + Q2 @ Q2 + I
    G = orc.cnp(Q[None], 3)[0]
    assert np.allclose(G, eq8, atol=1e-15) and np.allclose(G, eq9, atol=1e-15)
    assert np.allclose(G, I + 2 * Q, atol=4 * np.linalg.norm(Q, 2) ** 2)  # R ~ I + 2Q for small Q


def test_cnp_general_k_polynomial():
    rng = RNG(5)
    Q = orc.skew_from_packed(rand_theta(rng, 8, 8, 0.2), 8)[0]
    for k in (1, 2, 4, 5, 6):
        ref = np.eye(8) + np.linalg.matrix_power(Q, k + 1)
        for p in range(1, k + 1):
            ref += 2 * np.linalg.matrix_power(Q, p)
        assert np.allclose(orc.cnp(Q[None], k)[0], ref, atol=1e-14)


# ---------------------------------------------------------------- (c) orthogonality defect
@pytest.mark.parametrize("k", [3, 4, 5])
def test_orthogonality_defect(k):
    rng = RNG(6)
    b = 32
    Q = orc.skew_from_packed(rand_theta(rng, b, b, 0.01), b)[0]
    G = orc.cnp(Q[None], k)[0]
    defect = G.T @ G - np.eye(b)
    Qk1 = np.linalg.matrix_power(Q, k + 1)
    expect = (-2 * Qk1 + Qk1 @ Qk1) if k % 2 == 1 else (-Qk1 @ Qk1)
    assert np.allclose(defect, expect, atol=1e-15)
    q = np.linalg.norm(Q, 2)
    size = np.linalg.norm(defect, 2)
    if k % 2 == 1:
        assert size == pytest.approx(2 * q ** (k + 1), rel=1e-2)
    else:  # even k is far closer to orthogonal
        assert size <= 1.01 * q ** (2 * k + 2) + 1e-15


# ---------------------------------------------------------------- (a) dense vs block
SHAPES = [(8, 8, 1), (8, 12, 2), (12, 8, 4), (16, 24, 8), (10, 7, 4), (13, 13, 8), (6, 9, 16)]


@pytest.mark.parametrize("m,n,b", SHAPES)
@pytest.mark.parametrize("transpose", [False, True])
def test_apply_matches_dense(m, n, b, transpose):
    rng = RNG(10 + m + n + b)
    pi = rng.permutation(m)
    G = orc.cnp(orc.skew_from_packed(rand_theta(rng, m, b, 0.2), b, m), 4) if b > 1 else np.ones((m, 1, 1))
    R = orc.dense_orthogonal(G, pi, m)
    V = rng.standard_normal((m, 5))
    ref = (R.T if transpose else R) @ V
    assert np.allclose(orc.apply_left(V, pi, G, transpose), ref, atol=1e-14)
    U = rng.standard_normal((3, m))
    ref = U @ (R.T if transpose else R)
    assert np.allclose(orc.apply_right(U, pi, G, transpose), ref, atol=1e-14)
    # entry statement of Eq. 2: R[pi[i], pi[j]] = D[i, j]
    D = orc.block_diag(G, m)
    assert np.array_equal(R[np.ix_(pi, pi)], D)


@pytest.mark.parametrize("m,n,b", SHAPES[1:])
def test_linear_block_matches_dense(m, n, b):
    rng = RNG(100 + m + n + b)
    N, k = 6, 4
    W = rng.standard_normal((n, m))
    X = rng.standard_normal((m, N))
    pi_R, pi_P = rng.permutation(m), rng.permutation(n)
    G_R = orc.cnp(orc.skew_from_packed(rand_theta(rng, m, b, 0.2), b, m), k)
    G_P = orc.cnp(orc.skew_from_packed(rand_theta(rng, n, b, 0.2), b, n), k)
    Zd, W_eff = orc.linear_fwd_dense(X, W, pi_R, pi_P, G_R, G_P)
    f = orc.linear_fwd(X, W, pi_R, pi_P, G_R, G_P)
    assert np.allclose(f["Z"], Zd, atol=1e-13)
    # Eq. 4 written with the structured applies in physical order
    Z2 = orc.apply_left(W @ orc.apply_left(X, pi_R, G_R, True), pi_P, G_P, True)
    assert np.allclose(Z2, Zd, atol=1e-13)
    # merged weight (Sec. 2): W_eff = R W0 P via the one-sided applies
    W_eff2 = orc.apply_right(orc.apply_left(W.T, pi_R, G_R, False), pi_P, G_P, False)
    assert np.allclose(W_eff2, W_eff, atol=1e-13)
    # linear in X: dX = W_eff dZ
    dZ = rng.standard_normal((n, N))
    g = orc.linear_bwd(dZ, f, pi_R, pi_P, G_R, G_P)
    assert np.allclose(g["dX"], W_eff @ dZ, atol=1e-13)


def test_identity_special_cases():
    rng = RNG(7)
    m, n, b, N = 12, 8, 4, 5
    W, X = rng.standard_normal((n, m)), rng.standard_normal((m, N))
    pi_R, pi_P = rng.permutation(m), rng.permutation(n)
    zR, zP = np.zeros((3, 6)), np.zeros((2, 6))
    G_R, G_P = orc.cnp(orc.skew_from_packed(zR, b), 4), orc.cnp(orc.skew_from_packed(zP, b), 4)
    f = orc.linear_fwd(X, W, pi_R, pi_P, G_R, G_P)
    assert np.allclose(f["Z"], W @ X, atol=1e-14)  # theta = 0 -> plain linear layer
    assert np.array_equal(orc.apply_left(X, pi_R, G_R, True), X)  # gather . scatter = id, bit for bit
    # b = d with identity permutation: two dense products
    G1 = orc.cnp(orc.skew_from_packed(rand_theta(rng, m, m, 0.1), m), 3)
    G2 = orc.cnp(orc.skew_from_packed(rand_theta(rng, n, n, 0.1), n), 3)
    f = orc.linear_fwd(X, W, np.arange(m), np.arange(n), G1, G2)
    assert np.allclose(f["Z"], G2[0].T @ (W @ (G1[0].T @ X)), atol=1e-14)


# ---------------------------------------------------------------- (d) spectrum
def test_singular_values_preserved_with_exact_cayley():
    rng = RNG(8)
    m, n, b = 24, 16, 8
    W0 = rng.standard_normal((m, n)) * 0.02
    pi_R, pi_P = rng.permutation(m), rng.permutation(n)
    Q_R = orc.skew_from_packed(rand_theta(rng, m, b, 0.1), b)
    Q_P = orc.skew_from_packed(rand_theta(rng, n, b, 0.1), b)
    C_R = np.stack([orc.cayley_exact(q) for q in Q_R])
    C_P = np.stack([orc.cayley_exact(q) for q in Q_P])
    X = np.eye(m)
    _, W_eff = orc.linear_fwd_dense(X, W0.T, pi_R, pi_P, C_R, C_P)
    s0 = np.linalg.svd(W0, compute_uv=False)
    assert np.allclose(np.linalg.svd(W_eff, compute_uv=False), s0, rtol=1e-12)
    # truncated series: relative deviation bounded by (1 + delta)^2 - 1
    for k in (3, 4):
        _, W_k = orc.linear_fwd_dense(X, W0.T, pi_R, pi_P, orc.cnp(Q_R, k), orc.cnp(Q_P, k))
        delta = max(np.linalg.norm(q, 2) for q in list(Q_R) + list(Q_P)) ** (k + 1)
        dev = np.max(np.abs(np.linalg.svd(W_k, compute_uv=False) / s0 - 1))
        assert 0 < dev <= (1 + delta) ** 2 - 1 + 1e-14


# ---------------------------------------------------------------- (e) gradients
def paper_k3_backward(Q, d1):
    """The backward display of Sec. 3.4 (k = 3), both printed forms."""
    Qt, Q2t = Q.T, (Q @ Q).T
    d2 = d1 @ Qt + Qt @ d1
    d3 = d1 @ Q2t + Qt @ d2
    d4 = d2 @ Q2t + Q2t @ d2
    form1 = 2 * d1 + 2 * d2 + 2 * d3 + d4
    form2 = 2 * (d1 + d2) + (2 * Qt + Q2t) @ d2 + (2 * d1 + d2) @ Q2t
    return form1, form2


def test_cnp_bwd_k3_equals_paper_forms():
    rng = RNG(9)
    b = 10
    Q = orc.skew_from_packed(rand_theta(rng, b, b, 0.3), b)[0]
    dG = rng.standard_normal((b, b))
    f1, f2 = paper_k3_backward(Q, dG)
    mine = orc.cnp_bwd(Q[None], dG[None], 3)[0]
    assert np.allclose(f1, f2, atol=1e-13)
    assert np.allclose(mine, f1, atol=1e-13)


@pytest.mark.parametrize("k", [1, 3, 4, 5])
def test_cnp_bwd_finite_difference_unconstrained(k):
    """cnp_bwd treats Q as a free b x b matrix; check entrywise by central differences."""
    rng = RNG(20 + k)
    b = 6
    Q = rng.standard_normal((1, b, b)) * 0.2  # not skew on purpose
    dG = rng.standard_normal((1, b, b))
    g = orc.cnp_bwd(Q, dG, k)
    h = 1e-6
    for (i, j) in [(0, 0), (1, 4), (4, 1), (5, 2)]:
        Qp, Qm = Q.copy(), Q.copy()
        Qp[0, i, j] += h
        Qm[0, i, j] -= h
        fd = (np.sum(dG * orc.cnp(Qp, k)) - np.sum(dG * orc.cnp(Qm, k))) / (2 * h)
        assert fd == pytest.approx(g[0, i, j], rel=1e-7, abs=1e-9)


@pytest.mark.parametrize("m,n,b,k", [(12, 8, 4, 3), (10, 14, 4, 4), (16, 16, 8, 5)])
def test_full_path_finite_difference(m, n, b, k):
    """L(theta, X) = <dZ, Z> with Z from the DENSE definition; gradients from the block path."""
    rng = RNG(30 + m + n + k)
    N = 7
    W = rng.standard_normal((n, m)) * 0.3
    X = rng.standard_normal((m, N))
    dZ = rng.standard_normal((n, N))
    pi_R, pi_P = rng.permutation(m), rng.permutation(n)
    th_R, th_P = rand_theta(rng, m, b, 0.1), rand_theta(rng, n, b, 0.1)
    res = orc.linear_fwd_bwd_from_theta(X, dZ, W, pi_R, pi_P, th_R, th_P, b, k)

    def loss(tR, tP, Xv):
        G_R = orc.cnp(orc.skew_from_packed(tR, b, m), k)
        G_P = orc.cnp(orc.skew_from_packed(tP, b, n), k)
        Z, _ = orc.linear_fwd_dense(Xv, W, pi_R, pi_P, G_R, G_P)
        return np.sum(dZ * Z)

    h = 1e-6
    nbR, nbP, L = th_R.shape[0], th_P.shape[0], th_R.shape[1]
    picks = [(0, 0), (0, L - 1), (nbR - 1, 0), (nbR - 1, L - 1), (nbR // 2, L // 2)]
    rR = orc.tail_side(m, b)
    for (blk, s) in picks:
        tp, tm = th_R.copy(), th_R.copy()
        tp[blk, s] += h
        tm[blk, s] -= h
        fd = (loss(tp, th_P, X) - loss(tm, th_P, X)) / (2 * h)
        assert fd == pytest.approx(res["dtheta_R"][blk, s], rel=1e-7, abs=1e-8)
    picks = [(0, 1), (nbP - 1, 0), (nbP - 1, L - 1), (nbP // 2, L // 3)]
    for (blk, s) in picks:
        tp, tm = th_P.copy(), th_P.copy()
        tp[blk, s] += h
        tm[blk, s] -= h
        fd = (loss(th_R, tp, X) - loss(th_R, tm, X)) / (2 * h)
        assert fd == pytest.approx(res["dtheta_P"][blk, s], rel=1e-7, abs=1e-8)
    for (i, t) in [(0, 0), (m - 1, N - 1), (m // 2, 3)]:
        Xp, Xm = X.copy(), X.copy()
        Xp[i, t] += h
        Xm[i, t] -= h
        fd = (loss(th_R, th_P, Xp) - loss(th_R, th_P, Xm)) / (2 * h)
        assert fd == pytest.approx(res["dX"][i, t], rel=1e-7, abs=1e-8)
    # ragged tail: unused slots carry exactly zero gradient
    if rR < b:
        iu, ju = np.triu_indices(b, k=1)
        dead = (iu >= rR) | (ju >= rR)
        assert np.all(res["dtheta_R"][-1, dead] == 0) and np.any(res["dtheta_R"][-1, ~dead] != 0)


def test_packed_grad_is_skew_projection():
    rng = RNG(11)
    b = 6
    dQ = rng.standard_normal((2, b, b))
    dth = orc.packed_from_skew_grad(dQ, b)
    A = dQ - np.swapaxes(dQ, 1, 2)
    iu, ju = np.triu_indices(b, k=1)
    assert np.array_equal(dth, A[:, iu, ju])
    # directional check: <dQ, skew(t)> = <dtheta, t>
    t = rng.standard_normal((2, b * (b - 1) // 2))
    assert np.sum(dQ * orc.skew_from_packed(t, b)) == pytest.approx(np.sum(dth * t), rel=1e-12)


# ------------------------------------------------------------------ POET-XQ weight codes (Sec. 3.6, this build's reading)
def test_q8_error_bound_range_and_zero_rows():
    rng = np.random.Generator(np.random.PCG64(811))
    W = rng.standard_normal((37, 129)) * 0.02
    W[5] = 0.0
    W[9, :] = 0.0
    W[9, 17] = -0.3                      # a single non-zero: it must become code -127 exactly
    q, s = orc.weight_quantize_q8(W)
    assert q.dtype == np.int8 and s.dtype == np.float32 and q.shape == W.shape and s.shape == (37,)
    assert q.min() >= -127 and q.max() <= 127
    assert s[5] == 1.0 and not q[5].any()
    assert q[9, 17] == -127 and np.count_nonzero(q[9]) == 1
    # every row attains +-127 at its absolute maximum
    assert np.all(np.max(np.abs(q.astype(int)), axis=1)[np.abs(W).max(axis=1) > 0] == 127)
    # rounding to the nearest code: error at most half a step (plus fp32 slack on the quotient)
    err = np.abs(orc.weight_dequantize_q8(q, s) - W.astype(np.float32))
    assert np.all(err <= 0.5 * s[:, None].astype(np.float64) * (1 + 1e-6))


def test_q8_exact_roundtrip_and_idempotence():
    rng = np.random.Generator(np.random.PCG64(812))
    codes = rng.integers(-127, 128, size=(16, 64)).astype(np.int8)
    codes[:, 0] = 127                    # fix the row maximum so that the scale is recovered
    scale = (2.0 ** rng.integers(-12, -4, size=16)).astype(np.float32)   # powers of two: products exact
    W = orc.weight_dequantize_q8(codes, scale)
    q, s = orc.weight_quantize_q8(W)
    assert np.array_equal(q, codes) and np.array_equal(s, scale)
    # quantising a dequantised weight changes nothing
    W2 = rng.standard_normal((8, 50))
    q1, s1 = orc.weight_quantize_q8(W2)
    q2, s2 = orc.weight_quantize_q8(orc.weight_dequantize_q8(q1, s1).astype(np.float32))
    assert np.array_equal(q1, q2)
    assert np.allclose(s1, s2, rtol=1e-6)


def test_q8_half_steps_round_to_even():
    s = np.float32(2.0 ** -7)
    row = np.array([127, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 126.5], dtype=np.float64) * float(s)
    q, sc = orc.weight_quantize_q8(row[None, :])
    assert sc[0] == s
    assert q[0].tolist() == [127, 0, 2, 2, 0, -2, -2, 126]


# ------------------------------------------------------------------ the two-pass form of the series backward
@pytest.mark.parametrize("k", [1, 2, 3, 4, 5, 6])
def test_series_backward_two_pass_regrouping(k):
    """The on-chip backward kernels evaluate dL/dQ as  Y_0 = D, Y_m = W_m^T - Q Y_{m-1}, dL/dQ = Y_k  with
    V_m = Q^m D^T and W_m = 2 (V_0 + .. + V_m) - V_m  (2k products, all left multiplications by Q).
    Written out here in fp64 it must equal the oracle's double sum, which is pinned separately
    against the paper's k = 3 display and against finite differences."""
    rng = np.random.Generator(np.random.PCG64(600 + k))
    b = 12
    Q = orc.skew_from_packed(rng.standard_normal((1, b * (b - 1) // 2)) * 0.2, b)[0]
    D = rng.standard_normal((b, b))
    V = [D.T.copy()]
    for _ in range(k):
        V.append(Q @ V[-1])
    S = np.zeros((b, b))
    W = []
    for m in range(k + 1):
        S = S + V[m]
        W.append(2.0 * S - V[m])
    Y = D.copy()
    for m in range(1, k + 1):
        Y = W[m].T - Q @ Y
    ref = orc.cnp_bwd(Q, D, k)
    assert np.max(np.abs(Y - ref)) <= 1e-12 * max(1.0, np.max(np.abs(ref)))
    # and the forward chain of the same kernels: H_1 = Q, H_{s+1} = 2Q + Q H_s, G = I + H_{k+1}
    H = Q.copy()
    for _ in range(k):
        H = 2.0 * Q + Q @ H
    assert np.max(np.abs(np.eye(b) + H - orc.cnp(Q, k))) <= 1e-13
