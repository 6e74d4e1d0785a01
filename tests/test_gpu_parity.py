"""GPU parity: the HIP library against the fp64 oracle, element by element, on
seeded inputs.  Tolerances (max |gpu - ref| / max |ref| per tensor): 1e-4 for
fp32 tensors, 2e-2 for bf16 tensors; index work is bit-exact."""
import numpy as np
import pytest
import torch

from oracle import poetx_oracle as orc
from workloads import get_config, draw_projection, round_bf16, round_f32
from tests.harness import TOL, build_blocks, rel_err, row_rel_err, run_layer, tdtype, to_dev, to_np, ws_tensor

pytestmark = pytest.mark.gpu
RNG = lambda s: np.random.Generator(np.random.PCG64(s))


def draw_theta(rng, d, b, sigma):
    nb = orc.n_blocks(d, b)
    return round_f32(rng.standard_normal((nb, b * (b - 1) // 2)) * sigma)


def pair(E):
    """bf16 block storage: (E, E^T) per block."""
    return np.stack([E, np.swapaxes(E, 1, 2)], axis=1)


# ------------------------------------------------------------------ cnp_build
@pytest.mark.parametrize("d,b,k", [(64, 32, 3), (256, 32, 4), (96, 64, 4), (1376, 64, 4), (512, 256, 5),
                                   (1024, 512, 5), (40, 8, 1), (48, 16, 2), (256, 256, 1), (768, 256, 2), (1024, 256, 3)])
@pytest.mark.parametrize("precision", ["fp32", "bf16"])
def test_cnp_build(lib, d, b, k, precision):
    rng = RNG(1000 + d + b + k)
    theta = draw_theta(rng, d, b, 0.01 if b < 256 else 0.005)
    th = to_dev(theta, torch.float32)
    nb = theta.shape[0]
    G = torch.empty((nb, b, b), dtype=torch.float32, device="cuda")
    E = torch.empty((nb, 2, b, b), dtype=torch.bfloat16, device="cuda")
    ws = ws_tensor(lib.poetx_cnp_workspace_bytes(d, b))
    lib.poetx_cnp_build(th, d, b, k, lib.CNP_FP32 if precision == "fp32" else lib.CNP_BF16, G, E, ws)
    torch.cuda.synchronize()
    ref = orc.cnp(orc.skew_from_packed(theta, b, d), k)
    tol = 1e-4 if precision == "fp32" else 2e-2
    assert rel_err(to_np(G), ref) <= (1e-6 if precision == "fp32" else tol)
    eye = np.eye(b)
    # the residual must keep the small part of G: compare G - I on its own scale
    assert rel_err(to_np(G) - eye, ref - eye) <= tol
    assert rel_err(to_np(E)[:, 0], ref - eye) <= 2e-2
    assert torch.equal(E[:, 1], E[:, 0].transpose(1, 2))  # stored transpose, bit for bit
    r = orc.tail_side(d, b)
    if r < b:  # identity padding of the ragged tail block, exactly
        Gt = to_np(G)[-1]
        assert np.array_equal(Gt[r:, :], eye[r:, :]) and np.array_equal(Gt[:, r:], eye[:, r:])


# ------------------------------------------------------------------ structured apply
APPLY_SHAPES = [(64, 32, 48), (256, 32, 512), (96, 64, 100), (1376, 64, 1024), (160, 64, 333), (512, 256, 640),
                (40, 8, 7)]


@pytest.mark.parametrize("d,b,cols", APPLY_SHAPES)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("transpose", [False, True])
def test_apply_left(lib, d, b, cols, dtype, transpose):
    rng = RNG(2000 + d + b + cols)
    rnd = round_f32 if dtype == "f32" else round_bf16
    theta = draw_theta(rng, d, b, 0.02)
    V = rnd(rng.standard_normal((d, cols)))
    pi = rng.permutation(d).astype(np.int32)
    blocks, G = build_blocks(theta, d, b, 4, dtype, lib.CNP_FP32)
    Vd = to_dev(V, tdtype(dtype))
    out = torch.empty_like(Vd)
    lib.poetx_perm_blockdiag_apply_left(Vd, out, torch.from_numpy(pi).cuda(), blocks, b, transpose)
    torch.cuda.synchronize()
    G_used = G if dtype == "f32" else to_np(blocks)[:, 0] + np.eye(b)  # the blocks the kernel was given
    ref = orc.apply_left(V, pi, G_used, transpose)
    assert rel_err(to_np(out), ref) <= TOL[dtype]
    ref_exactG = orc.apply_left(V, pi, orc.cnp(orc.skew_from_packed(theta, b, d), 4), transpose)
    assert rel_err(to_np(out), ref_exactG) <= TOL[dtype]


@pytest.mark.parametrize("d,b,rows", [(64, 32, 48), (96, 64, 130), (1376, 64, 512), (512, 256, 300), (40, 8, 5)])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("transpose", [False, True])
def test_apply_right(lib, d, b, rows, dtype, transpose):
    rng = RNG(3000 + d + b + rows)
    rnd = round_f32 if dtype == "f32" else round_bf16
    theta = draw_theta(rng, d, b, 0.02)
    V = rnd(rng.standard_normal((rows, d)))
    pi = rng.permutation(d).astype(np.int32)
    blocks, G = build_blocks(theta, d, b, 4, dtype, lib.CNP_FP32)
    Vd = to_dev(V, tdtype(dtype))
    out = torch.empty_like(Vd)
    lib.poetx_perm_blockdiag_apply_right(Vd, out, torch.from_numpy(pi).cuda(), blocks, b, transpose)
    torch.cuda.synchronize()
    ref = orc.apply_right(V, pi, orc.cnp(orc.skew_from_packed(theta, b, d), 4), transpose)
    assert rel_err(to_np(out), ref) <= TOL[dtype]


@pytest.mark.parametrize("d,b,cols", [(256, 32, 512), (1376, 64, 256), (1024, 256, 512), (96, 64, 77)])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_apply_indexing_bit_exact(lib, d, b, cols, dtype):
    """Blocks that are themselves permutation matrices make the whole apply a pure row
    permutation; on small-integer data every product and sum is exact, so the result must
    equal numpy index arithmetic bit for bit (gather, block offsets, scatter)."""
    rng = RNG(4000 + d + b)
    nb = orc.n_blocks(d, b)
    r = orc.tail_side(d, b)
    G = np.zeros((nb, b, b))
    for j in range(nb):
        s = b if j < nb - 1 else r
        sig = rng.permutation(s)
        G[j, np.arange(s), sig] = 1.0
        G[j, np.arange(s, b), np.arange(s, b)] = 1.0
    V = rng.integers(-64, 65, size=(d, cols)).astype(np.float64)
    pi = rng.permutation(d).astype(np.int32)
    blocks = to_dev(G if dtype == "f32" else pair(G - np.eye(b)), tdtype(dtype))
    Vd = to_dev(V, tdtype(dtype))
    for transpose in (False, True):
        out = torch.empty_like(Vd)
        lib.poetx_perm_blockdiag_apply_left(Vd, out, torch.from_numpy(pi).cuda(), blocks, b, transpose)
        torch.cuda.synchronize()
        assert np.array_equal(to_np(out), orc.apply_left(V, pi, G, transpose))
    # identity blocks: gather followed by scatter is the identity map, bit for bit
    eye = np.broadcast_to(np.eye(b), (nb, b, b)).copy()
    blocks = to_dev(eye if dtype == "f32" else pair(eye * 0), tdtype(dtype))
    Vr = to_dev((round_f32 if dtype == "f32" else round_bf16)(rng.standard_normal((d, cols))), tdtype(dtype))
    out = torch.empty_like(Vr)
    lib.poetx_perm_blockdiag_apply_left(Vr, out, torch.from_numpy(pi).cuda(), blocks, b, True)
    torch.cuda.synchronize()
    assert torch.equal(out, Vr)


def test_perm_validate(lib):
    rng = RNG(5)
    d = 1000
    pi = rng.permutation(d).astype(np.int32)
    scratch = torch.empty(d + 1, dtype=torch.int32, device="cuda")
    assert lib.poetx_perm_validate(torch.from_numpy(pi).cuda(), scratch)
    bad = pi.copy()
    bad[3] = bad[4]
    assert not lib.poetx_perm_validate(torch.from_numpy(bad).cuda(), scratch)
    bad = pi.copy()
    bad[0] = d
    assert not lib.poetx_perm_validate(torch.from_numpy(bad).cuda(), scratch)


# ------------------------------------------------------------------ whole layer, configs 1 and 2
def check_layer(res, ref, pi_P, dtype):
    """Every output against the oracle: on the tensor's scale (the tolerance's metric) and row by row
    (a feature across tokens / a block of packed parameters on its own scale).  The blocks are
    compared on the scale of G - I: G itself is dominated by the identity."""
    tol = TOL[dtype]
    errs = {}
    B_ref = np.empty_like(ref["Bp"])
    B_ref[pi_P, :] = ref["Bp"]  # the library keeps B in physical feature order
    eye = np.eye(ref["G_R"].shape[-1])
    pairs = {"G_R-I": (res["G_R"] - eye, ref["G_R"] - eye), "G_P-I": (res["G_P"] - eye, ref["G_P"] - eye),
             "Z": (res["Z"], ref["Z"]), "B": (res["B"], B_ref), "dX": (res["dX"], ref["dX"]),
             "dtheta_R": (res["dtheta_R"], ref["dtheta_R"]), "dtheta_P": (res["dtheta_P"], ref["dtheta_P"])}
    if "one_call" in res:   # poetx_linear_bwd: the same three outputs from the single backward call
        for key in ("dX", "dtheta_R", "dtheta_P"):
            pairs["one-call " + key] = (res["one_call"][key], ref[key])
    for key, (got, want) in pairs.items():
        errs[key] = rel_err(got, want)
        errs["row " + key] = row_rel_err(got, want)
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, f"over tolerance {tol}: {bad} (all: {errs})"
    return errs


def test_config1_fp32_layer(lib):
    cfg = get_config(1)
    data = draw_projection(cfg, 0)
    res = run_layer(data, "f32")
    ref = orc.linear_fwd_bwd_from_theta(data["X"], data["dZ"], data["W"], data["pi_R"], data["pi_P"],
                                        data["theta_R"], data["theta_P"], data["b"], data["k"])
    check_layer(res, ref, data["pi_P"], "f32")


@pytest.mark.parametrize("proj", range(7))
def test_config2_bf16_layer(lib, proj):
    cfg = get_config(2)
    data = draw_projection(cfg, proj)
    res = run_layer(data, "bf16")
    ref = orc.linear_fwd_bwd_from_theta(data["X"], data["dZ"], data["W"], data["pi_R"], data["pi_P"],
                                        data["theta_R"], data["theta_P"], data["b"], data["k"])
    check_layer(res, ref, data["pi_P"], "bf16")
    # ragged tail: unused parameter slots get exactly zero gradient
    for side, d in (("dtheta_R", data["m"]), ("dtheta_P", data["n"])):
        r = orc.tail_side(d, data["b"])
        if r < data["b"]:
            iu, ju = np.triu_indices(data["b"], k=1)
            assert np.all(res[side][-1, (iu >= r) | (ju >= r)] == 0)


@pytest.mark.parametrize("proj", [4, 6])   # gate: ragged output side; down: ragged input side
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_config2_dead_slots_of_the_tail_block_are_ignored(lib, proj, dtype):
    """The packed parameters of a ragged tail block keep b(b-1)/2 slots; those with an index beyond
    the tail side hold arbitrary non-zero values here.  Forward, input gradient and parameter
    gradients must not see them, and their own gradient must be exactly zero."""
    cfg = get_config(2)
    data = draw_projection(cfg, proj, zero_dead=False)
    b = data["b"]
    iu, ju = np.triu_indices(b, k=1)
    for side, d in (("theta_R", data["m"]), ("theta_P", data["n"])):
        r = orc.tail_side(d, b)
        if r < b:
            dead = (iu >= r) | (ju >= r)
            data[side][-1, dead] = round_f32(RNG(77 + proj).standard_normal(dead.sum()) * 3.0 + 5.0)   # loud
            assert np.all(data[side][-1, dead] != 0)
    if dtype == "f32":
        for key in ("X", "dZ", "W"):
            data[key] = round_f32(data[key])
    res = run_layer(data, dtype)
    ref = orc.linear_fwd_bwd_from_theta(data["X"], data["dZ"], data["W"], data["pi_R"], data["pi_P"],
                                        data["theta_R"], data["theta_P"], b, data["k"])
    check_layer(res, ref, data["pi_P"], dtype)
    for side, d in (("dtheta_R", data["m"]), ("dtheta_P", data["n"])):
        r = orc.tail_side(d, b)
        if r < b:
            assert np.all(res[side][-1, (iu >= r) | (ju >= r)] == 0)


def test_config2_fp32_storage_and_accumulate(lib):
    """Same shapes in fp32 storage (tight tolerance) and the accumulate flag of bwd_skew."""
    cfg = get_config(2)
    data = draw_projection(cfg, 6)  # down: 512 x 1376, ragged input side
    for key in ("X", "dZ", "W"):
        data[key] = round_f32(data[key])
    res = run_layer(data, "f32")
    ref = orc.linear_fwd_bwd_from_theta(data["X"], data["dZ"], data["W"], data["pi_R"], data["pi_P"],
                                        data["theta_R"], data["theta_P"], data["b"], data["k"])
    check_layer(res, ref, data["pi_P"], "f32")
    dev = res["dev"]
    dth_R = torch.ones_like(dev["th_R"])
    dth_P = torch.ones_like(dev["th_P"])
    lib.poetx_linear_bwd_skew(dev["desc"], dev["X"], dev["dZ"], dev["B"], dev["dA"], dev["pi_R"], dev["pi_P"],
                              dev["th_R"], dev["th_P"], dth_R, dth_P, True, dev["ws"])
    torch.cuda.synchronize()
    assert rel_err(to_np(dth_R) - 1.0, ref["dtheta_R"]) <= 1e-4
    assert rel_err(to_np(dth_P) - 1.0, ref["dtheta_P"]) <= 1e-4


# ------------------------------------------------------------------ matrix-core shapes (multiples of 256)
def synth_layer(seed, m, n, N, b, k, dtype, sigma_theta=0.01):
    rng = RNG(seed)
    rnd = round_f32 if dtype == "f32" else round_bf16
    return {"m": m, "n": n, "N": N, "b": b, "k": k,
            "X": rnd(rng.standard_normal((m, N))), "dZ": rnd(rng.standard_normal((n, N))),
            "W": rnd(rng.standard_normal((n, m)) * 0.02),
            "theta_R": draw_theta(rng, m, b, sigma_theta), "theta_P": draw_theta(rng, n, b, sigma_theta),
            "pi_R": rng.permutation(m).astype(np.int32), "pi_P": rng.permutation(n).astype(np.int32)}


@pytest.mark.parametrize("m,n,N,b,k", [(512, 256, 512, 64, 4), (256, 768, 256, 256, 5), (1024, 512, 768, 512, 3),
                                       (768, 1024, 1280, 256, 4)])
def test_bf16_layer_matrix_core_shapes(lib, m, n, N, b, k):
    data = synth_layer(7000 + m + n + N + b, m, n, N, b, k, "bf16", 0.01 if b < 256 else 0.005)
    ref = orc.linear_fwd_bwd_from_theta(data["X"], data["dZ"], data["W"], data["pi_R"], data["pi_P"],
                                        data["theta_R"], data["theta_P"], b, k)
    res = run_layer(data, "bf16")
    check_layer(res, ref, data["pi_P"], "bf16")
    # the plain-FMA kernels on the same inputs: both families must agree with the oracle
    lib.poetx_debug_force_fma(True)
    try:
        res2 = run_layer(data, "bf16")
    finally:
        lib.poetx_debug_force_fma(False)
    check_layer(res2, ref, data["pi_P"], "bf16")


@pytest.mark.parametrize("k", [1, 2, 3, 6])
def test_on_chip_series_orders(lib, k):
    """b = 256 runs the series and its backward as one-launch chains with the block resident on
    chip; the chain length is a run-time loop, so every order takes its own path through it
    (k = 1: no intermediate step at all).  theta is drawn larger than in the workloads so
    that the high-order terms are well above the bf16 noise of the low-order ones."""
    m, n, N, b = 256, 512, 256, 256
    data = synth_layer(7300 + k, m, n, N, b, k, "bf16", 0.01)
    ref = orc.linear_fwd_bwd_from_theta(data["X"], data["dZ"], data["W"], data["pi_R"], data["pi_P"],
                                        data["theta_R"], data["theta_P"], b, k)
    res = run_layer(data, "bf16")
    check_layer(res, ref, data["pi_P"], "bf16")


@pytest.mark.parametrize("k", [1, 2, 3])
@pytest.mark.parametrize("b,dtype", [(32, "f32"), (64, "bf16"), (256, "bf16")])
def test_plain_series_orders(lib, k, b, dtype):
    """The plain fp32 series kernels (fp32 tensors, small blocks, and bf16 tensors forced onto them) at
    the short orders: k = 1 runs no intermediate Horner step, k = 2 exactly one."""
    m, n, N = 3 * b, 2 * b, 128
    data = synth_layer(7350 + 10 * k + b, m, n, N, b, k, dtype, 0.01)
    ref = orc.linear_fwd_bwd_from_theta(data["X"], data["dZ"], data["W"], data["pi_R"], data["pi_P"],
                                        data["theta_R"], data["theta_P"], b, k)
    lib.poetx_debug_force_fma(True)
    try:
        res = run_layer(data, dtype, cnp_precision=lib.CNP_FP32)
    finally:
        lib.poetx_debug_force_fma(False)
    check_layer(res, ref, data["pi_P"], dtype)


@pytest.mark.parametrize("m,n,N,b,k", [(256, 384, 256, 64, 4), (640, 128, 384, 128, 3), (128, 128, 128, 32, 5)])
def test_fp32_layer_dense_on_matrix_cores(lib, m, n, N, b, k):
    """fp32 tensors whose dense products fit the fp32 matrix-core kernel (multiples of 128): the layer
    against the oracle at the fp32 tolerance, and the same inputs through the plain-FMA kernels."""
    data = synth_layer(7600 + m + n + N + b, m, n, N, b, k, "f32", 0.01)
    ref = orc.linear_fwd_bwd_from_theta(data["X"], data["dZ"], data["W"], data["pi_R"], data["pi_P"],
                                        data["theta_R"], data["theta_P"], b, k)
    desc = lib.make_desc(m, n, b, k, N, lib.F32)
    assert lib.poetx_linear_path(desc) & lib.PATH_DENSE
    check_layer(run_layer(data, "f32"), ref, data["pi_P"], "f32")
    lib.poetx_debug_force_fma(True)
    try:
        assert not (lib.poetx_linear_path(desc) & lib.PATH_DENSE)
        res2 = run_layer(data, "f32")
    finally:
        lib.poetx_debug_force_fma(False)
    check_layer(res2, ref, data["pi_P"], "f32")


@pytest.mark.parametrize("N", [64, 128, 192, 320, 384, 576])
def test_kernel_family_boundaries(lib, N):
    """Token counts around the tile sizes of the matrix-core kernels (128-token apply tiles, 256-token
    dense tiles, 64-token reduction tiles): each stage falls back to the plain kernels on its own
    when its tiling does not fit, so every mix of the two families must still match the oracle."""
    m, n, b, k = 512, 256, 256, 2
    data = synth_layer(7400 + N, m, n, N, b, k, "bf16", 0.005)
    ref = orc.linear_fwd_bwd_from_theta(data["X"], data["dZ"], data["W"], data["pi_R"], data["pi_P"],
                                        data["theta_R"], data["theta_P"], b, k)
    check_layer(run_layer(data, "bf16"), ref, data["pi_P"], "bf16")


# ------------------------------------------------------------------ merge step W <- R W P
@pytest.mark.parametrize("m,n,b,dtype", [(256, 512, 256, "bf16"), (96, 160, 32, "f32"), (1376, 512, 64, "bf16"),
                                         (1024, 768, 256, "bf16")])
def test_merge_step(lib, m, n, b, dtype):
    """The periodic merge (Sec. 3, after Eq. 2): W_i = R W_{i-1} P.  On the stored weight W = W0^T this is
    W_new = P^T W R^T = apply_right(apply_left(W, P^T), R^T); checked against the dense definition, and
    a forward pass with the merged weight and zero parameters must reproduce the un-merged forward."""
    rng = RNG(9000 + m + n + b)
    rnd = round_f32 if dtype == "f32" else round_bf16
    k, N = 4, 256
    W = rnd(rng.standard_normal((n, m)) * 0.02)
    X = rnd(rng.standard_normal((m, N)))
    th_R, th_P = draw_theta(rng, m, b, 0.01), draw_theta(rng, n, b, 0.01)
    pi_R, pi_P = rng.permutation(m).astype(np.int32), rng.permutation(n).astype(np.int32)
    blk_R, G_R = build_blocks(th_R, m, b, k, dtype, lib.CNP_FP32)
    blk_P, G_P = build_blocks(th_P, n, b, k, dtype, lib.CNP_FP32)
    dt = tdtype(dtype)
    Wd = to_dev(W, dt)
    tmp, Wn = torch.empty_like(Wd), torch.empty_like(Wd)
    pR, pP = torch.from_numpy(pi_R).cuda(), torch.from_numpy(pi_P).cuda()
    lib.poetx_perm_blockdiag_apply_left(Wd, tmp, pP, blk_P, b, True)      # P^T W
    lib.poetx_perm_blockdiag_apply_right(tmp, Wn, pR, blk_R, b, True)     # (P^T W) R^T
    torch.cuda.synchronize()
    Zd, W_eff = orc.linear_fwd_dense(X, W, pi_R, pi_P, orc.cnp(orc.skew_from_packed(th_R, b, m), k),
                                     orc.cnp(orc.skew_from_packed(th_P, b, n), k))
    assert rel_err(to_np(Wn), W_eff.T) <= TOL[dtype]
    # mergeability: plain product with the merged weight == POET-X forward with the factors
    assert rel_err(to_np(Wn) @ X, Zd) <= 2 * TOL[dtype]
    # the merge entry point (both sides through the left-apply kernels): same matrix
    Wm = torch.full_like(Wd, float("nan"))
    wsm = ws_tensor(lib.poetx_merge_workspace_bytes(n, m, lib.F32 if dtype == "f32" else lib.BF16))
    lib.poetx_merge_weight(Wd, Wm, pR, pP, blk_R, blk_P, b, wsm)
    torch.cuda.synchronize()
    assert rel_err(to_np(Wm), W_eff.T) <= TOL[dtype] and row_rel_err(to_np(Wm), W_eff.T) <= TOL[dtype]


# ------------------------------------------------------------------ memory-saving variant
@pytest.mark.parametrize("m,n,N,b,k,dtype", [(512, 256, 512, 256, 4, "bf16"), (256, 256, 512, 32, 4, "f32")])
def test_mem_variant_matches_fast(lib, m, n, N, b, k, dtype):
    """POET-X_mem: no saved activation in forward, B recomputed in backward.  Its outputs are checked
    against the oracle, and -- same kernels -- must equal the fast variant bit for bit."""
    data = synth_layer(9500 + m + n, m, n, N, b, k, dtype)
    fast = run_layer(data, dtype)
    dev = fast["dev"]
    code = lib.F32 if dtype == "f32" else lib.BF16
    desc = lib.make_desc(m, n, b, k, N, code, flags=lib.FLAG_RECOMPUTE_B)
    ws = ws_tensor(lib.poetx_linear_workspace_bytes(desc))
    assert ws.numel() >= (m + n) * N * (4 if dtype == "f32" else 2)
    Z = torch.empty_like(dev["Z"])
    lib.poetx_linear_fwd(desc, dev["X"], dev["W"], dev["pi_R"], dev["pi_P"], dev["blk_R"], dev["blk_P"], Z, None, ws)
    dX, dA = torch.empty_like(dev["dX"]), torch.empty_like(dev["dA"])
    lib.poetx_linear_bwd_input(desc, dev["dZ"], dev["W"], dev["pi_R"], dev["pi_P"], dev["blk_R"], dev["blk_P"], dX, dA, ws)
    B = torch.empty_like(dev["B"])
    lib.poetx_linear_recompute_b(desc, dev["X"], dev["W"], dev["pi_R"], dev["blk_R"], B, ws)
    dR, dP = torch.empty_like(dev["th_R"]), torch.empty_like(dev["th_P"])
    lib.poetx_linear_bwd_skew(desc, dev["X"], dev["dZ"], B, dA, dev["pi_R"], dev["pi_P"], dev["th_R"], dev["th_P"],
                              dR, dP, False, ws)
    torch.cuda.synchronize()
    # against the oracle, on its own: forward, recomputed activation, both backward halves
    ref = orc.linear_fwd_bwd_from_theta(data["X"], data["dZ"], data["W"], data["pi_R"], data["pi_P"],
                                        data["theta_R"], data["theta_P"], b, k)
    mem = {"G_R": fast["G_R"], "G_P": fast["G_P"], "Z": to_np(Z), "B": to_np(B), "dX": to_np(dX),
           "dtheta_R": to_np(dR), "dtheta_P": to_np(dP)}
    check_layer(mem, ref, data["pi_P"], dtype)
    # and the same kernels as the fast variant, so bit for bit the same values
    assert torch.equal(Z, dev["Z"]) and torch.equal(B, dev["B"]) and torch.equal(dX, dev["dX"])
    assert np.array_equal(to_np(dR), fast["dtheta_R"]) and np.array_equal(to_np(dP), fast["dtheta_P"])
    # the one-call backward recomputes B itself when it gets none: the results of the one-call backward on the
    # recomputed B, bit for bit (same kernels, same summation order), and the oracle's
    outs = []
    for sb in (B, None):
        dX1 = torch.full_like(dX, float("nan"))
        dR1, dP1 = torch.full_like(dR, float("nan")), torch.full_like(dP, float("nan"))
        ws.fill_(0xFF)                                   # nothing may depend on what a previous call left behind
        lib.poetx_linear_bwd(desc, dev["X"], dev["dZ"], sb, dev["W"], dev["pi_R"], dev["pi_P"], dev["blk_R"],
                             dev["blk_P"], dev["th_R"], dev["th_P"], dX1, dR1, dP1, False, ws)
        torch.cuda.synchronize()
        outs.append((dX1, dR1, dP1))
    assert all(torch.equal(a, c) for a, c in zip(outs[0], outs[1]))
    assert torch.equal(outs[1][0], dX)
    assert rel_err(to_np(outs[1][1]), ref["dtheta_R"]) <= TOL[dtype] and rel_err(to_np(outs[1][2]), ref["dtheta_P"]) <= TOL[dtype]
    # without the flag a missing saved_B is refused on the host
    with pytest.raises(lib.PoetxError):
        lib.poetx_linear_fwd(dev["desc"], dev["X"], dev["W"], dev["pi_R"], dev["pi_P"], dev["blk_R"], dev["blk_P"],
                             Z, None, dev["ws"])
    with pytest.raises(lib.PoetxError):
        lib.poetx_linear_bwd(dev["desc"], dev["X"], dev["dZ"], None, dev["W"], dev["pi_R"], dev["pi_P"], dev["blk_R"],
                             dev["blk_P"], dev["th_R"], dev["th_P"], dX, dR, dP, False, dev["ws"])


# ------------------------------------------------------------------ quantised base weight (POET-XQ)
def q8_views(buf, n, m):
    """(codes int8 n x m, scales float32 n) of a quantised weight buffer brought to the host."""
    raw = buf.cpu().numpy()
    off = (n * m + 255) // 256 * 256
    return raw[: n * m].view(np.int8).reshape(n, m), raw[off: off + 4 * n].view(np.float32)


@pytest.mark.parametrize("n,m", [(37, 129), (256, 256), (512, 1376)])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_weight_q8_codes_bit_exact(lib, n, m, dtype):
    rng = RNG(8100 + n + m)
    W = (round_f32 if dtype == "f32" else round_bf16)(rng.standard_normal((n, m)) * 0.02)
    W[3] = 0.0                                           # an all-zero row: scale 1, codes 0
    Wd = to_dev(W, tdtype(dtype))
    buf = torch.zeros(lib.poetx_weight_q8_bytes(n, m), dtype=torch.uint8, device="cuda")
    lib.poetx_weight_quantize_q8(Wd, buf)
    out = torch.empty_like(Wd)
    lib.poetx_weight_dequantize_q8(buf, out)
    torch.cuda.synchronize()
    q, s = q8_views(buf, n, m)
    q_ref, s_ref = orc.weight_quantize_q8(W)
    assert np.array_equal(s, s_ref)                      # fp32 scale, bit for bit
    assert np.array_equal(q, q_ref)                      # integer codes, bit for bit
    # the device forms scale * code in fp32 (exactly rounded) and rounds once more to the storage type
    prod32 = s_ref[:, None] * q_ref.astype(np.float32)
    expect = prod32.astype(np.float64) if dtype == "f32" else round_bf16(prod32.astype(np.float64))
    assert np.array_equal(to_np(out), expect)
    assert rel_err(to_np(out), orc.weight_dequantize_q8(q_ref, s_ref)) <= (1e-6 if dtype == "f32" else 2 ** -8)


@pytest.mark.parametrize("m,n,N,b,k,dtype", [(256, 512, 256, 256, 4, "bf16"), (1376, 512, 384, 64, 4, "bf16"),
                                             (96, 160, 128, 32, 3, "f32"), (512, 768, 512, 256, 5, "bf16"),
                                             (1024, 256, 1280, 256, 3, "bf16"), (768, 2048, 768, 256, 2, "bf16")])
@pytest.mark.parametrize("fused", [False, True])
def test_xq_layer(lib, m, n, N, b, k, dtype, fused):
    """Memory-saving variant on an INT8 base weight: every product must be the oracle's on the
    dequantised weight scale_i * q[i][k] (the oracle quantises with its own routine) -- with the weight
    dequantised into the workspace ahead of the products, and with the products converting the codes
    themselves (fused)."""
    data = synth_layer(9700 + m + n, m, n, N, b, k, dtype)
    q_ref, s_ref = orc.weight_quantize_q8(data["W"])
    ref = orc.linear_fwd_bwd_from_theta(data["X"], data["dZ"], orc.weight_dequantize_q8(q_ref, s_ref), data["pi_R"],
                                        data["pi_P"], data["theta_R"], data["theta_P"], b, k)
    dt = tdtype(dtype)
    code = lib.F32 if dtype == "f32" else lib.BF16
    X, dZ, W = to_dev(data["X"], dt), to_dev(data["dZ"], dt), to_dev(data["W"], dt)
    Wq = torch.zeros(lib.poetx_weight_q8_bytes(n, m), dtype=torch.uint8, device="cuda")
    lib.poetx_weight_quantize_q8(W, Wq)
    del W                                                # only the 8-bit weight is kept
    pi_R, pi_P = torch.from_numpy(data["pi_R"]).cuda(), torch.from_numpy(data["pi_P"]).cuda()
    th_R, th_P = to_dev(data["theta_R"], torch.float32), to_dev(data["theta_P"], torch.float32)
    blk_R, G_R = build_blocks(data["theta_R"], m, b, k, dtype)
    blk_P, G_P = build_blocks(data["theta_P"], n, b, k, dtype)
    bad = lib.make_desc(m, n, b, k, N, code, flags=lib.FLAG_W_INT8)   # only valid in the variant that keeps no activation
    assert lib.poetx_linear_workspace_bytes(bad) == 0
    with pytest.raises(lib.PoetxError):
        lib.poetx_linear_fwd(bad, X, Wq, pi_R, pi_P, blk_R, blk_P, torch.empty((n, N), dtype=dt, device="cuda"),
                             torch.empty((n, N), dtype=dt, device="cuda"), ws_tensor(1 << 24))
    lone = lib.make_desc(m, n, b, k, N, code, flags=lib.FLAG_RECOMPUTE_B | lib.FLAG_W_INT8_FUSED)   # nothing to fuse
    assert lib.poetx_linear_workspace_bytes(lone) == 0
    desc = lib.make_desc(m, n, b, k, N, code, flags=lib.FLAG_RECOMPUTE_B | lib.FLAG_W_INT8 | (lib.FLAG_W_INT8_FUSED if fused else 0))
    plain = lib.make_desc(m, n, b, k, N, code, flags=lib.FLAG_RECOMPUTE_B)
    es = 4 if dtype == "f32" else 2
    in_kernel = fused and dtype == "bf16" and m % 256 == 0 and n % 256 == 0 and N % 256 == 0
    assert bool(lib.poetx_linear_path(desc) & lib.PATH_W_INT8_IN_KERNEL) == in_kernel
    if in_kernel:   # the dense kernels convert the codes themselves: no room for a high-precision weight
        assert lib.poetx_linear_workspace_bytes(desc) == lib.poetx_linear_workspace_bytes(plain)
    else:           # dequantised copy in the workspace
        assert lib.poetx_linear_workspace_bytes(desc) >= lib.poetx_linear_workspace_bytes(plain)
        assert lib.poetx_linear_workspace_bytes(desc) >= (m + n) * N * es + n * m * es
    ws = ws_tensor(lib.poetx_linear_workspace_bytes(desc))
    Z = torch.empty((n, N), dtype=dt, device="cuda")
    B = torch.empty((n, N), dtype=dt, device="cuda")
    dX, dA = torch.empty((m, N), dtype=dt, device="cuda"), torch.empty((m, N), dtype=dt, device="cuda")
    dR, dP = torch.full_like(th_R, float("nan")), torch.full_like(th_P, float("nan"))
    lib.poetx_linear_fwd(desc, X, Wq, pi_R, pi_P, blk_R, blk_P, Z, None, ws)
    lib.poetx_linear_bwd_input(desc, dZ, Wq, pi_R, pi_P, blk_R, blk_P, dX, dA, ws)
    lib.poetx_linear_recompute_b(desc, X, Wq, pi_R, blk_R, B, ws)
    lib.poetx_linear_bwd_skew(desc, X, dZ, B, dA, pi_R, pi_P, th_R, th_P, dR, dP, False, ws)
    torch.cuda.synchronize()
    res = {"G_R": G_R, "G_P": G_P, "Z": to_np(Z), "B": to_np(B), "dX": to_np(dX), "dtheta_R": to_np(dR),
           "dtheta_P": to_np(dP)}
    check_layer(res, ref, data["pi_P"], dtype)
    # The same layer on the explicitly dequantised weight (stand-alone dequantiser + plain memory-saving
    # variant): the in-kernel conversion rounds the same way, so every output is the same bit for bit.
    Wd = torch.empty((n, m), dtype=dt, device="cuda")
    lib.poetx_weight_dequantize_q8(Wq, Wd)
    wsp = ws_tensor(lib.poetx_linear_workspace_bytes(plain))
    Z2, B2 = torch.empty_like(Z), torch.empty_like(B)
    dX2, dA2 = torch.empty_like(dX), torch.empty_like(dA)
    lib.poetx_linear_fwd(plain, X, Wd, pi_R, pi_P, blk_R, blk_P, Z2, None, wsp)
    lib.poetx_linear_bwd_input(plain, dZ, Wd, pi_R, pi_P, blk_R, blk_P, dX2, dA2, wsp)
    lib.poetx_linear_recompute_b(plain, X, Wd, pi_R, blk_R, B2, wsp)
    torch.cuda.synchronize()
    assert torch.equal(Z2, Z) and torch.equal(B2, B) and torch.equal(dX2, dX) and torch.equal(dA2, dA)
    # one-call backward on the quantised weight
    dX3 = torch.full_like(dX, float("nan"))
    dR3, dP3 = torch.full_like(th_R, float("nan")), torch.full_like(th_P, float("nan"))
    lib.poetx_linear_bwd(desc, X, dZ, B, Wq, pi_R, pi_P, blk_R, blk_P, th_R, th_P, dX3, dR3, dP3, False, ws)
    torch.cuda.synchronize()
    assert torch.equal(dX3, dX)
    assert rel_err(to_np(dR3), ref["dtheta_R"]) <= TOL[dtype] and rel_err(to_np(dP3), ref["dtheta_P"]) <= TOL[dtype]
    # ... and with B recomputed inside the call (one dequantisation serves both of its products)
    dX4 = torch.full_like(dX, float("nan"))
    dR4, dP4 = torch.full_like(th_R, float("nan")), torch.full_like(th_P, float("nan"))
    ws.fill_(0xFF)
    lib.poetx_linear_bwd(desc, X, dZ, None, Wq, pi_R, pi_P, blk_R, blk_P, th_R, th_P, dX4, dR4, dP4, False, ws)
    torch.cuda.synchronize()
    assert torch.equal(dX4, dX3) and torch.equal(dR4, dR3) and torch.equal(dP4, dP3)


# ------------------------------------------------------------------ stream capture
def test_step_can_be_captured_in_a_graph(lib):
    """The library enqueues kernels only (no allocation, no memset, no synchronisation on the hot
    path), so a whole layer step can be stream-captured.  Every replay, with eager work and
    synchronisations in between, must reproduce the eager result bit for bit."""
    m, n, N, b, k = 256, 512, 256, 256, 3
    data = synth_layer(9900, m, n, N, b, k, "bf16", 0.005)
    eager = run_layer(data, "bf16")            # also warms every kernel up (function attributes are set on first use)
    dev = eager["dev"]
    desc, ws = dev["desc"], dev["ws"]
    nbR = m // b
    theta_all = torch.cat([dev["th_R"], dev["th_P"]]).contiguous()
    blk_all = torch.empty((nbR + n // b, 2, b, b), dtype=torch.bfloat16, device="cuda")
    cws = ws_tensor(lib.poetx_cnp_workspace_bytes(m + n, b))
    Z, B = torch.empty_like(dev["Z"]), torch.empty_like(dev["B"])
    dX, dA = torch.empty_like(dev["dX"]), torch.empty_like(dev["dA"])
    dR, dP = torch.empty_like(dev["th_R"]), torch.empty_like(dev["th_P"])

    def step():
        lib.poetx_cnp_build(theta_all, m + n, b, k, lib.CNP_BF16, E_bf16=blk_all, ws=cws)
        bR, bP = blk_all[:nbR], blk_all[nbR:]
        lib.poetx_linear_fwd(desc, dev["X"], dev["W"], dev["pi_R"], dev["pi_P"], bR, bP, Z, B, ws)
        lib.poetx_linear_bwd_input(desc, dev["dZ"], dev["W"], dev["pi_R"], dev["pi_P"], bR, bP, dX, dA, ws)
        lib.poetx_linear_bwd_skew(desc, dev["X"], dev["dZ"], B, dA, dev["pi_R"], dev["pi_P"], dev["th_R"], dev["th_P"],
                                  dR, dP, False, ws)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    want = [t.clone() for t in (Z, B, dX, dR, dP)]
    assert torch.equal(Z, dev["Z"]) and torch.equal(dX, dev["dX"])     # one batched block build == two separate ones
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        for t in (Z, B, dX, dR, dP):
            t.fill_(float("nan"))                                    # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref_t in zip((Z, B, dX, dR, dP), want):
            assert torch.equal(got, ref_t), f"replay {rep} differs from the eager step"


# ------------------------------------------------------------------ optional outputs / accumulation on the on-chip path
def test_on_chip_build_optional_outputs(lib):
    """b = 256, matrix-core series: G only, E only and both must give the same values."""
    d, b, k = 512, 256, 4
    theta = draw_theta(RNG(4321), d, b, 0.005)
    th = to_dev(theta, torch.float32)
    ws = ws_tensor(lib.poetx_cnp_workspace_bytes(d, b))
    G1 = torch.empty((2, b, b), dtype=torch.float32, device="cuda")
    G2 = torch.empty_like(G1)
    E1 = torch.empty((2, 2, b, b), dtype=torch.bfloat16, device="cuda")
    E2 = torch.empty_like(E1)
    lib.poetx_cnp_build(th, d, b, k, lib.CNP_BF16, G1, E1, ws)
    lib.poetx_cnp_build(th, d, b, k, lib.CNP_BF16, G2, None, ws)
    lib.poetx_cnp_build(th, d, b, k, lib.CNP_BF16, None, E2, ws)
    torch.cuda.synchronize()
    assert torch.equal(G1, G2) and torch.equal(E1, E2)
    ref = orc.cnp(orc.skew_from_packed(theta, b, d), k)
    assert rel_err(to_np(G1) - np.eye(b), ref - np.eye(b)) <= 2e-2


def test_bwd_skew_accumulates_on_the_batched_path(lib):
    """accumulate != 0 adds to dtheta (both sides go through one batched series backward at b = 256)."""
    m, n, N, b, k = 512, 256, 256, 256, 3
    data = synth_layer(9950, m, n, N, b, k, "bf16", 0.005)
    res = run_layer(data, "bf16")
    dev = res["dev"]
    dR = torch.full_like(dev["th_R"], 0.25)
    dP = torch.full_like(dev["th_P"], -0.5)
    lib.poetx_linear_bwd_skew(dev["desc"], dev["X"], dev["dZ"], dev["B"], dev["dA"], dev["pi_R"], dev["pi_P"],
                              dev["th_R"], dev["th_P"], dR, dP, True, dev["ws"])
    torch.cuda.synchronize()
    assert np.array_equal(to_np(dR), (torch.from_numpy(res["dtheta_R"]).float() + 0.25).double().numpy())
    assert np.array_equal(to_np(dP), (torch.from_numpy(res["dtheta_P"]).float() - 0.5).double().numpy())


# ------------------------------------------------------------------ deferred series backward
@pytest.mark.parametrize("m,n,N,b,k,dtype", [(512, 768, 512, 256, 5, "bf16"), (1376, 512, 256, 64, 4, "bf16"),
                                             (256, 256, 128, 32, 3, "f32"), (1024, 512, 256, 512, 3, "bf16")])
def test_block_grads_and_cnp_bwd(lib, m, n, N, b, k, dtype):
    """POETX_FLAG_BLOCK_GRADS: both backward entry points stop after the block gradients (checked against
    the oracle's dG), and poetx_cnp_bwd finishes the job -- for both sides in one call when b divides
    both dimensions, side by side otherwise."""
    data = synth_layer(9900 + m + n + b, m, n, N, b, k, dtype, 0.01 if b < 256 else 0.005)
    res = run_layer(data, dtype)
    dev = res["dev"]
    G_R = orc.cnp(orc.skew_from_packed(data["theta_R"], b, m), k)
    G_P = orc.cnp(orc.skew_from_packed(data["theta_P"], b, n), k)
    f = orc.linear_fwd(data["X"], data["W"], data["pi_R"], data["pi_P"], G_R, G_P)
    g = orc.linear_bwd(data["dZ"], f, data["pi_R"], data["pi_P"], G_R, G_P)
    ref = orc.linear_fwd_bwd_from_theta(data["X"], data["dZ"], data["W"], data["pi_R"], data["pi_P"],
                                        data["theta_R"], data["theta_P"], b, k)
    code = lib.F32 if dtype == "f32" else lib.BF16
    desc = lib.make_desc(m, n, b, k, N, code, flags=lib.FLAG_BLOCK_GRADS)
    nbR, nbP = orc.n_blocks(m, b), orc.n_blocks(n, b)
    tol = TOL[dtype]
    prec = lib.CNP_FP32 if dtype == "f32" else lib.CNP_BF16
    for entry in ("bwd", "bwd_skew"):
        dG = torch.full((nbR + nbP, b, b), float("nan"), dtype=torch.float32, device="cuda")
        dG_R, dG_P = dG[:nbR], dG[nbR:]
        if entry == "bwd":
            dX = torch.empty_like(dev["dX"])
            lib.poetx_linear_bwd(desc, dev["X"], dev["dZ"], dev["B"], dev["W"], dev["pi_R"], dev["pi_P"], dev["blk_R"],
                                 dev["blk_P"], dev["th_R"], dev["th_P"], dX, dG_R, dG_P, False, dev["ws"])
            torch.cuda.synchronize()
            assert rel_err(to_np(dX), ref["dX"]) <= tol
        else:
            lib.poetx_linear_bwd_skew(desc, dev["X"], dev["dZ"], dev["B"], dev["dA"], dev["pi_R"], dev["pi_P"],
                                      dev["th_R"], dev["th_P"], dG_R, dG_P, False, dev["ws"])
            torch.cuda.synchronize()
        # the oracle's blocks are exact for the tail's live part; dead rows / columns of a ragged tail hold
        # whatever the padded reduction gives and are ignored by the series backward
        for side, got, want, d in (("R", to_np(dG_R), g["dG_R"], m), ("P", to_np(dG_P), g["dG_P"], n)):
            r = orc.tail_side(d, b)
            got, want = got.copy(), want.copy()
            got[-1, r:, :] = 0; got[-1, :, r:] = 0; want[-1, r:, :] = 0; want[-1, :, r:] = 0
            assert rel_err(got, want) <= tol, (entry, side)
            assert row_rel_err(got, want) <= tol, (entry, side)
        # series backward of the two sides
        if m % b == 0 and n % b == 0:   # one call for all blocks
            th = torch.cat([dev["th_R"], dev["th_P"]], 0).contiguous()
            dth = torch.full_like(th, float("nan"))
            ws = ws_tensor(lib.poetx_cnp_bwd_workspace_bytes(m + n, b, k))
            lib.poetx_cnp_bwd(th, dG, m + n, b, k, prec, dth, False, ws)
            torch.cuda.synchronize()
            got_R, got_P = to_np(dth[:nbR]), to_np(dth[nbR:])
        else:
            outs = []
            for th, dGs, d in ((dev["th_R"], dG_R, m), (dev["th_P"], dG_P, n)):
                dth = torch.full_like(th, float("nan"))
                ws = ws_tensor(lib.poetx_cnp_bwd_workspace_bytes(d, b, k))
                lib.poetx_cnp_bwd(th, dGs.contiguous(), d, b, k, prec, dth, False, ws)
                torch.cuda.synchronize()
                outs.append(to_np(dth))
            got_R, got_P = outs
        assert rel_err(got_R, ref["dtheta_R"]) <= tol and rel_err(got_P, ref["dtheta_P"]) <= tol, entry
        assert row_rel_err(got_R, ref["dtheta_R"]) <= tol and row_rel_err(got_P, ref["dtheta_P"]) <= tol, entry


# ------------------------------------------------------------------ token-major activations
@pytest.mark.parametrize("m,n,N,b,k,dtype", [(256, 256, 512, 32, 4, "f32"), (512, 1376, 1000, 64, 4, "bf16"),
                                             (768, 512, 1280, 256, 5, "bf16"), (96, 40, 77, 8, 2, "f32")])
def test_token_major_layout(lib, m, n, N, b, k, dtype):
    """layout = POETX_TOKEN_MAJOR: X, Z, dZ, dX are [N][d].  The re-laying passes are exact, so every
    output must be the transposed feature-major output bit for bit (which run_layer has already
    produced and which is checked against the oracle here as well), through both backward routes."""
    data = synth_layer(9950 + m + n + N, m, n, N, b, k, dtype, 0.01 if b < 256 else 0.005)
    ref = orc.linear_fwd_bwd_from_theta(data["X"], data["dZ"], data["W"], data["pi_R"], data["pi_P"],
                                        data["theta_R"], data["theta_P"], b, k)
    res = run_layer(data, dtype)
    check_layer(res, ref, data["pi_P"], dtype)
    dev = res["dev"]
    code = lib.F32 if dtype == "f32" else lib.BF16
    desc = lib.make_desc(m, n, b, k, N, code, layout=lib.TOKEN_MAJOR)
    fm = lib.make_desc(m, n, b, k, N, code)
    es = 4 if dtype == "f32" else 2
    assert lib.poetx_linear_workspace_bytes(desc) >= lib.poetx_linear_workspace_bytes(fm) + (2 * m + n) * N * es
    ws = ws_tensor(lib.poetx_linear_workspace_bytes(desc))
    Xt, dZt = dev["X"].t().contiguous(), dev["dZ"].t().contiguous()          # [N][m], [N][n]
    Zt = torch.full((N, n), float("nan"), dtype=Xt.dtype, device="cuda")
    B = torch.empty_like(dev["B"])
    lib.poetx_linear_fwd(desc, Xt, dev["W"], dev["pi_R"], dev["pi_P"], dev["blk_R"], dev["blk_P"], Zt, B, ws)
    torch.cuda.synchronize()
    assert torch.equal(Zt, dev["Z"].t()) and torch.equal(B, dev["B"])
    assert rel_err(to_np(Zt).T, ref["Z"]) <= TOL[dtype]
    # backward, two calls
    dXt = torch.full((N, m), float("nan"), dtype=Xt.dtype, device="cuda")
    dA = torch.empty_like(dev["dA"])
    dR, dP = torch.full_like(dev["th_R"], float("nan")), torch.full_like(dev["th_P"], float("nan"))
    lib.poetx_linear_bwd_input(desc, dZt, dev["W"], dev["pi_R"], dev["pi_P"], dev["blk_R"], dev["blk_P"], dXt, dA, ws)
    lib.poetx_linear_bwd_skew(desc, Xt, dZt, B, dA, dev["pi_R"], dev["pi_P"], dev["th_R"], dev["th_P"], dR, dP, False, ws)
    torch.cuda.synchronize()
    assert torch.equal(dXt, dev["dX"].t()) and torch.equal(dA, dev["dA"])
    assert np.array_equal(to_np(dR), res["dtheta_R"]) and np.array_equal(to_np(dP), res["dtheta_P"])
    # backward, one call
    dXt1 = torch.full((N, m), float("nan"), dtype=Xt.dtype, device="cuda")
    dR1, dP1 = torch.full_like(dev["th_R"], float("nan")), torch.full_like(dev["th_P"], float("nan"))
    lib.poetx_linear_bwd(desc, Xt, dZt, B, dev["W"], dev["pi_R"], dev["pi_P"], dev["blk_R"], dev["blk_P"],
                         dev["th_R"], dev["th_P"], dXt1, dR1, dP1, False, ws)
    torch.cuda.synchronize()
    assert np.array_equal(to_np(dXt1).T, res["one_call"]["dX"])
    assert np.array_equal(to_np(dR1), res["one_call"]["dtheta_R"]) and np.array_equal(to_np(dP1), res["one_call"]["dtheta_P"])
    # memory-saving variant: recompute B from the token-major X
    mem = lib.make_desc(m, n, b, k, N, code, flags=lib.FLAG_RECOMPUTE_B, layout=lib.TOKEN_MAJOR)
    wsm = ws_tensor(lib.poetx_linear_workspace_bytes(mem))
    B2 = torch.full_like(B, float("nan"))
    lib.poetx_linear_recompute_b(mem, Xt, dev["W"], dev["pi_R"], dev["blk_R"], B2, wsm)
    torch.cuda.synchronize()
    assert torch.equal(B2, dev["B"])
    # ... and the one-call backward that recomputes B itself, from token-major X and dZ
    dXt2 = torch.full((N, m), float("nan"), dtype=Xt.dtype, device="cuda")
    dR2, dP2 = torch.full_like(dev["th_R"], float("nan")), torch.full_like(dev["th_P"], float("nan"))
    lib.poetx_linear_bwd(mem, Xt, dZt, None, dev["W"], dev["pi_R"], dev["pi_P"], dev["blk_R"], dev["blk_P"],
                         dev["th_R"], dev["th_P"], dXt2, dR2, dP2, False, wsm)
    torch.cuda.synchronize()
    assert torch.equal(dXt2, dXt1) and torch.equal(dR2, dR1) and torch.equal(dP2, dP1)
    # a layout code that does not exist is refused on the host
    assert lib.poetx_linear_workspace_bytes(lib.make_desc(m, n, b, k, N, code, layout=2)) == 0
