#!/usr/bin/env python3
"""Benchmark of the POET-X linear hot path on one MI355X.

One "step" = one pass of the whole hot path over one Llama-8B-shaped decoder
layer: for each of the seven projections, Cayley-Neumann build of both block
sets, forward, backward to the input and backward to the packed skew
parameters (the `fast` variant, which keeps B).  All inputs are synthetic,
seeded and resident in HBM before the timed region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0
# L2<->fabric bytes per dense launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, scaled by
# what the same counters read for a 1 GiB copy (2.0 and 1.0); see profiles/llama8b_b256_layer_counters.md.
DENSE_TRAFFIC_BYTES_PER_LAUNCH = {"llama8b-b256": 1.81e9}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama8b-b256",
                    help="llama8b-b256 (default, the metric's configuration), llama8b-b512, llama3b (fresh "
                         "permutations every step), llama1b; or `micro`: the shapes of the paper's kernel tables "
                         "(permutation, block-diagonal product, Cayley-Neumann build) on the library's entry points; "
                         "or `vendor-gemm`: torch.matmul on the layer's dense shapes, as a reference for the dense kernel")
    ap.add_argument("--xq-fused", action="store_true",
                    help="with --variant xq: the dense products convert the INT8 codes themselves (no dequantised copy in the workspace)")
    ap.add_argument("--variant", default="fast", choices=["fast", "mem", "xq"],
                    help="fast keeps B from the forward pass (the measured metric); mem recomputes it in backward; "
                         "xq is mem on an INT8 base weight that every dense product dequantises first")
    ap.add_argument("--layout", default="feature", choices=["feature", "token"],
                    help="feature: X, Z, dZ, dX are [d][N] (native, the measured metric); token: [N][d], re-laid by "
                         "the library on the way in and out")
    ap.add_argument("--per-projection-series", action="store_true",
                    help="build the blocks and run the series backward once per projection instead of once per "
                         "layer step for all seven projections together")
    ap.add_argument("--two-call-backward", action="store_true",
                    help="run the backward pass as poetx_linear_bwd_input + poetx_linear_bwd_skew instead of the "
                         "single poetx_linear_bwd call")
    ap.add_argument("--no-b512", action="store_true", help="skip the short llama8b-b512 pass that the default run appends")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-tokens", type=int, default=128, help="tokens in the oracle's timed sample")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run one plain 1 GiB device-to-device copy first (a known-size kernel for scaling "
                         "FETCH_SIZE / WRITE_SIZE counters under rocprofv3 --pmc)")
    return ap.parse_args()


def layer_flops(cfg):
    """Algorithmic flops of one step: two dense products, six block products per side,
    and the series (k products forward, 2k backward per block)."""
    N, b, k = cfg.n_tokens, cfg.block, cfg.neumann_k
    dense = block = cnp = 0.0
    for p in cfg.projections:
        m, n = p.d_in, p.d_out
        dense += 4.0 * N * m * n
        block += 6.0 * N * (m + n) * b
        nb = -(-m // b) + -(-n // b)
        cnp += nb * (k + 2 * k) * 2.0 * b ** 3
    return dense, block, cnp


def make_inputs(cfg, torch):
    """Seeded device-side draws with the distributions of the configuration."""
    g = torch.Generator(device="cuda")
    g.manual_seed(20260305 + 1000 * cfg.index)
    dt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    N, b = cfg.n_tokens, cfg.block
    projs = []
    for p in cfg.projections:
        m, n = p.d_in, p.d_out
        d = {"m": m, "n": n, "name": p.name}
        d["X"] = torch.randn((m, N), generator=g, device="cuda", dtype=torch.float32).to(dt)
        d["dZ"] = torch.randn((n, N), generator=g, device="cuda", dtype=torch.float32).to(dt)
        d["W"] = (torch.randn((n, m), generator=g, device="cuda", dtype=torch.float32) * cfg.sigma_w).to(dt)
        # The packed parameters (and the blocks built from them) of the two sides of a projection live
        # in one buffer, R side first, so that one poetx_cnp_build call covers both sides when b
        # divides both dimensions (the series of a block does not depend on which side it belongs to).
        nbs = {"R": -(-m // b), "P": -(-n // b)}
        d["theta_all"] = torch.randn((nbs["R"] + nbs["P"], b * (b - 1) // 2), generator=g, device="cuda",
                                     dtype=torch.float32) * cfg.sigma_theta
        bshape = (nbs["R"] + nbs["P"], 2, b, b) if cfg.dtype == "bf16" else (nbs["R"] + nbs["P"], b, b)
        d["blk_all"] = torch.empty(bshape, device="cuda", dtype=dt)   # bf16: (G - I, its transpose)
        d["one_build"] = m % b == 0 and n % b == 0
        for side, dim in (("R", m), ("P", n)):
            nb = nbs[side]
            lo = 0 if side == "R" else nbs["R"]
            d["theta_" + side] = d["theta_all"][lo:lo + nb]
            # fresh permutations per step (Sec. 3, merge-and-resample): a pool of index vectors made
            # before the timed region, walked round robin; permutations are inputs of every call, so a new
            # one costs the path nothing
            npool = 4 if cfg.fresh_perms else 1
            d["pool_" + side] = [torch.randperm(dim, generator=g, device="cuda").to(torch.int32) for _ in range(npool)]
            d["pi_" + side] = d["pool_" + side][0]
            d["blk_" + side] = d["blk_all"][lo:lo + nb]
            d["dtheta_" + side] = torch.empty_like(d["theta_" + side])
        projs.append(d)
    return projs


def cpu_baseline(cfg, n_tok):
    """The fp64 oracle as it stands, timed on the host cores for a token sample of the
    same layer; token-proportional and token-independent parts are timed apart and
    recombined for the full token count."""
    import numpy as np
    from oracle import poetx_oracle as orc
    from workloads import draw_projection
    try:
        from threadpoolctl import threadpool_info
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    t_tok = t_cnp = 0.0
    for pi_, p in enumerate(cfg.projections):
        data = draw_projection(cfg, pi_, want=("W", "theta_R", "theta_P", "pi_R", "pi_P"))
        rng = np.random.Generator(np.random.PCG64(7 + pi_))
        X = rng.standard_normal((p.d_in, n_tok))
        dZ = rng.standard_normal((p.d_out, n_tok))
        b, k = cfg.block, cfg.neumann_k
        t0 = time.perf_counter()
        Q_R = orc.skew_from_packed(data["theta_R"], b, p.d_in)
        Q_P = orc.skew_from_packed(data["theta_P"], b, p.d_out)
        G_R, G_P = orc.cnp(Q_R, k), orc.cnp(Q_P, k)
        t1 = time.perf_counter()
        f = orc.linear_fwd(X, data["W"], data["pi_R"], data["pi_P"], G_R, G_P)
        g = orc.linear_bwd(dZ, f, data["pi_R"], data["pi_P"], G_R, G_P)
        t2 = time.perf_counter()
        orc.packed_from_skew_grad(orc.cnp_bwd(Q_R, g["dG_R"], k), b, p.d_in)
        orc.packed_from_skew_grad(orc.cnp_bwd(Q_P, g["dG_P"], k), b, p.d_out)
        t3 = time.perf_counter()
        t_cnp += (t1 - t0) + (t3 - t2)
        t_tok += t2 - t1
    full = t_cnp + t_tok * (cfg.n_tokens / n_tok)
    return {"value": cfg.n_tokens / full, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"all 7 projections of {cfg.name}, {n_tok} of {cfg.n_tokens} tokens in fp64 numpy; "
                      f"token-proportional part {t_tok:.2f}s scaled by {cfg.n_tokens // n_tok}, "
                      f"series build/backward {t_cnp:.2f}s counted once"}


def time_call(torch, fn, iters, warm=3):
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


def micro(args, torch, px):
    """The shapes of the paper's kernel tables on this library's entry points (bf16, b = 256 unless
    said): permutation + block-diagonal product fused (apply_left) over hidden sizes and over
    token counts, and the Cayley-Neumann build at k = 3 over block counts.  The paper does not
    state batch / sequence for its tables, so the token counts here are this build's choice."""
    g = torch.Generator(device="cuda")
    g.manual_seed(20260305)
    it = max(args.steps, 5)
    out = {"apply_vs_hidden": [], "apply_vs_tokens": [], "cnp_build_k3": [], "merge": []}
    b = 256

    def apply_case(d, N):
        # The calls rotate through enough input / output pairs that their combined footprint (>= 800 MB,
        # at least 3 pairs) is several times the 256 MB Infinity Cache: the figures are HBM figures.
        sets = max(3, -(-800_000_000 // (4 * d * N)))
        Vs = [torch.randn((d, N), generator=g, device="cuda").to(torch.bfloat16) for _ in range(sets)]
        Os = [torch.empty_like(Vs[0]) for _ in range(sets)]
        E = (torch.randn((d // b, 2, b, b), generator=g, device="cuda") * 0.01).to(torch.bfloat16)
        perm = torch.randperm(d, generator=g, device="cuda").to(torch.int32)
        turn = [0]

        def call():
            i = turn[0] % sets
            turn[0] += 1
            px.poetx_perm_blockdiag_apply_left(Vs[i], Os[i], perm, E, b, True)
        ms = time_call(torch, call, max(it, 2 * sets), warm=sets)
        return {"hidden": d, "tokens": N, "ms": ms, "GBs": 4.0 * d * N / ms / 1e6, "buffer_pairs": sets}

    for d in (2048, 4096, 8192, 16384):      # permutation table: hidden size sweep
        out["apply_vs_hidden"].append(apply_case(d, 8192))
    for N in (2048, 4096, 8192, 16384):      # block-diagonal table: sequence length sweep
        out["apply_vs_tokens"].append(apply_case(4096, N))
    for n, m in ((4096, 4096), (14336, 4096), (4096, 14336)):   # merge W <- P^T W R^T on the stored weight (every 400 steps)
        W = (torch.randn((n, m), generator=g, device="cuda") * 0.02).to(torch.bfloat16)
        T1, T2 = torch.empty_like(W), torch.empty_like(W)
        EP = (torch.randn((n // b, 2, b, b), generator=g, device="cuda") * 0.01).to(torch.bfloat16)
        ER = (torch.randn((m // b, 2, b, b), generator=g, device="cuda") * 0.01).to(torch.bfloat16)
        pP = torch.randperm(n, generator=g, device="cuda").to(torch.int32)
        pR = torch.randperm(m, generator=g, device="cuda").to(torch.int32)

        def merge():
            px.poetx_perm_blockdiag_apply_left(W, T1, pP, EP, b, True)
            px.poetx_perm_blockdiag_apply_right(T1, T2, pR, ER, b, True)
        wsm = torch.empty(px.poetx_merge_workspace_bytes(n, m, px.BF16), dtype=torch.uint8, device="cuda")
        out["merge"].append({"out": n, "in": m, "ms_apply_left_then_right": time_call(torch, merge, it),
                             "ms_merge_weight": time_call(torch, lambda: px.poetx_merge_weight(W, T2, pR, pP, ER, EP, b, wsm), it)})
    for bb in (256, 512):                    # Cayley-Neumann table: number of blocks sweep, k = 3
        for nb in (64, 128, 192, 256, 320):
            d = nb * bb
            theta = torch.randn((nb, bb * (bb - 1) // 2), generator=g, device="cuda") * 0.005
            E = torch.empty((nb, 2, bb, bb), device="cuda", dtype=torch.bfloat16)
            ws = torch.empty(px.poetx_cnp_workspace_bytes(d, bb), dtype=torch.uint8, device="cuda")
            ms = time_call(torch, lambda: px.poetx_cnp_build(theta, d, bb, 3, px.CNP_BF16, E_bf16=E, ws=ws), it)
            out["cnp_build_k3"].append({"block": bb, "blocks": nb, "ms": ms,
                                        "TFLOPs": nb * 3 * 2.0 * bb ** 3 / ms / 1e9})
            del theta, E, ws
    return out


def run_workload(args, torch, px, get_config):
    """One layer workload: warm-up, the timed steps, a second pass with stage events; returns the result line's dict."""
    cfg = get_config(args.workload)
    torch.cuda.set_device(0)
    code = px.BF16 if cfg.dtype == "bf16" else px.F32
    dt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    N, b, k = cfg.n_tokens, cfg.block, cfg.neumann_k
    projs = make_inputs(cfg, torch)
    # The series of a block does not depend on the projection it belongs to: when b divides every
    # dimension, the packed parameters, blocks, block gradients and parameter gradients of all seven
    # projections live end to end in layer-wide buffers, so that ONE poetx_cnp_build at the start of a
    # step and ONE poetx_cnp_bwd at its end serve the whole layer (320 chains fill the GPU; the 8 to 72
    # of one projection do not).
    layer_series = (not args.per_projection_series and cfg.dtype == "bf16" and all(p["one_build"] for p in projs)
                    and not args.two_call_backward)
    if layer_series:
        nbt = sum(p["theta_all"].shape[0] for p in projs)
        theta_layer = torch.cat([p["theta_all"] for p in projs], 0).contiguous()
        blk_layer = torch.empty((nbt, 2, b, b), device="cuda", dtype=torch.bfloat16)
        dG_layer = torch.empty((nbt, b, b), device="cuda", dtype=torch.float32)
        dtheta_layer = torch.empty_like(theta_layer)
        lo = 0
        for p in projs:
            nR, nP = p["theta_R"].shape[0], p["theta_P"].shape[0]
            p["theta_all"] = theta_layer[lo:lo + nR + nP]
            p["theta_R"], p["theta_P"] = theta_layer[lo:lo + nR], theta_layer[lo + nR:lo + nR + nP]
            p["blk_R"], p["blk_P"] = blk_layer[lo:lo + nR], blk_layer[lo + nR:lo + nR + nP]
            p["dG_R"], p["dG_P"] = dG_layer[lo:lo + nR], dG_layer[lo + nR:lo + nR + nP]
            p["dtheta_R"], p["dtheta_P"] = dtheta_layer[lo:lo + nR], dtheta_layer[lo + nR:lo + nR + nP]
            lo += nR + nP
        d_layer = nbt * b
    nmax = max(p["n"] for p in projs)
    mmax = max(p["m"] for p in projs)
    Z = torch.empty((nmax, N), device="cuda", dtype=dt)
    B = torch.empty((nmax, N), device="cuda", dtype=dt)
    dX = torch.empty((mmax, N), device="cuda", dtype=dt)
    dA = torch.empty((mmax, N), device="cuda", dtype=dt)
    ws_bytes = cnp_bytes = 0
    for p in projs:
        flags = {"fast": 0, "mem": px.FLAG_RECOMPUTE_B, "xq": px.FLAG_RECOMPUTE_B | px.FLAG_W_INT8}[args.variant]
        if args.xq_fused and args.variant == "xq":
            flags |= px.FLAG_W_INT8_FUSED
        if layer_series:
            flags |= px.FLAG_BLOCK_GRADS
        p["desc"] = px.make_desc(p["m"], p["n"], b, k, N, code, flags=flags,
                                 layout=px.TOKEN_MAJOR if args.layout == "token" else px.FEATURE_MAJOR)
        if args.layout == "token":
            p["X"], p["dZ"] = p["X"].t().contiguous(), p["dZ"].t().contiguous()
            p["Z_tm"] = torch.empty((N, p["n"]), device="cuda", dtype=dt)
            p["dX_tm"] = torch.empty((N, p["m"]), device="cuda", dtype=dt)
        if args.variant == "xq":   # only the 8-bit weight stays resident
            wq = torch.zeros(px.poetx_weight_q8_bytes(p["n"], p["m"]), dtype=torch.uint8, device="cuda")
            px.poetx_weight_quantize_q8(p["W"], wq)
            torch.cuda.synchronize()
            p["W"] = wq
        ws_bytes = max(ws_bytes, px.poetx_linear_workspace_bytes(p["desc"]))
        cnp_bytes = max(cnp_bytes, px.poetx_cnp_workspace_bytes(p["m"] + p["n"], b))
    if layer_series:
        cnp_bytes = max(px.poetx_cnp_workspace_bytes(d_layer, b), px.poetx_cnp_bwd_workspace_bytes(d_layer, b, k))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    cws = torch.empty(cnp_bytes, dtype=torch.uint8, device="cuda")
    prec = px.CNP_BF16 if code == px.BF16 else px.CNP_FP32

    step_no = [0]

    def step():
        if layer_series:
            px.poetx_cnp_build(theta_layer, d_layer, b, k, prec, ws=cws, E_bf16=blk_layer)
        for p in projs:
            m, n = p["m"], p["n"]
            p["pi_R"] = p["pool_R"][step_no[0] % len(p["pool_R"])]
            p["pi_P"] = p["pool_P"][step_no[0] % len(p["pool_P"])]
            if layer_series:
                pass
            elif p["one_build"]:
                kw = {"E_bf16": p["blk_all"]} if code == px.BF16 else {"G_f32": p["blk_all"]}
                px.poetx_cnp_build(p["theta_all"], m + n, b, k, prec, ws=cws, **kw)
            else:
                kw = {"E_bf16": p["blk_R"]} if code == px.BF16 else {"G_f32": p["blk_R"]}
                px.poetx_cnp_build(p["theta_R"], m, b, k, prec, ws=cws, **kw)
                kw = {"E_bf16": p["blk_P"]} if code == px.BF16 else {"G_f32": p["blk_P"]}
                px.poetx_cnp_build(p["theta_P"], n, b, k, prec, ws=cws, **kw)
            Zp = p["Z_tm"] if args.layout == "token" else Z[:n]
            dXp = p["dX_tm"] if args.layout == "token" else dX[:m]
            px.poetx_linear_fwd(p["desc"], p["X"], p["W"], p["pi_R"], p["pi_P"], p["blk_R"], p["blk_P"],
                                Zp, None if args.variant != "fast" else B[:n], ws)
            keep = args.variant == "fast"
            if not keep and args.two_call_backward:   # the one-call backward recomputes B itself
                px.poetx_linear_recompute_b(p["desc"], p["X"], p["W"], p["pi_R"], p["blk_R"], B[:n], ws)
            if args.two_call_backward:
                px.poetx_linear_bwd_input(p["desc"], p["dZ"], p["W"], p["pi_R"], p["pi_P"], p["blk_R"], p["blk_P"],
                                          dXp, dA[:m], ws)
                px.poetx_linear_bwd_skew(p["desc"], p["X"], p["dZ"], B[:n], dA[:m], p["pi_R"], p["pi_P"],
                                         p["theta_R"], p["theta_P"], p["dtheta_R"], p["dtheta_P"], False, ws)
            else:   # the whole backward pass in one call: each side's gradient is streamed once
                px.poetx_linear_bwd(p["desc"], p["X"], p["dZ"], B[:n] if keep else None, p["W"], p["pi_R"], p["pi_P"], p["blk_R"],
                                    p["blk_P"], p["theta_R"], p["theta_P"], dXp,
                                    p["dG_R"] if layer_series else p["dtheta_R"],
                                    p["dG_P"] if layer_series else p["dtheta_P"], False, ws)
        if layer_series:
            px.poetx_cnp_bwd(theta_layer, dG_layer, d_layer, b, k, prec, dtheta_layer, False, cws)
        step_no[0] += 1

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")   # 1 GiB
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # Timed region: exactly `steps` steps, nothing else on the stream.
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ms = e0.elapsed_time(e1) / args.steps
    # Second pass over the same steps with the library's stage events switched on: per-stage split and
    # the dense kernel's launch durations.  Kept apart from the timed region because the ~260 event
    # records per step cost a few per cent of it.
    px.poetx_profile_begin(1 << 16)
    e2, e3 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e2.record()
    for _ in range(args.steps):
        step()
    e3.record()
    torch.cuda.synchronize()
    ms_split = e2.elapsed_time(e3) / args.steps
    stages = px.poetx_profile_end()
    assert all(torch.isfinite(p["dtheta_R"]).all() and torch.isfinite(p["dtheta_P"]).all() for p in projs)

    dense_f, block_f, cnp_f = layer_flops(cfg)
    dense_ms, dense_cnt = stages["dense"]
    # the memory-saving variants run the forward product a second time in the backward pass (Sec. 3.5):
    # the stage rates count the work executed, mfma_peak_frac_layer the algorithmic work of a step
    recompute = args.variant != "fast"
    dense_exec = dense_f * (1.5 if recompute else 1.0)
    dense_tflops = dense_exec * args.steps / (dense_ms * 1e-3) / 1e12 if dense_ms > 0 else 0.0
    # HBM-bound block stages: algorithmic bytes = 2 s N d per apply (4 per projection side pair) ...
    es = 2 if cfg.dtype == "bf16" else 4
    unit = sum(es * N * (p["m"] + p["n"]) for p in projs)                 # one pass over an activation of each side
    ag_ms, ag_cnt = stages["apply_grad"]
    fused = ag_cnt > 0
    apply_bytes = (2 if fused else 4) * unit      # forward applies (+ backward applies when not fused): read + write
    if recompute:
        apply_bytes += 2 * sum(es * N * p["m"] for p in projs)            # A = R^T X once more
    bgrad_bytes = 2 * unit                        # separate block gradients: two reads per side
    ag_bytes = 3 * unit                           # one-pass backward block stage: read V, read U, write out
    apply_ms, _ = stages["apply"]
    bgrad_ms, _ = stages["blockgrad"]
    out = {
        "metric": "POET-X linear fwd+bwd tokens/sec at Llama-8B shapes; % MFMA peak",
        "value": N / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: one decoder layer = 7 POET-X linears "
                               f"({', '.join(f'{p.name} {p.d_out}x{p.d_in}' for p in cfg.projections)}), "
                               f"N={N} tokens, b={b}, k={k}, cnp_build + fwd + bwd (input and skew-parameter gradients), "
                               f"{args.variant} variant, {args.layout}-major activations"
                               + (", blocks built and series backward run once per step for the whole layer" if layer_series else "")
                               + (", a fresh permutation pair per projection every step" if cfg.fresh_perms else ""),
                   "tokens_per_step": N, "block": b, "neumann_k": k},
        "mfma_peak_frac_layer": (dense_f + block_f + cnp_f) / (ms * 1e-3) / (PEAK_BF16_TFLOPS * 1e12),
        "algorithmic_tflop_per_step": (dense_f + block_f + cnp_f) / 1e12,
        "wall_ms_per_step": wall_ms / args.steps,
        "ms_per_step_with_stage_events": ms_split,
        "stage_ms_per_step": {s: v[0] / args.steps for s, v in stages.items()},
        "stage_rates": {
            "dense_TFLOPs": dense_tflops,
            "apply_GBs": apply_bytes * args.steps / (apply_ms * 1e-3) / 1e9 if apply_ms > 0 else 0.0,
            "blockgrad_GBs": bgrad_bytes * args.steps / (bgrad_ms * 1e-3) / 1e9 if bgrad_ms > 0 else 0.0,
            "apply_grad_GBs": ag_bytes * args.steps / (ag_ms * 1e-3) / 1e9 if ag_ms > 0 else 0.0,
        },
        "roofline": {"bound": "mfma", "kernel": "dense bf16 product (B = W A, dA = W^T dB)",
                     "achieved": dense_tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": dense_tflops / PEAK_BF16_TFLOPS, "traffic": DENSE_TRAFFIC_BYTES_PER_LAUNCH.get(cfg.name),
                     "launches": int(dense_cnt), "avg_launch_ms": dense_ms / max(int(dense_cnt), 1)},
    }
    return out, cfg


def vendor_gemm(args, torch):
    """Reference points for the dense product: the vendor GEMM behind torch.matmul on the layer's three
    dense shapes, same value distributions, sustained (60 launches of warm-up).  NN is the layout this
    library's products have (activations feature major); NT has both operands contraction-major."""
    g = torch.Generator(device="cuda")
    g.manual_seed(20260305)
    rows = []
    for n, m, N in ((4096, 4096, 16384), (14336, 4096, 16384), (4096, 14336, 16384)):
        W = (torch.randn((n, m), generator=g, device="cuda") * 0.02).to(torch.bfloat16)
        A = torch.randn((m, N), generator=g, device="cuda").to(torch.bfloat16)
        At = A.t().contiguous()
        r = {"n": n, "m": m, "N": N}
        for name, fn in (("NN", lambda: torch.matmul(W, A)), ("NT", lambda: torch.matmul(W, At.t()))):
            ms = time_call(torch, fn, 40, warm=60)
            r[name + "_ms"], r[name + "_TFLOPs"] = ms, 2.0 * n * m * N / ms / 1e9
        rows.append(r)
        del W, A, At
    return rows


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU; run with --gpus 1 (no multi-GPU path exists)", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2603_05500_amd as px
    from workloads import get_config

    px.load_library()
    if args.workload == "vendor-gemm":
        torch.cuda.set_device(0)
        print(json.dumps({"metric": "vendor GEMM (torch.matmul) on the dense shapes of the llama8b layer", "unit": "TFLOP/s",
                          "n_gpus": 1, "dtype": "bf16", "data": "synthetic",
                          "config": {"workload": "vendor-gemm"}, "vendor_gemm": vendor_gemm(args, torch)}))
        return
    if args.workload == "micro":
        torch.cuda.set_device(0)
        res = micro(args, torch, px)
        print(json.dumps({"metric": "POET-X kernel microbenchmarks at the shapes of the paper's kernel tables",
                          "unit": "ms", "n_gpus": 1, "dtype": "bf16", "data": "synthetic",
                          "config": {"workload": "micro: fused permutation + block-diagonal apply (b=256) over hidden "
                                                 "size and token count; Cayley-Neumann build k=3 over block count"},
                          "micro": res}))
        return
    out, cfg = run_workload(args, torch, px, get_config)
    if args.workload == "llama8b-b256" and args.variant == "fast" and not args.no_b512:
        # config 5 names both block sizes: a short pass of the b = 512 variant rides along under its own key
        import copy
        import gc
        gc.collect()
        torch.cuda.empty_cache()
        a2 = copy.copy(args)
        a2.workload, a2.steps, a2.warmup = "llama8b-b512", max(3, args.steps // 3), 1
        o2, _ = run_workload(a2, torch, px, get_config)
        out["also"] = {"llama8b-b512": {k2: o2[k2] for k2 in ("value", "unit", "ms_per_step", "steps", "warmup",
                                                              "mfma_peak_frac_layer", "stage_ms_per_step", "stage_rates")}}
        out["also"]["llama8b-b512"]["workload"] = o2["config"]["workload"]
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, args.cpu_tokens)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
