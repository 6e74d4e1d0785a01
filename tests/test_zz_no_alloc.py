"""The entry point that allocates nothing (poetx_cnp_build_static) against the entry point it
is a variant of (poetx_cnp_build), through the raw C ABI: two calls in a row on the library's
own static scratch, the second with a smaller input, every output compared bit for bit (the two
run the same kernels); the first call is also checked against the fp64 oracle."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2603_05500_amd as px
from oracle import poetx_oracle as orc
from tests.harness import TOL, rel_err, to_np

pytestmark = pytest.mark.gpu


def _run_pair(clib, d, b, k, precision, seed):
    nb = -(-d // b)
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    theta = (torch.randn((nb, b * (b - 1) // 2), generator=g) * 0.005).cuda()
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    out = {}
    for name in ("ws", "static"):
        G = torch.full((nb, b, b), float("nan"), dtype=torch.float32, device="cuda")
        E = torch.full((nb, 2, b, b), float("nan"), dtype=torch.bfloat16, device="cuda")
        if name == "ws":
            nbytes = clib.poetx_cnp_workspace_bytes(d, b)
            ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
            rc = clib.poetx_cnp_build(ctypes.c_void_p(theta.data_ptr()), d, b, k, precision,
                                      ctypes.c_void_p(G.data_ptr()), ctypes.c_void_p(E.data_ptr()),
                                      ctypes.c_void_p(ws.data_ptr()), nbytes, st)
        else:
            rc = clib.poetx_cnp_build_static(ctypes.c_void_p(theta.data_ptr()), d, b, k, precision,
                                             ctypes.c_void_p(G.data_ptr()), ctypes.c_void_p(E.data_ptr()), st)
        assert rc == 0, (name, rc)
        torch.cuda.synchronize()
        out[name] = (G, E)
    assert torch.equal(out["ws"][0], out["static"][0]), "G differs between the two entry points"
    assert torch.equal(out["ws"][1].view(torch.int16), out["static"][1].view(torch.int16)), "E differs"
    return theta, out["static"][0]


@pytest.mark.parametrize("b,precision", [(256, px.CNP_BF16), (512, px.CNP_BF16), (64, px.CNP_FP32)])
def test_static_scratch_matches_workspace_variant(lib, b, precision):
    clib = px.load_library()
    k = 5
    d1, d2 = 8 * b, 3 * b - (b // 2 if b == 64 else 0)     # second call smaller (ragged tail on the plain path)
    theta, G = _run_pair(clib, d1, b, k, precision, seed=11)
    ref = orc.cnp(orc.skew_from_packed(to_np(theta), b, d1), k)
    tol = TOL["bf16"] if precision == px.CNP_BF16 else TOL["f32"]
    eye = np.eye(b)
    assert rel_err(to_np(G) - eye, ref - eye) <= tol
    _run_pair(clib, d2, b, k, precision, seed=12)


def test_static_scratch_rejects_oversize(lib):
    clib = px.load_library()
    fake = ctypes.c_void_p(0x1000)   # never dereferenced: the size check fails first
    # 65 blocks of 256 x 256 exceed the 2^22-element static scratch
    assert clib.poetx_cnp_build_static(fake, 65 * 256, 256, 3, px.CNP_BF16, fake, None, None) == 4
    assert clib.poetx_cnp_build_static(None, 512, 256, 3, px.CNP_BF16, fake, None, None) == 1
