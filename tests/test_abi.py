"""CPU-side checks of the C ABI: the library loads, exports what the header
declares, and rejects bad arguments on the host before touching a device."""
import ctypes
import os
import re

import pytest

import paper_2603_05500_amd as px

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def clib():
    if not os.path.exists(px.LIB_PATH):
        from paper_2603_05500_amd import build
        build.build()
    return px.load_library()


def header_symbols():
    text = open(os.path.join(ROOT, "include", "poetx.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(poetx_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_exported(clib):
    syms = header_symbols()
    assert len(syms) >= 12
    for s in syms:
        assert hasattr(clib, s), f"{s} declared in poetx.h but not exported"
    assert set(px.EXPORTS) == set(syms)


def test_status_strings(clib):
    assert px.status_string(0) == "ok"
    for s in range(1, 7):
        assert px.status_string(s) not in ("ok", "unknown status")
    assert px.status_string(99) == "unknown status"
    assert clib.poetx_version() >= 100


def test_workspace_queries(clib):
    assert px.poetx_cnp_workspace_bytes(256, 32) >= 2 * 8 * 32 * 32 * 4
    assert px.poetx_cnp_workspace_bytes(0, 32) == 0
    d = px.make_desc(256, 256, 32, 4, 512, px.F32)
    assert px.poetx_linear_workspace_bytes(d) >= 256 * 512 * 4
    bad = px.make_desc(256, 256, 32, 0, 512, px.F32)  # k < 1
    assert px.poetx_linear_workspace_bytes(bad) == 0


def test_host_argument_checks(clib):
    """Null pointers and bad sizes are refused on the host (no device needed)."""
    fake = ctypes.c_void_p(0x1000)  # never dereferenced: checks fail first
    assert clib.poetx_cnp_build(None, 64, 32, 3, 0, fake, None, fake, 1 << 20, None) == 1
    assert clib.poetx_cnp_build(fake, 64, 32, 0, 0, fake, None, fake, 1 << 20, None) == 1   # k < 1
    assert clib.poetx_cnp_build(fake, 16, 32, 3, 0, fake, None, fake, 1 << 20, None) == 2   # b > d
    assert clib.poetx_cnp_build(fake, 64, 32, 3, 0, fake, None, fake, 16, None) == 5        # workspace
    assert clib.poetx_cnp_build(fake, 64, 32, 3, 7, fake, None, fake, 1 << 20, None) == 1   # precision
    assert clib.poetx_perm_blockdiag_apply_left(fake, fake, 64, 8, 8, fake, fake, 32, 0, 0, None) == 1  # alias
    assert clib.poetx_perm_blockdiag_apply_left(fake, ctypes.c_void_p(0x100000), 64, 8, 4, fake, fake, 32, 0, 0,
                                                None) == 2  # ld < cols
    assert clib.poetx_perm_blockdiag_apply_right(None, fake, 8, 64, 64, fake, fake, 32, 0, 0, None) == 1
    d = px.make_desc(256, 256, 32, 4, 512, px.F32)
    args = [fake] * 9
    assert clib.poetx_linear_fwd(ctypes.byref(d), *args, 0, None) == 5
    assert clib.poetx_linear_fwd(None, *args, 1 << 30, None) == 1
    d2 = px.make_desc(256, 256, 32, 4, 512, 9)
    assert clib.poetx_linear_bwd_input(ctypes.byref(d2), *args, 1 << 30, None) == 1
    d3 = px.make_desc(256, 16, 32, 4, 512, px.F32)
    assert clib.poetx_linear_bwd_skew(ctypes.byref(d3), *([fake] * 10), 0, fake, 1 << 30, None) == 2


def test_flag_and_quantised_weight_checks(clib):
    fake = ctypes.c_void_p(0x1000)
    plain = px.make_desc(256, 512, 32, 4, 512, px.BF16)
    mem = px.make_desc(256, 512, 32, 4, 512, px.BF16, flags=px.FLAG_RECOMPUTE_B)
    xq = px.make_desc(256, 512, 32, 4, 512, px.BF16, flags=px.FLAG_RECOMPUTE_B | px.FLAG_W_INT8)
    only_q = px.make_desc(256, 512, 32, 4, 512, px.BF16, flags=px.FLAG_W_INT8)
    xqf = px.make_desc(256, 512, 32, 4, 512, px.BF16, flags=px.FLAG_RECOMPUTE_B | px.FLAG_W_INT8 | px.FLAG_W_INT8_FUSED)
    fused_alone = px.make_desc(256, 512, 32, 4, 512, px.BF16, flags=px.FLAG_RECOMPUTE_B | px.FLAG_W_INT8_FUSED)
    unknown = px.make_desc(256, 512, 32, 4, 512, px.BF16, flags=16)
    w_plain, w_mem, w_xq, w_xqf = (px.poetx_linear_workspace_bytes(d) for d in (plain, mem, xq, xqf))
    assert w_mem >= (256 + 512) * 512 * 2 and w_mem >= w_plain
    # the backward call that recomputes B itself keeps B (and the dequantised weight) behind everything else
    assert w_mem >= (256 + 2 * 512) * 512 * 2
    # the weight is dequantised into the workspace: room for one n x m weight more ...
    assert w_xq >= w_mem + 512 * 256 * 2
    # ... unless the product kernel that converts the codes itself is asked for (these shapes are covered by it)
    assert w_xqf == w_mem
    # a shape it does not cover keeps the dequantised weight whatever the flag says
    xq2 = px.make_desc(96, 160, 32, 4, 512, px.BF16, flags=px.FLAG_RECOMPUTE_B | px.FLAG_W_INT8 | px.FLAG_W_INT8_FUSED)
    assert px.poetx_linear_workspace_bytes(xq2) >= (96 + 160) * 512 * 2 + 160 * 96 * 2
    assert px.poetx_linear_workspace_bytes(fused_alone) == 0                     # nothing to fuse without the INT8 weight
    assert px.poetx_linear_workspace_bytes(only_q) == 0                          # INT8 weight needs the no-activation variant
    assert px.poetx_linear_workspace_bytes(unknown) == 0
    assert clib.poetx_linear_fwd(ctypes.byref(only_q), *([fake] * 9), 1 << 30, None) == 1
    # saved_B may be absent only in the memory-saving variant
    args = [fake] * 7 + [None, fake]
    assert clib.poetx_linear_fwd(ctypes.byref(plain), *args, 1 << 30, None) == 1
    bargs = [fake, fake, None] + [fake] * 10 + [0, fake]
    assert clib.poetx_linear_bwd(ctypes.byref(plain), *bargs, 1 << 30, None) == 1
    assert px.poetx_weight_q8_bytes(512, 256) >= 512 * 256 + 4 * 512
    assert px.poetx_weight_q8_bytes(0, 256) == 0
    assert clib.poetx_weight_quantize_q8(None, px.BF16, 8, 8, fake, None) == 1
    assert clib.poetx_weight_quantize_q8(fake, 5, 8, 8, fake, None) == 1
    assert clib.poetx_weight_dequantize_q8(fake, 8, 0, px.BF16, fake, None) == 1


def test_linear_path_query(clib):
    """poetx_linear_path tells which stages the matrix-core kernels serve: all of them for the benchmark
    shapes, the dense products alone for fp32 tensors, none for small shapes, and the INT8 bit only with the flag."""
    full = px.PATH_APPLY | px.PATH_DENSE | px.PATH_BLOCKGRAD | px.PATH_SERIES | px.PATH_SERIES_ON_CHIP | px.PATH_BWD_ONE_PASS
    assert px.poetx_linear_path(px.make_desc(4096, 14336, 256, 5, 16384, px.BF16)) == full
    b512 = px.poetx_linear_path(px.make_desc(4096, 1024, 512, 5, 16384, px.BF16))
    assert b512 == px.PATH_APPLY | px.PATH_DENSE | px.PATH_BLOCKGRAD | px.PATH_SERIES
    # fp32 tensors: only the dense products have a matrix-core kernel (fp32 MFMA), for multiples of 128
    assert px.poetx_linear_path(px.make_desc(256, 256, 32, 4, 512, px.F32)) == px.PATH_DENSE
    assert px.poetx_linear_path(px.make_desc(64, 64, 16, 3, 256, px.F32)) == 0
    assert px.poetx_linear_path(px.make_desc(512, 1376, 64, 4, 1024, px.BF16)) == 0
    xq = px.make_desc(4096, 4096, 256, 5, 16384, px.BF16, flags=px.FLAG_RECOMPUTE_B | px.FLAG_W_INT8)
    assert px.poetx_linear_path(xq) == full                       # dequantised into the workspace
    xqf = px.make_desc(4096, 4096, 256, 5, 16384, px.BF16, flags=px.FLAG_RECOMPUTE_B | px.FLAG_W_INT8 | px.FLAG_W_INT8_FUSED)
    assert px.poetx_linear_path(xqf) == full | px.PATH_W_INT8_IN_KERNEL
    assert px.poetx_linear_path(px.make_desc(256, 256, 32, 0, 512, px.F32)) == -1     # k < 1
