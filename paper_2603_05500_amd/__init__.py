"""Thin Python binding of libpoetx.so (the C ABI declared in include/poetx.h).

Argument marshalling only: every function takes torch tensors that already
live on the GPU, passes their device pointers and the current HIP stream to
the C entry point of the same name, and raises on a non-zero status.  No step
of the method is computed in Python and there is no CPU fallback: if the
library is missing, loading fails.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, Structure, c_char_p, c_int, c_int32, c_int64, c_size_t, c_void_p

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libpoetx.so")

F32, BF16 = 0, 1
CNP_FP32, CNP_BF16 = 0, 1
FLAG_RECOMPUTE_B = 1
FLAG_W_INT8 = 2
FLAG_W_INT8_FUSED = 8
FLAG_BLOCK_GRADS = 4
FEATURE_MAJOR, TOKEN_MAJOR = 0, 1

EXPORTS = (
    "poetx_status_string", "poetx_version", "poetx_debug_force_fma",
    "poetx_cnp_workspace_bytes", "poetx_cnp_build", "poetx_cnp_build_static", "poetx_cnp_bwd_workspace_bytes", "poetx_cnp_bwd",
    "poetx_perm_blockdiag_apply_left", "poetx_perm_blockdiag_apply_right", "poetx_perm_validate", "poetx_merge_workspace_bytes", "poetx_merge_weight",
    "poetx_linear_workspace_bytes", "poetx_linear_path", "poetx_linear_fwd", "poetx_linear_bwd_input", "poetx_linear_bwd_skew",
    "poetx_linear_recompute_b", "poetx_linear_bwd",
    "poetx_weight_q8_bytes", "poetx_weight_quantize_q8", "poetx_weight_dequantize_q8",
    "poetx_profile_begin", "poetx_profile_end",
)
STAGES = ("cnp_fwd", "apply", "dense", "blockgrad", "cnp_bwd", "apply_grad", "layout", "dequant")


class LinearDesc(Structure):
    _fields_ = [("d_in", c_int32), ("d_out", c_int32), ("block", c_int32), ("neumann_k", c_int32),
                ("n_tokens", c_int64), ("dtype", c_int32), ("cnp_precision", c_int32),
                ("flags", c_int32), ("layout", c_int32)]


class PoetxError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


_lib = None


def load_library(path: str | None = None):
    """dlopen libpoetx.so and declare its prototypes.  Raises if it is not built."""
    global _lib
    if _lib is not None:
        return _lib
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise FileNotFoundError(f"{p} not built: run `python -m paper_2603_05500_amd.build` "
                                "(or __graft_entry__.build()) first")
    lib = ctypes.CDLL(p)
    lib.poetx_status_string.restype = c_char_p
    lib.poetx_status_string.argtypes = [c_int]
    lib.poetx_version.restype = c_int
    lib.poetx_debug_force_fma.restype = None
    lib.poetx_debug_force_fma.argtypes = [c_int]
    lib.poetx_cnp_workspace_bytes.restype = c_size_t
    lib.poetx_cnp_workspace_bytes.argtypes = [c_int32, c_int32]
    lib.poetx_cnp_build.restype = c_int
    lib.poetx_cnp_build.argtypes = [c_void_p, c_int32, c_int32, c_int32, c_int32, c_void_p, c_void_p,
                                    c_void_p, c_size_t, c_void_p]
    lib.poetx_cnp_bwd_workspace_bytes.restype = c_size_t
    lib.poetx_cnp_bwd_workspace_bytes.argtypes = [c_int32, c_int32, c_int32]
    lib.poetx_cnp_bwd.restype = c_int
    lib.poetx_cnp_bwd.argtypes = [c_void_p, c_void_p, c_int32, c_int32, c_int32, c_int32, c_void_p, c_int32, c_void_p,
                                  c_size_t, c_void_p]
    lib.poetx_cnp_build_static.restype = c_int
    lib.poetx_cnp_build_static.argtypes = [c_void_p, c_int32, c_int32, c_int32, c_int32, c_void_p, c_void_p, c_void_p]
    for name in ("poetx_perm_blockdiag_apply_left",):
        f = getattr(lib, name)
        f.restype = c_int
        f.argtypes = [c_void_p, c_void_p, c_int32, c_int64, c_int64, c_void_p, c_void_p, c_int32, c_int32,
                      c_int32, c_void_p]
    lib.poetx_perm_blockdiag_apply_right.restype = c_int
    lib.poetx_perm_blockdiag_apply_right.argtypes = [c_void_p, c_void_p, c_int64, c_int32, c_int64, c_void_p,
                                                     c_void_p, c_int32, c_int32, c_int32, c_void_p]
    lib.poetx_merge_workspace_bytes.restype = c_size_t
    lib.poetx_merge_workspace_bytes.argtypes = [c_int32, c_int32, c_int32]
    lib.poetx_merge_weight.restype = c_int
    lib.poetx_merge_weight.argtypes = [c_void_p, c_void_p, c_int32, c_int32, c_void_p, c_void_p, c_void_p, c_void_p,
                                       c_int32, c_int32, c_void_p, c_size_t, c_void_p]
    lib.poetx_perm_validate.restype = c_int
    lib.poetx_perm_validate.argtypes = [c_void_p, c_int32, c_void_p, c_void_p]
    lib.poetx_linear_workspace_bytes.restype = c_size_t
    lib.poetx_linear_workspace_bytes.argtypes = [POINTER(LinearDesc)]
    lib.poetx_linear_path.restype = c_int
    lib.poetx_linear_path.argtypes = [POINTER(LinearDesc)]
    lib.poetx_linear_fwd.restype = c_int
    lib.poetx_linear_fwd.argtypes = [POINTER(LinearDesc)] + [c_void_p] * 9 + [c_size_t, c_void_p]
    lib.poetx_linear_bwd_input.restype = c_int
    lib.poetx_linear_bwd_input.argtypes = [POINTER(LinearDesc)] + [c_void_p] * 9 + [c_size_t, c_void_p]
    lib.poetx_linear_bwd_skew.restype = c_int
    lib.poetx_linear_bwd_skew.argtypes = [POINTER(LinearDesc)] + [c_void_p] * 10 + [c_int32, c_void_p, c_size_t,
                                                                                   c_void_p]
    lib.poetx_linear_bwd.restype = c_int
    lib.poetx_linear_bwd.argtypes = [POINTER(LinearDesc)] + [c_void_p] * 13 + [c_int32, c_void_p, c_size_t, c_void_p]
    lib.poetx_linear_recompute_b.restype = c_int
    lib.poetx_linear_recompute_b.argtypes = [POINTER(LinearDesc)] + [c_void_p] * 6 + [c_size_t, c_void_p]
    lib.poetx_weight_q8_bytes.restype = c_size_t
    lib.poetx_weight_q8_bytes.argtypes = [c_int32, c_int32]
    lib.poetx_weight_quantize_q8.restype = c_int
    lib.poetx_weight_quantize_q8.argtypes = [c_void_p, c_int32, c_int32, c_int32, c_void_p, c_void_p]
    lib.poetx_weight_dequantize_q8.restype = c_int
    lib.poetx_weight_dequantize_q8.argtypes = [c_void_p, c_int32, c_int32, c_int32, c_void_p, c_void_p]
    lib.poetx_profile_begin.restype = c_int
    lib.poetx_profile_begin.argtypes = [c_int32]
    lib.poetx_profile_end.restype = c_int
    lib.poetx_profile_end.argtypes = [POINTER(ctypes.c_double), POINTER(c_int64)]
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().poetx_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != 0:
        raise PoetxError(status, where)


def _torch():
    import torch
    return torch


def _ptr(t):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensors only"
    return c_void_p(t.data_ptr())


def _stream():
    return c_void_p(_torch().cuda.current_stream().cuda_stream)


def dtype_code(t) -> int:
    torch = _torch()
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def make_desc(d_in, d_out, block, neumann_k, n_tokens, dtype, cnp_precision=None, flags=0,
              layout=FEATURE_MAJOR) -> LinearDesc:
    if cnp_precision is None:
        cnp_precision = CNP_FP32 if dtype == F32 else CNP_BF16
    return LinearDesc(d_in, d_out, block, neumann_k, n_tokens, dtype, cnp_precision, flags, layout)


def poetx_debug_force_fma(on: bool):
    load_library().poetx_debug_force_fma(1 if on else 0)


def poetx_cnp_workspace_bytes(d: int, b: int) -> int:
    return load_library().poetx_cnp_workspace_bytes(d, b)


def poetx_linear_workspace_bytes(desc: LinearDesc) -> int:
    return load_library().poetx_linear_workspace_bytes(ctypes.byref(desc))


def poetx_cnp_build(theta, d, b, k, precision, G_f32=None, E_bf16=None, ws=None):
    lib = load_library()
    _check(lib.poetx_cnp_build(_ptr(theta), d, b, k, precision, _ptr(G_f32), _ptr(E_bf16), _ptr(ws),
                               ws.numel() * ws.element_size() if ws is not None else 0, _stream()),
           "poetx_cnp_build")


def poetx_cnp_bwd_workspace_bytes(d: int, b: int, k: int) -> int:
    return load_library().poetx_cnp_bwd_workspace_bytes(d, b, k)


def poetx_cnp_bwd(theta, dG, d, b, k, precision, dtheta, accumulate, ws):
    lib = load_library()
    _check(lib.poetx_cnp_bwd(_ptr(theta), _ptr(dG), d, b, k, precision, _ptr(dtheta), int(bool(accumulate)), _ptr(ws),
                             _ws_bytes(ws), _stream()),
           "poetx_cnp_bwd")


def poetx_cnp_build_static(theta, d, b, k, precision, G_f32=None, E_bf16=None):
    lib = load_library()
    _check(lib.poetx_cnp_build_static(_ptr(theta), d, b, k, precision, _ptr(G_f32), _ptr(E_bf16), _stream()),
           "poetx_cnp_build_static")


def poetx_perm_blockdiag_apply_left(V, out, perm, blocks, b, transpose_G):
    lib = load_library()
    d, cols = V.shape
    _check(lib.poetx_perm_blockdiag_apply_left(_ptr(V), _ptr(out), d, cols, V.stride(0), _ptr(perm), _ptr(blocks),
                                               b, int(bool(transpose_G)), dtype_code(V), _stream()),
           "poetx_perm_blockdiag_apply_left")


def poetx_perm_blockdiag_apply_right(V, out, perm, blocks, b, transpose_G):
    lib = load_library()
    rows, d = V.shape
    _check(lib.poetx_perm_blockdiag_apply_right(_ptr(V), _ptr(out), rows, d, V.stride(0), _ptr(perm), _ptr(blocks),
                                                b, int(bool(transpose_G)), dtype_code(V), _stream()),
           "poetx_perm_blockdiag_apply_right")


def poetx_merge_workspace_bytes(n: int, m: int, dtype: int) -> int:
    return load_library().poetx_merge_workspace_bytes(n, m, dtype)


def poetx_merge_weight(W, W_out, perm_R, perm_P, blocks_R, blocks_P, b, ws):
    n, m = W.shape
    _check(load_library().poetx_merge_weight(_ptr(W), _ptr(W_out), n, m, _ptr(perm_R), _ptr(perm_P), _ptr(blocks_R),
                                             _ptr(blocks_P), b, dtype_code(W), _ptr(ws), _ws_bytes(ws), _stream()),
           "poetx_merge_weight")


def poetx_perm_validate(perm, scratch) -> bool:
    """True if perm is a bijection; False if the library reports BAD_PERM."""
    lib = load_library()
    rc = lib.poetx_perm_validate(_ptr(perm), perm.numel(), _ptr(scratch), _stream())
    if rc == 3:
        return False
    _check(rc, "poetx_perm_validate")
    return True


def _ws_bytes(ws):
    return ws.numel() * ws.element_size()


PATH_APPLY, PATH_DENSE, PATH_BLOCKGRAD, PATH_SERIES, PATH_SERIES_ON_CHIP, PATH_BWD_ONE_PASS, PATH_W_INT8_IN_KERNEL = \
    1, 2, 4, 8, 16, 32, 64


def poetx_linear_path(desc) -> int:
    """Bit mask of the stages the matrix-core kernels serve for `desc` (negative: invalid descriptor)."""
    return load_library().poetx_linear_path(ctypes.byref(desc))


def poetx_linear_fwd(desc, X, W, perm_R, perm_P, blocks_R, blocks_P, Z, saved_B, ws):
    lib = load_library()
    _check(lib.poetx_linear_fwd(ctypes.byref(desc), _ptr(X), _ptr(W), _ptr(perm_R), _ptr(perm_P), _ptr(blocks_R),
                                _ptr(blocks_P), _ptr(Z), _ptr(saved_B), _ptr(ws), _ws_bytes(ws), _stream()),
           "poetx_linear_fwd")


def poetx_linear_recompute_b(desc, X, W, perm_R, blocks_R, B_out, ws):
    lib = load_library()
    _check(lib.poetx_linear_recompute_b(ctypes.byref(desc), _ptr(X), _ptr(W), _ptr(perm_R), _ptr(blocks_R), _ptr(B_out),
                                        _ptr(ws), _ws_bytes(ws), _stream()),
           "poetx_linear_recompute_b")


def poetx_linear_bwd_input(desc, dZ, W, perm_R, perm_P, blocks_R, blocks_P, dX, dA, ws):
    lib = load_library()
    _check(lib.poetx_linear_bwd_input(ctypes.byref(desc), _ptr(dZ), _ptr(W), _ptr(perm_R), _ptr(perm_P),
                                      _ptr(blocks_R), _ptr(blocks_P), _ptr(dX), _ptr(dA), _ptr(ws), _ws_bytes(ws),
                                      _stream()),
           "poetx_linear_bwd_input")


def poetx_linear_bwd_skew(desc, X, dZ, saved_B, dA, perm_R, perm_P, theta_R, theta_P, dtheta_R, dtheta_P,
                          accumulate, ws):
    lib = load_library()
    _check(lib.poetx_linear_bwd_skew(ctypes.byref(desc), _ptr(X), _ptr(dZ), _ptr(saved_B), _ptr(dA), _ptr(perm_R),
                                     _ptr(perm_P), _ptr(theta_R), _ptr(theta_P), _ptr(dtheta_R), _ptr(dtheta_P),
                                     int(bool(accumulate)), _ptr(ws), _ws_bytes(ws), _stream()),
           "poetx_linear_bwd_skew")


def poetx_linear_bwd(desc, X, dZ, saved_B, W, perm_R, perm_P, blocks_R, blocks_P, theta_R, theta_P, dX,
                     dtheta_R, dtheta_P, accumulate, ws):
    lib = load_library()
    _check(lib.poetx_linear_bwd(ctypes.byref(desc), _ptr(X), _ptr(dZ), _ptr(saved_B), _ptr(W), _ptr(perm_R),
                                _ptr(perm_P), _ptr(blocks_R), _ptr(blocks_P), _ptr(theta_R), _ptr(theta_P),
                                _ptr(dX), _ptr(dtheta_R), _ptr(dtheta_P), int(bool(accumulate)), _ptr(ws),
                                _ws_bytes(ws), _stream()),
           "poetx_linear_bwd")


def poetx_weight_q8_bytes(n: int, m: int) -> int:
    return load_library().poetx_weight_q8_bytes(n, m)


def poetx_weight_quantize_q8(W, Wq):
    """W: n x m tensor (f32 or bf16) -> Wq: uint8/int8 buffer of poetx_weight_q8_bytes(n, m) bytes."""
    n, m = W.shape
    _check(load_library().poetx_weight_quantize_q8(_ptr(W), dtype_code(W), n, m, _ptr(Wq), _stream()),
           "poetx_weight_quantize_q8")


def poetx_weight_dequantize_q8(Wq, W_out):
    n, m = W_out.shape
    _check(load_library().poetx_weight_dequantize_q8(_ptr(Wq), n, m, dtype_code(W_out), _ptr(W_out), _stream()),
           "poetx_weight_dequantize_q8")


def poetx_profile_begin(max_records: int = 65536):
    _check(load_library().poetx_profile_begin(max_records), "poetx_profile_begin")


def poetx_profile_end() -> dict:
    """{stage: (milliseconds, timed launch groups)} since poetx_profile_begin."""
    ms = (ctypes.c_double * len(STAGES))()
    cnt = (c_int64 * len(STAGES))()
    _check(load_library().poetx_profile_end(ms, cnt), "poetx_profile_end")
    return {s: (ms[i], cnt[i]) for i, s in enumerate(STAGES)}
