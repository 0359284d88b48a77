"""Thin binding over the C ABI in include/moe_ffn.h: argument marshalling only.

Tensors are torch tensors on the GPU (torch is used for device memory and
streams, nothing else); every step runs in the library's HIP kernels.  The
library is loaded from the package directory and a missing build is an error:
there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libmoe_ffn.so")

MOE_BF16, MOE_F32 = 0, 1
EXPORTS = ("moe_status_string", "moe_workspace_bytes", "moe_route_topk", "moe_permute",
           "moe_grouped_swiglu", "moe_combine", "moe_forward", "moe_forward_noalloc", "moe_forward_stage_times")
NOALLOC_SCRATCH_BYTES = 32 << 20
NUM_STAGES = 8
STAGE_NAMES = ("router_logits", "topk", "permute", "tile_list", "gate_up_gemm", "down_gemm", "combine", "empty_interval")


class MoeShape(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int32), ("H", ctypes.c_int32), ("E", ctypes.c_int32), ("K", ctypes.c_int32),
                ("I", ctypes.c_int32), ("dtype", ctypes.c_int32), ("renormalize", ctypes.c_int32)]


class MoeError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"moe_ffn status {code}: {msg}")
        self.code = code


_lib = None


def load_library() -> ctypes.CDLL:
    """Open libmoe_ffn.so (built in-tree by paper_2511_11373_amd.build); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is not built; run `python -m paper_2511_11373_amd.build`")
        lib = ctypes.CDLL(LIB_PATH)
        vp, sz = ctypes.c_void_p, ctypes.c_size_t
        sp = ctypes.POINTER(MoeShape)
        lib.moe_status_string.restype = ctypes.c_char_p
        lib.moe_status_string.argtypes = [ctypes.c_int]
        lib.moe_workspace_bytes.argtypes = [sp, ctypes.POINTER(sz)]
        lib.moe_route_topk.argtypes = [sp, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.moe_permute.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.moe_grouped_swiglu.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.moe_combine.argtypes = [sp, vp, vp, vp, vp, vp]
        lib.moe_forward.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.moe_forward_noalloc.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        lib.moe_forward_stage_times.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp,
                                                ctypes.POINTER(ctypes.c_float)]
        for name in EXPORTS[1:]:
            getattr(lib, name).restype = ctypes.c_int
        _lib = lib
    return _lib


def _check(code: int):
    if code != 0:
        raise MoeError(code, load_library().moe_status_string(code).decode())


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_contiguous()
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return MOE_BF16
    if t.dtype == torch.float32:
        return MOE_F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def make_shape(T, H, E, K, I, dtype_code, renormalize=True) -> MoeShape:
    return MoeShape(T, H, E, K, I, dtype_code, int(bool(renormalize)))


def workspace_bytes(shape: MoeShape) -> int:
    out = ctypes.c_size_t(0)
    _check(load_library().moe_workspace_bytes(ctypes.byref(shape), ctypes.byref(out)))
    return out.value


def alloc_workspace(shape: MoeShape, device="cuda") -> torch.Tensor:
    return torch.empty(max(workspace_bytes(shape), 256), dtype=torch.uint8, device=device)


def moe_route_topk(shape: MoeShape, x, w_router, router_bias, ws) -> Tuple[torch.Tensor, torch.Tensor]:
    idx = torch.empty((shape.T, shape.K), dtype=torch.int32, device=x.device)
    w = torch.empty((shape.T, shape.K), dtype=torch.float32, device=x.device)
    _check(load_library().moe_route_topk(ctypes.byref(shape), _ptr(x), _ptr(w_router), _ptr(router_bias), _ptr(idx),
                                         _ptr(w), _ptr(ws), ws.numel(), _stream()))
    return idx, w


def moe_permute(shape: MoeShape, topk_idx, x, ws, want_x_perm=True):
    n = shape.T * shape.K
    dev = topk_idx.device
    off = torch.empty(shape.E + 1, dtype=torch.int32, device=dev)
    r2a = torch.empty(n, dtype=torch.int32, device=dev)
    a2r = torch.empty(n, dtype=torch.int32, device=dev)
    xp = torch.empty((n, shape.H), dtype=x.dtype, device=dev) if want_x_perm else None
    _check(load_library().moe_permute(ctypes.byref(shape), _ptr(topk_idx), _ptr(x), _ptr(off), _ptr(r2a), _ptr(a2r),
                                      _ptr(xp), _ptr(ws), ws.numel(), _stream()))
    return off, r2a, a2r, xp


def moe_grouped_swiglu(shape: MoeShape, x_perm, expert_offsets, w_gate, w_up, w_down, ws) -> torch.Tensor:
    y = torch.empty((shape.T * shape.K, shape.H), dtype=x_perm.dtype, device=x_perm.device)
    _check(load_library().moe_grouped_swiglu(ctypes.byref(shape), _ptr(x_perm), _ptr(expert_offsets), _ptr(w_gate),
                                             _ptr(w_up), _ptr(w_down), _ptr(y), _ptr(ws), ws.numel(), _stream()))
    return y


def moe_combine(shape: MoeShape, y_perm, assign_to_row, topk_w) -> torch.Tensor:
    out = torch.empty((shape.T, shape.H), dtype=y_perm.dtype, device=y_perm.device)
    _check(load_library().moe_combine(ctypes.byref(shape), _ptr(y_perm), _ptr(assign_to_row), _ptr(topk_w), _ptr(out),
                                      _stream()))
    return out


def moe_forward(shape: MoeShape, x, w_router, router_bias, w_gate, w_up, w_down, ws, out=None,
                topk_idx_out=None, topk_w_out=None) -> torch.Tensor:
    if out is None:
        out = torch.empty((shape.T, shape.H), dtype=x.dtype, device=x.device)
    _check(load_library().moe_forward(ctypes.byref(shape), _ptr(x), _ptr(w_router), _ptr(router_bias), _ptr(w_gate),
                                      _ptr(w_up), _ptr(w_down), _ptr(out), _ptr(topk_idx_out), _ptr(topk_w_out),
                                      _ptr(ws), ws.numel(), _stream()))
    return out


def moe_forward_noalloc(shape: MoeShape, x, w_router, router_bias, w_gate, w_up, w_down, out,
                        topk_idx_out=None, topk_w_out=None) -> torch.Tensor:
    """moe_forward on the library's own static scratch: no workspace argument; the call itself allocates nothing, so
    `out` is the caller's."""
    _check(load_library().moe_forward_noalloc(ctypes.byref(shape), _ptr(x), _ptr(w_router), _ptr(router_bias),
                                              _ptr(w_gate), _ptr(w_up), _ptr(w_down), _ptr(out), _ptr(topk_idx_out),
                                              _ptr(topk_w_out), _stream()))
    return out


def moe_forward_stage_times(shape: MoeShape, x, w_router, router_bias, w_gate, w_up, w_down, ws, out=None):
    """moe_forward with per-stage event timing; blocks. Returns (out, [ms per stage])."""
    if out is None:
        out = torch.empty((shape.T, shape.H), dtype=x.dtype, device=x.device)
    ms = (ctypes.c_float * NUM_STAGES)()
    _check(load_library().moe_forward_stage_times(ctypes.byref(shape), _ptr(x), _ptr(w_router), _ptr(router_bias),
                                                  _ptr(w_gate), _ptr(w_up), _ptr(w_down), _ptr(out), _ptr(ws),
                                                  ws.numel(), _stream(), ms))
    return out, [float(v) for v in ms]
