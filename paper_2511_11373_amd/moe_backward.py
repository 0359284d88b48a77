"""Thin binding over the C ABI in include/moe_ffn_backward.h: argument marshalling only.

Same rules as the forward binding: torch supplies device memory and streams, every step runs in the
library's HIP kernels, a missing build is an error.
"""
from __future__ import annotations

import ctypes
from typing import Dict, Optional

import torch

from . import moe
from .moe import MoeShape, _check, _ptr, _stream

EXPORTS = ("moe_backward_workspace_bytes", "moe_grouped_swiglu_backward", "moe_backward", "moe_backward_stage_times",
           "moe_forward_saving", "moe_backward_saved")
NUM_STAGES = 13
STAGE_NAMES = ("route", "permute_copy", "tile_list", "g_gemm", "u_gemm", "dq_gemm", "swiglu_rows", "dx_rows_gemm", "d_w_down",
               "d_w_gate", "d_w_up", "softmax_dx_router", "empty_interval")

_ready = False


def _lib() -> ctypes.CDLL:
    global _ready
    lib = moe.load_library()
    if not _ready:
        vp, sz = ctypes.c_void_p, ctypes.c_size_t
        sp = ctypes.POINTER(MoeShape)
        lib.moe_backward_workspace_bytes.argtypes = [sp, ctypes.POINTER(sz)]
        lib.moe_grouped_swiglu_backward.argtypes = [sp] + [vp] * 11 + [sz, vp]
        lib.moe_backward.argtypes = [sp] + [vp] * 14 + [sz, vp]
        lib.moe_backward_stage_times.argtypes = [sp] + [vp] * 14 + [sz, vp, ctypes.POINTER(ctypes.c_float)]
        lib.moe_forward_saving.argtypes = [sp] + [vp] * 12 + [sz, vp]
        lib.moe_backward_saved.argtypes = [sp] + [vp] * 18 + [sz, vp]
        for name in EXPORTS:
            getattr(lib, name).restype = ctypes.c_int
        _ready = True
    return lib


def workspace_bytes(shape: MoeShape) -> int:
    out = ctypes.c_size_t(0)
    _check(_lib().moe_backward_workspace_bytes(ctypes.byref(shape), ctypes.byref(out)))
    return out.value


def alloc_workspace(shape: MoeShape, device="cuda") -> torch.Tensor:
    return torch.empty(max(workspace_bytes(shape), 256), dtype=torch.uint8, device=device)


def moe_grouped_swiglu_backward(shape: MoeShape, x_perm, expert_offsets, w_gate, w_up, w_down, dy_perm, ws) -> Dict[str, torch.Tensor]:
    n = shape.T * shape.K
    dev = x_perm.device
    out = {"d_x_perm": torch.empty((n, shape.H), dtype=x_perm.dtype, device=dev),
           "d_w_gate": torch.empty((shape.E, shape.I, shape.H), dtype=torch.float32, device=dev),
           "d_w_up": torch.empty((shape.E, shape.I, shape.H), dtype=torch.float32, device=dev),
           "d_w_down": torch.empty((shape.E, shape.H, shape.I), dtype=torch.float32, device=dev)}
    _check(_lib().moe_grouped_swiglu_backward(ctypes.byref(shape), _ptr(x_perm), _ptr(expert_offsets), _ptr(w_gate), _ptr(w_up),
                                              _ptr(w_down), _ptr(dy_perm), _ptr(out["d_x_perm"]), _ptr(out["d_w_gate"]),
                                              _ptr(out["d_w_up"]), _ptr(out["d_w_down"]), _ptr(ws), ws.numel(), _stream()))
    return out


def moe_backward(shape: MoeShape, x, w_router, router_bias: Optional[torch.Tensor], w_gate, w_up, w_down, d_out, ws,
                 out: Optional[Dict[str, torch.Tensor]] = None) -> Dict[str, torch.Tensor]:
    dev = x.device
    if out is None:
        out = {"d_x": torch.empty((shape.T, shape.H), dtype=x.dtype, device=dev),
               "d_w_router": torch.empty((shape.E, shape.H), dtype=torch.float32, device=dev),
               "d_router_bias": torch.empty((shape.E,), dtype=torch.float32, device=dev),
               "d_w_gate": torch.empty((shape.E, shape.I, shape.H), dtype=torch.float32, device=dev),
               "d_w_up": torch.empty((shape.E, shape.I, shape.H), dtype=torch.float32, device=dev),
               "d_w_down": torch.empty((shape.E, shape.H, shape.I), dtype=torch.float32, device=dev)}
    _check(_lib().moe_backward(ctypes.byref(shape), _ptr(x), _ptr(w_router), _ptr(router_bias), _ptr(w_gate), _ptr(w_up),
                               _ptr(w_down), _ptr(d_out), _ptr(out["d_x"]), _ptr(out["d_w_router"]), _ptr(out["d_router_bias"]),
                               _ptr(out["d_w_gate"]), _ptr(out["d_w_up"]), _ptr(out["d_w_down"]), _ptr(ws), ws.numel(), _stream()))
    return out


def moe_forward_saving(shape: MoeShape, x, w_router, router_bias: Optional[torch.Tensor], w_gate, w_up, w_down, ws,
                       out=None, g_rows=None, u_rows=None, topk_idx_out=None, topk_w_out=None):
    """moe_forward that also returns the expert pre-activations of every expert-sorted row: (out, g_rows, u_rows); the
    routing goes to topk_idx_out / topk_w_out when given.  ws: a forward workspace (moe.alloc_workspace)."""
    dev, n = x.device, shape.T * shape.K
    if out is None:
        out = torch.empty((shape.T, shape.H), dtype=torch.bfloat16, device=dev)
    if g_rows is None:
        g_rows = torch.empty((max(n, 1), shape.I), dtype=torch.bfloat16, device=dev)
    if u_rows is None:
        u_rows = torch.empty((max(n, 1), shape.I), dtype=torch.bfloat16, device=dev)
    _check(_lib().moe_forward_saving(ctypes.byref(shape), _ptr(x), _ptr(w_router), _ptr(router_bias), _ptr(w_gate), _ptr(w_up),
                                     _ptr(w_down), _ptr(out), _ptr(g_rows), _ptr(u_rows), _ptr(topk_idx_out), _ptr(topk_w_out), _ptr(ws),
                                     ws.numel(), _stream()))
    return out, g_rows, u_rows


def moe_backward_saved(shape: MoeShape, x, w_router, router_bias: Optional[torch.Tensor], w_gate, w_up, w_down, d_out, g_rows,
                       u_rows, ws, out: Optional[Dict[str, torch.Tensor]] = None, topk_idx=None, topk_w=None) -> Dict[str, torch.Tensor]:
    """moe_backward reading the pre-activations (and, when given, the routing) that moe_forward_saving kept.
    ws: a backward workspace."""
    dev = x.device
    if out is None:
        out = {"d_x": torch.empty((shape.T, shape.H), dtype=torch.bfloat16, device=dev),
               "d_w_router": torch.empty((shape.E, shape.H), dtype=torch.float32, device=dev),
               "d_router_bias": torch.empty((shape.E,), dtype=torch.float32, device=dev),
               "d_w_gate": torch.empty((shape.E, shape.I, shape.H), dtype=torch.float32, device=dev),
               "d_w_up": torch.empty((shape.E, shape.I, shape.H), dtype=torch.float32, device=dev),
               "d_w_down": torch.empty((shape.E, shape.H, shape.I), dtype=torch.float32, device=dev)}
    _check(_lib().moe_backward_saved(ctypes.byref(shape), _ptr(x), _ptr(w_router), _ptr(router_bias), _ptr(w_gate), _ptr(w_up),
                                     _ptr(w_down), _ptr(d_out), _ptr(g_rows), _ptr(u_rows), _ptr(topk_idx), _ptr(topk_w), _ptr(out["d_x"]),
                                     _ptr(out["d_w_router"]),
                                     _ptr(out["d_router_bias"]), _ptr(out["d_w_gate"]), _ptr(out["d_w_up"]), _ptr(out["d_w_down"]),
                                     _ptr(ws), ws.numel(), _stream()))
    return out


def moe_backward_stage_times(shape: MoeShape, x, w_router, router_bias, w_gate, w_up, w_down, d_out, ws, out):
    """moe_backward with per-stage event timing; blocks.  Returns [ms per stage]."""
    ms = (ctypes.c_float * NUM_STAGES)()
    _check(_lib().moe_backward_stage_times(ctypes.byref(shape), _ptr(x), _ptr(w_router), _ptr(router_bias), _ptr(w_gate), _ptr(w_up),
                                           _ptr(w_down), _ptr(d_out), _ptr(out["d_x"]), _ptr(out["d_w_router"]),
                                           _ptr(out["d_router_bias"]), _ptr(out["d_w_gate"]), _ptr(out["d_w_up"]),
                                           _ptr(out["d_w_down"]), _ptr(ws), ws.numel(), _stream(), ms))
    return list(ms)
