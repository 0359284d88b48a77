"""Thin binding over the C ABI in include/attn_decode.h: argument marshalling only (torch supplies device memory and
streams; every step runs in the library's HIP kernels; a missing build is an error)."""
from __future__ import annotations

import ctypes

import torch

from . import moe
from .moe import _ptr, _stream

EXPORTS = ("attn_decode_workspace_bytes", "attn_decode")
PAGE, HEAD_DIM = 256, 128
_STATUS = {1: "a required pointer is NULL", 2: "unsupported shape", 4: "workspace missing or too small",
           5: "pointer not 16-byte aligned", 6: "HIP launch error"}


class AttnShape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("B", "Hq", "Hkv", "D", "max_pages", "n_pages")]


class AttnError(RuntimeError):
    def __init__(self, code: int):
        super().__init__(f"attn_decode status {code}: {_STATUS.get(code, 'unknown')}")
        self.code = code


_ready = False


def _lib() -> ctypes.CDLL:
    global _ready
    lib = moe.load_library()
    if not _ready:
        vp, sz = ctypes.c_void_p, ctypes.c_size_t
        sp = ctypes.POINTER(AttnShape)
        lib.attn_decode_workspace_bytes.argtypes = [sp, ctypes.POINTER(sz)]
        lib.attn_decode.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        for name in EXPORTS:
            getattr(lib, name).restype = ctypes.c_int
        _ready = True
    return lib


def _check(code: int):
    if code != 0:
        raise AttnError(code)


def make_shape(B, Hq, Hkv, max_pages, n_pages, D=HEAD_DIM) -> AttnShape:
    return AttnShape(B, Hq, Hkv, D, max_pages, n_pages)


def workspace_bytes(shape: AttnShape) -> int:
    out = ctypes.c_size_t(0)
    _check(_lib().attn_decode_workspace_bytes(ctypes.byref(shape), ctypes.byref(out)))
    return out.value


def alloc_workspace(shape: AttnShape, device="cuda") -> torch.Tensor:
    return torch.empty(max(workspace_bytes(shape), 256), dtype=torch.uint8, device=device)


def attn_decode(shape: AttnShape, q, k_pages, v_pages, block_table, seq_lens, ws, out=None) -> torch.Tensor:
    if out is None:
        out = torch.empty((shape.B, shape.Hq, shape.D), dtype=torch.bfloat16, device=q.device)
    _check(_lib().attn_decode(ctypes.byref(shape), _ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(block_table), _ptr(seq_lens),
                              _ptr(out), _ptr(ws), ws.numel(), _stream()))
    return out
