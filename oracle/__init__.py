"""CPU oracle of the routed-expert MoE FFN block: ctypes front end.

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the
benchmark's CPU-baseline leg; never by the GPU library or its binding.
The arithmetic lives in moe_oracle.c (see its header for the definition and
for what pins it); this file only builds that C file with gcc and marshals
numpy arrays.  `bruteforce.py` is a second, independent definition in numpy.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.c")
_LIB = os.path.join(_HERE, "libmoe_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile moe_oracle.c with gcc (plain -O2, OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
    return _lib


def num_threads() -> int:
    """Threads the OpenMP loops of the oracle will use."""
    omp = ctypes.CDLL("libgomp.so.1")
    return int(omp.omp_get_max_threads())


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"oracle {what} failed with code {rc}")


def router_logits(x, w_router, bias=None) -> np.ndarray:
    x, w_router = _f32(x), _f32(w_router)
    T, H = x.shape
    E = w_router.shape[0]
    assert w_router.shape == (E, H)
    b = None if bias is None else _f32(bias)
    out = np.empty((T, E), dtype=np.float32)
    _check(_load().oracle_router_logits(T, H, E, _p(x), _p(w_router), _p(b), _p(out)), "router_logits")
    return out


def topk_from_logits(logits, K: int, renormalize: bool = True) -> Tuple[np.ndarray, np.ndarray]:
    logits = _f32(logits)
    T, E = logits.shape
    idx = np.empty((T, K), dtype=np.int32)
    w = np.empty((T, K), dtype=np.float32)
    _check(_load().oracle_topk_from_logits(T, E, K, int(renormalize), _p(logits), _p(idx), _p(w)), "topk")
    return idx, w


def route_topk(x, w_router, K: int, bias=None, renormalize: bool = True):
    x, w_router = _f32(x), _f32(w_router)
    T, H = x.shape
    E = w_router.shape[0]
    b = None if bias is None else _f32(bias)
    idx = np.empty((T, K), dtype=np.int32)
    w = np.empty((T, K), dtype=np.float32)
    _check(_load().oracle_route_topk(T, H, E, K, int(renormalize), _p(x), _p(w_router), _p(b),
                                     _p(idx), _p(w)), "route_topk")
    return idx, w


def permute(topk_idx, E: int):
    idx = _i32(topk_idx).reshape(-1)
    n = idx.shape[0]
    off = np.empty(E + 1, dtype=np.int32)
    r2a = np.empty(n, dtype=np.int32)
    a2r = np.empty(n, dtype=np.int32)
    _check(_load().oracle_permute(n, E, _p(idx), _p(off), _p(r2a), _p(a2r)), "permute")
    return off, r2a, a2r


def gather_rows(x, row_to_assign, K: int) -> np.ndarray:
    x, r2a = _f32(x), _i32(row_to_assign)
    n, H = r2a.shape[0], x.shape[1]
    xp = np.empty((n, H), dtype=np.float32)
    _check(_load().oracle_gather_rows(n, K, H, _p(x), _p(r2a), _p(xp)), "gather_rows")
    return xp


def grouped_swiglu(x_perm, expert_offsets, w_gate, w_up, w_down) -> np.ndarray:
    xp, off = _f32(x_perm), _i32(expert_offsets)
    wg, wu, wd = _f32(w_gate), _f32(w_up), _f32(w_down)
    n, H = xp.shape
    E, I, _ = wg.shape
    assert wg.shape == (E, I, H) and wu.shape == (E, I, H) and wd.shape == (E, H, I)
    y = np.empty((n, H), dtype=np.float64)
    _check(_load().oracle_grouped_swiglu(n, H, E, I, _p(xp), _p(off), _p(wg), _p(wu), _p(wd), _p(y)),
           "grouped_swiglu")
    return y


def combine(y_perm, assign_to_row, topk_w) -> np.ndarray:
    y = np.ascontiguousarray(y_perm, dtype=np.float64)
    w = _f32(topk_w)
    T, K = w.shape
    H = y.shape[1]
    a2r = _i32(assign_to_row).reshape(-1)
    out = np.empty((T, H), dtype=np.float64)
    _check(_load().oracle_combine(T, H, K, _p(y), _p(a2r), _p(w), _p(out)), "combine")
    return out


def forward(x, w_router, w_gate, w_up, w_down, K: int, bias=None, renormalize: bool = True):
    """Returns (out [T,H] float64, topk_idx [T,K] int32, topk_w [T,K] float32)."""
    x, wr = _f32(x), _f32(w_router)
    wg, wu, wd = _f32(w_gate), _f32(w_up), _f32(w_down)
    T, H = x.shape
    E, I, _ = wg.shape
    b = None if bias is None else _f32(bias)
    out = np.empty((T, H), dtype=np.float64)
    idx = np.empty((T, K), dtype=np.int32)
    w = np.empty((T, K), dtype=np.float32)
    _check(_load().oracle_forward(T, H, E, K, I, int(renormalize), _p(x), _p(wr), _p(b), _p(wg), _p(wu),
                                  _p(wd), _p(out), _p(idx), _p(w)), "forward")
    return out, idx, w


def forward_tokens(x, topk_idx, topk_w, w_gate, w_up, w_down, tokens) -> np.ndarray:
    """Block output rows for the listed tokens only, given the batch's routing."""
    x = _f32(x)
    wg, wu, wd = _f32(w_gate), _f32(w_up), _f32(w_down)
    idx, w = _i32(topk_idx), _f32(topk_w)
    K = idx.shape[1]
    H = x.shape[1]
    I = wg.shape[1]
    tok = _i32(tokens)
    out = np.empty((tok.shape[0], H), dtype=np.float64)
    _check(_load().oracle_forward_tokens(H, K, I, _p(x), _p(idx), _p(w), _p(wg), _p(wu), _p(wd),
                                         tok.shape[0], _p(tok), _p(out)), "forward_tokens")
    return out
