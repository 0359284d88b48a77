"""Thin binding over the C ABI in include/mars_sched.h (host-only scheduling simulator): argument marshalling only."""
from __future__ import annotations

import ctypes
import os
from typing import Dict

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libmars_sched.so")
EXPORTS = ("mars_sched_bounds", "mars_sched_simulate")
RANDOM, BALANCED, ADAPTIVE = 0, 1, 2
_ROLE_FIELDS = ("short_lo", "short_hi", "long_hi", "p_long", "p_correct", "p_keep", "p_flag_wrong", "p_flag_right")
_I32 = ("item_problem", "item_role", "item_group", "item_member", "item_parent", "item_length", "item_value", "item_reward")
_G32 = ("group_problem", "group_role", "group_index", "group_parent")
_G64 = ("group_t_submit", "group_t_group", "group_t_train")


class Config(ctypes.Structure):
    _fields_ = ([(n, ctypes.c_int32) for n in ("problems", "group_size", "n_select", "segment", "capacity", "strategy", "pipeline", "reserved")] +
                [("seed", ctypes.c_uint64), ("adv_eps", ctypes.c_double)] + [(n, ctypes.c_int32 * 5) for n in _ROLE_FIELDS])


class Summary(ctypes.Structure):
    _fields_ = [("makespan", ctypes.c_int64), ("tokens", ctypes.c_int64), ("sum_t_train", ctypes.c_int64), ("sum_wait", ctypes.c_int64),
                ("n_items", ctypes.c_int32), ("n_groups", ctypes.c_int32), ("early_stop", ctypes.c_int32 * 5)]


class Arrays(ctypes.Structure):
    _fields_ = ([(n, ctypes.c_void_p) for n in _I32] + [("item_t_done", ctypes.c_void_p)] + [(n, ctypes.c_void_p) for n in _G32] +
                [(n, ctypes.c_void_p) for n in _G64] + [("group_adv", ctypes.c_void_p)])


class SchedError(RuntimeError):
    pass


_lib = None


def load_library() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is not built; run `python -m paper_2511_11373_amd.build`")
        lib = ctypes.CDLL(LIB_PATH)
        lib.mars_sched_bounds.argtypes = [ctypes.POINTER(Config), ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64)]
        lib.mars_sched_simulate.argtypes = [ctypes.POINTER(Config), ctypes.POINTER(Summary), ctypes.POINTER(Arrays), ctypes.c_int64, ctypes.c_int64]
        _lib = lib
    return _lib


def make_config(cfg: Dict) -> Config:
    c = Config()
    for n in ("problems", "group_size", "n_select", "segment", "capacity", "strategy", "pipeline"):
        setattr(c, n, int(cfg[n]))
    c.seed = int(cfg["seed"]) & ((1 << 64) - 1)
    c.adv_eps = float(cfg["adv_eps"])
    for n in _ROLE_FIELDS:
        setattr(c, n, (ctypes.c_int32 * 5)(*[int(v) for v in cfg[n]]))
    return c


def simulate(cfg: Dict, details: bool = True) -> Dict:
    """Runs the native simulator.  Returns the summary fields and, with details, one numpy array per table column."""
    lib = load_library()
    c = make_config(cfg)
    mi, mg = ctypes.c_int64(0), ctypes.c_int64(0)
    st = lib.mars_sched_bounds(ctypes.byref(c), ctypes.byref(mi), ctypes.byref(mg))
    if st:
        raise SchedError(f"mars_sched_bounds status {st}")
    out, arrs = {}, Arrays()
    if details:
        for n in _I32:
            out[n] = np.empty(mi.value, dtype=np.int32)
        out["item_t_done"] = np.empty(mi.value, dtype=np.int64)
        for n in _G32:
            out[n] = np.empty(mg.value, dtype=np.int32)
        for n in _G64:
            out[n] = np.empty(mg.value, dtype=np.int64)
        out["group_adv"] = np.empty(mg.value * c.group_size, dtype=np.float64)
        for n, a in out.items():
            setattr(arrs, n, a.ctypes.data)
    s = Summary()
    st = lib.mars_sched_simulate(ctypes.byref(c), ctypes.byref(s), ctypes.byref(arrs) if details else None, mi.value, mg.value)
    if st:
        raise SchedError(f"mars_sched_simulate status {st}")
    res = {"makespan": s.makespan, "tokens": s.tokens, "sum_t_train": s.sum_t_train, "sum_wait": s.sum_wait,
           "n_items": s.n_items, "n_groups": s.n_groups, "early_stop": list(s.early_stop)}
    for n, a in out.items():
        k = s.n_items if n.startswith("item") else s.n_groups * (c.group_size if n == "group_adv" else 1)
        res[n] = a[:k]
    return res
