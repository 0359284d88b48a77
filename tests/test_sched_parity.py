"""The native scheduling simulator against the Python oracle, bit for bit (host code on both sides: runs without a GPU).
Every table column, every time stamp and every advantage must be identical for all strategies, with and without the
pipeline, with and without segments, with and without a slot limit."""
import ctypes
import itertools
import os
import re

import numpy as np
import pytest

from oracle import sched_oracle as so
from paper_2511_11373_amd import build as hip_build
from paper_2511_11373_amd import sched

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ONE = 1 << 24


@pytest.fixture(scope="module", autouse=True)
def lib():
    if not os.path.exists(sched.LIB_PATH):
        hip_build.build_host()
    return sched.load_library()


def cfg_of(seed, **kw):
    cfg = dict(problems=9, group_size=8, n_select=2, segment=4096, capacity=0, strategy=so.ADAPTIVE, pipeline=1, seed=seed,
               adv_eps=1e-6,
               short_lo=[1000, 500, 1000, 500, 1000], short_hi=[8000, 4000, 8000, 4000, 8000], long_hi=[65536, 30000, 65536, 30000, 65536],
               p_long=[ONE // 8, ONE // 16, ONE // 8, ONE // 16, ONE // 8],
               p_correct=[ONE * 2 // 5, 0, ONE // 2, 0, ONE // 2], p_keep=[0, 0, ONE * 9 // 10, 0, ONE * 9 // 10],
               p_flag_wrong=[0, ONE * 7 // 10, 0, ONE * 3 // 4, 0], p_flag_right=[0, ONE // 5, 0, ONE // 6, 0])
    cfg.update(kw)
    return cfg


def compare(cfg):
    o = so.simulate(cfg)
    n = sched.simulate(cfg)
    assert n["makespan"] == o["makespan"] and n["tokens"] == o["tokens"]
    assert n["n_items"] == len(o["items"]) and n["n_groups"] == len(o["groups"])
    assert n["early_stop"] == o["early_stop"]
    assert n["sum_t_train"] == o["sum_t_train"] and n["sum_wait"] == o["sum_wait"]
    for col, key in (("item_problem", "problem"), ("item_role", "role"), ("item_group", "group"), ("item_member", "member"),
                     ("item_parent", "parent"), ("item_length", "length"), ("item_value", "value"), ("item_reward", "reward"),
                     ("item_t_done", "t_done")):
        assert np.array_equal(n[col], np.array([it[key] for it in o["items"]], dtype=n[col].dtype)), col
    for col, key in (("group_problem", "problem"), ("group_role", "role"), ("group_index", "group"), ("group_parent", "parent"),
                     ("group_t_submit", "t_submit"), ("group_t_group", "t_group"), ("group_t_train", "t_train")):
        assert np.array_equal(n[col], np.array([g[key] for g in o["groups"]], dtype=n[col].dtype)), col
    adv = np.array([a for g in o["groups"] for a in g["adv"]], dtype=np.float64)
    assert np.array_equal(n["group_adv"].view(np.uint64), adv.view(np.uint64))       # same bits
    return o


@pytest.mark.parametrize("strategy,pipeline,segment,capacity",
                         list(itertools.product((0, 1, 2), (0, 1), (4096, 1 << 20), (0, 37))))
def test_native_equals_oracle(strategy, pipeline, segment, capacity):
    compare(cfg_of(11 + strategy, strategy=strategy, pipeline=pipeline, segment=segment, capacity=capacity))


def test_other_group_sizes_selections_and_degenerate_cases():
    compare(cfg_of(3, group_size=5, n_select=3, problems=7))
    compare(cfg_of(4, group_size=1, n_select=1, problems=30, capacity=4))
    compare(cfg_of(5, n_select=8, problems=3, strategy=so.BALANCED))
    compare(cfg_of(6, p_correct=[ONE] * 5))                                    # nothing to correct: stops after Verifier1
    compare(cfg_of(7, p_correct=[0] * 5, p_keep=[0] * 5, p_flag_wrong=[0, ONE, 0, ONE, 0]))     # never fixed: all five roles run
    compare(cfg_of(8, segment=1, problems=1, short_lo=[3] * 5, short_hi=[5] * 5, long_hi=[9] * 5))   # one token per stage
    o = compare(cfg_of((1 << 64) - 1, problems=1))
    assert len(o["groups"]) >= 1


def test_symbols_and_rejection_of_bad_configurations(lib):
    hdr = open(os.path.join(ROOT, "include", "mars_sched.h")).read()
    declared = set(re.findall(r"\b(mars_sched_[a-z_]+)\s*\(", hdr))
    assert declared == set(sched.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None
    mi, mg = ctypes.c_int64(0), ctypes.c_int64(0)
    assert lib.mars_sched_bounds(None, ctypes.byref(mi), ctypes.byref(mg)) == 1
    for bad in (dict(problems=0), dict(group_size=65), dict(n_select=9), dict(segment=0), dict(strategy=3), dict(capacity=-1),
                dict(short_hi=[10, 4000, 8000, 4000, 8000]), dict(p_long=[ONE + 1] * 5)):
        c = sched.make_config(cfg_of(1, **bad))
        assert lib.mars_sched_bounds(ctypes.byref(c), ctypes.byref(mi), ctypes.byref(mg)) == 2, bad
    c = sched.make_config(cfg_of(1))
    assert lib.mars_sched_bounds(ctypes.byref(c), ctypes.byref(mi), ctypes.byref(mg)) == 0
    assert mg.value == 9 * 9 and mi.value == 9 * 9 * 8
    s = sched.Summary()
    arrs = sched.Arrays()
    assert lib.mars_sched_simulate(ctypes.byref(c), None, None, 0, 0) == 1
    assert lib.mars_sched_simulate(ctypes.byref(c), ctypes.byref(s), ctypes.byref(arrs), 1, 1) == 3       # tables too small
    assert lib.mars_sched_simulate(ctypes.byref(c), ctypes.byref(s), None, 0, 0) == 0 and s.n_groups > 0
