"""Pins of the scheduling oracle to things other than itself (CPU only): the published SplitMix64 outputs, Eq. 1's closed
form on 0/1 rewards, degenerate configurations whose whole timeline can be written down by hand, conservation laws of
the event model, the defining properties of the three sampling strategies, and the paper's qualitative claims (agent-level
pipelining and segment rollout shorten the time from submission to training; Sections 2.3 and 3.3)."""
import math

import numpy as np
import pytest

from oracle import sched_oracle as so

ONE = 1 << 24


def base_cfg(**kw):
    cfg = dict(problems=6, group_size=8, n_select=2, segment=4096, capacity=0, strategy=so.ADAPTIVE, pipeline=1, seed=7,
               adv_eps=1e-6,
               short_lo=[1000] * 5, short_hi=[8000] * 5, long_hi=[64000] * 5, p_long=[ONE // 8] * 5,
               p_correct=[ONE // 2, 0, ONE // 2, 0, ONE // 2], p_keep=[0, 0, ONE * 9 // 10, 0, ONE * 9 // 10],
               p_flag_wrong=[0, ONE * 7 // 10, 0, ONE * 7 // 10, 0], p_flag_right=[0, ONE // 5, 0, ONE // 5, 0])
    cfg.update(kw)
    return cfg


def test_splitmix64_published_outputs():
    # the generator seeded with 0 yields these first three values (reference implementation by Vigna)
    g = 0x9E3779B97F4A7C15
    assert so.splitmix64(0) == 0xE220A8397B1DCDAF
    assert so.splitmix64(g) == 0x6E789E6AA1B965F4
    assert so.splitmix64((2 * g) & so.MASK) == 0x06C45D188009454F


def test_advantages_closed_form():
    a = so.advantages([1, 0, 0, 1, 0, 0, 0, 0], 0.0)
    p = 0.25
    assert a[0] == pytest.approx((1 - p) / math.sqrt(p * (1 - p)), rel=1e-15)
    assert abs(sum(a)) < 1e-12 and np.var(a) == pytest.approx(1.0, rel=1e-12)
    assert so.advantages([1] * 8, 1e-6) == [0.0] * 8


def test_hand_worked_timeline_all_wrong_then_fixed():
    # every solution wrong, every error found, every correction right, no false alarms, every output exactly L tokens:
    # Solver (1 group) -> Verifier1 (2) -> Corrector1 (2) -> Verifier2 (2 groups, nothing flagged) -> stop.  Each agent takes L.
    L = 3000
    cfg = base_cfg(problems=3, segment=1 << 20, short_lo=[L] * 5, short_hi=[L] * 5, long_hi=[L] * 5, p_long=[0] * 5,
                   p_correct=[0, 0, ONE, 0, ONE], p_keep=[0, 0, ONE, 0, ONE], p_flag_wrong=[0, ONE, 0, ONE, 0],
                   p_flag_right=[0] * 5)
    r = so.simulate(cfg)
    assert len(r["groups"]) == 3 * 7 and len(r["items"]) == 3 * 7 * 8
    assert r["makespan"] == 4 * L and r["tokens"] == 3 * 7 * 8 * L
    assert r["early_stop"] == [0, 0, 0, 0, 3]                  # Corrector2 found nothing to correct
    for g in r["groups"]:
        assert g["t_group"] == (g["role"] + 1) * L and g["t_train"] == g["t_group"]
        assert g["adv"] == [0.0] * 8                           # all rewards equal inside every group
    base = so.simulate(dict(cfg, pipeline=0))
    assert all(g["t_train"] == 4 * L for g in base["groups"])
    # mean time to training: (1*1 + 2*2 + 2*3 + 2*4) / 7 * L with the pipeline, 4 L without
    assert r["sum_t_train"] == 3 * 19 * L and base["sum_t_train"] == 3 * 28 * L


def test_all_correct_stops_after_verifier1():
    cfg = base_cfg(problems=2, p_correct=[ONE, 0, ONE, 0, ONE], p_flag_right=[0] * 5)
    r = so.simulate(cfg)
    assert len(r["groups"]) == 2 * 3 and r["early_stop"] == [0, 0, 2, 0, 0]
    assert all(it["reward"] == 1 for it in r["items"])         # correct solutions, and Verifiers that rightly raise no flag


def test_conservation_and_event_consistency():
    for strat in (so.RANDOM, so.BALANCED, so.ADAPTIVE):
        r = so.simulate(base_cfg(strategy=strat, problems=12, capacity=40))
        items, groups = r["items"], r["groups"]
        assert r["tokens"] == sum(it["length"] for it in items)
        assert r["makespan"] >= r["tokens"] / 40               # 40 decode slots, one token per slot and time unit
        for g in groups:
            assert len(g["members"]) == 8 and g["t_group"] == max(items[i]["t_done"] for i in g["members"])
            assert g["t_group"] >= g["t_submit"] + max(items[i]["length"] for i in g["members"])
            assert abs(sum(g["adv"])) < 1e-9
            if g["role"] > 0:
                par = items[g["parent"]]
                assert par["problem"] == g["problem"] and par["role"] == g["role"] - 1 and par["t_done"] <= g["t_submit"]
                if g["role"] in (2, 4):
                    assert par["value"] == 1                   # a Corrector only works on a report that flags an error
        per = {}
        for g in groups:
            per.setdefault((g["problem"], g["role"]), []).append(g)
        assert all(len(v) <= 2 for v in per.values()) and all(len(per[(p, 0)]) == 1 for p in range(12))
        # rewards follow Section 3.2
        for it in items:
            if it["role"] in (1, 3):
                assert it["reward"] == int(it["value"] == (1 - items[it["parent"]]["value"]))
            else:
                assert it["reward"] == it["value"]


def test_sampling_strategies_on_a_crafted_pool():
    items = [{"reward": r} for r in (1, 1, 0, 1, 0, 0, 1, 1)]
    pool = list(range(8))
    for problem in range(20):
        c = base_cfg(strategy=so.BALANCED)
        sel = so.select_inputs(c, items, pool, problem, 1)
        assert len(set(sel)) == 2 and sorted(items[i]["reward"] for i in sel) == [0, 1]
        c = base_cfg(strategy=so.ADAPTIVE)
        assert all(items[i]["reward"] == 0 for i in so.select_inputs(c, items, pool, problem, 1))      # Verifier: wrong solutions
        assert all(items[i]["reward"] == 1 for i in so.select_inputs(c, items, pool, problem, 2))      # Corrector: right reports
        sel = so.select_inputs(base_cfg(strategy=so.RANDOM), items, pool, problem, 1)
        assert len(set(sel)) == 2
    only_pos = [0, 1, 3]
    sel = so.select_inputs(base_cfg(strategy=so.BALANCED), items, only_pos, 0, 1)
    assert len(set(sel)) == 2 and set(sel) <= set(only_pos)                      # one class empty: filled from the other
    sel = so.select_inputs(base_cfg(strategy=so.ADAPTIVE), items, only_pos, 0, 1)
    assert len(set(sel)) == 2
    assert so.select_inputs(base_cfg(), items, [4], 0, 2) == [4] and so.select_inputs(base_cfg(), items, [], 0, 2) == []
    # the random pick is uniform enough: every element of the pool is chosen for some problem
    seen = set()
    for problem in range(200):
        seen.update(so.select_inputs(base_cfg(strategy=so.RANDOM), items, pool, problem, 1))
    assert seen == set(pool)


def test_pipeline_and_segments_shorten_the_time_to_training():
    cfg = base_cfg(problems=24, capacity=0)
    pipe = so.simulate(cfg)
    traj = so.simulate(dict(cfg, pipeline=0))
    # same decode schedule either way; handing a group over when its agent is done can only be earlier
    assert [g["t_group"] for g in pipe["groups"]] == [g["t_group"] for g in traj["groups"]]
    assert all(a["t_train"] <= b["t_train"] for a, b in zip(pipe["groups"], traj["groups"]))
    assert pipe["sum_wait"] < 0.7 * traj["sum_wait"]
    # without segments a stage lasts as long as its longest sequence and everybody in it waits for that one
    whole = so.simulate(dict(cfg, segment=1 << 20))
    assert pipe["sum_wait"] / len(pipe["groups"]) < 0.8 * whole["sum_wait"] / len(whole["groups"])
    assert pipe["makespan"] <= whole["makespan"]


def test_decode_slots_are_a_hard_limit():
    # one problem, 8 Solver outputs of exactly L tokens, 3 decode slots, no segmentation: 3 + 3 + 2 -> back at 3 L
    L = 500
    cfg = base_cfg(problems=1, capacity=3, segment=1 << 20, short_lo=[L] * 5, short_hi=[L] * 5, long_hi=[L] * 5, p_long=[0] * 5,
                   p_correct=[ONE, 0, ONE, 0, ONE], p_flag_right=[0] * 5)
    r = so.simulate(cfg)
    assert r["groups"][0]["role"] == 0 and r["groups"][0]["t_group"] == 3 * L
    assert sorted(it["t_done"] for it in r["items"][:8]) == [L] * 3 + [2 * L] * 3 + [3 * L] * 2
    # the two Verifier groups (16 outputs) follow: 6 more stages of 3, 3, 3, 3, 3, 1
    assert r["makespan"] == 9 * L


def test_a_corrector_starts_from_the_solution_not_from_the_report():
    # every solution wrong, every error flagged: the Corrector repairs a WRONG solution, so p_correct applies, not p_keep
    cfg = base_cfg(problems=4, p_correct=[0, 0, ONE, 0, ONE], p_keep=[0] * 5, p_flag_wrong=[0, ONE, 0, ONE, 0], p_flag_right=[0] * 5)
    r = so.simulate(cfg)
    c1 = [it for it in r["items"] if it["role"] == 2]
    assert c1 and all(it["value"] == 1 and it["reward"] == 1 for it in c1)
    # ... and a RIGHT solution wrongly flagged is kept with p_keep, not repaired with p_correct
    cfg = base_cfg(problems=4, p_correct=[ONE, 0, 0, 0, 0], p_keep=[0, 0, ONE, 0, ONE], p_flag_wrong=[0, ONE, 0, ONE, 0],
                   p_flag_right=[0, ONE, 0, ONE, 0])
    r = so.simulate(cfg)
    c1 = [it for it in r["items"] if it["role"] == 2]
    assert c1 and all(it["value"] == 1 for it in c1)
