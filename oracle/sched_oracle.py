"""Discrete-event model of MarsRL's agentic rollout scheduling, plain Python.

TEST INFRASTRUCTURE ONLY: the reference the native simulator (paper_2511_11373_amd/csrc_host/mars_sched.cpp) is compared
with, bit for bit.  Shares no code with it.

What is modelled (all from the paper's text; numbers such as lengths and success rates are synthetic inputs):
  * the Verifier-Corrector pipeline unrolled over five roles, Solver, Verifier1, Corrector1, Verifier2, Corrector2
    (Section 3.1), at most five rollout iterations per problem;
  * agent-specific verifiable rewards (Section 3.2): a Solver/Corrector output is rewarded for being correct, a Verifier
    output for flagging exactly the incorrect solutions;
  * grouped agentic rollouts (Section 3.3): the Solver produces one group of G outputs per problem, every later agent picks
    n_select outputs of the preceding agent and produces a group of G for each; a Corrector only picks bug reports that
    flag an error, and the trajectory ends early when there is none;
  * the three sampling strategies (Section 3.4): Random, Balanced (one positive, one negative), Adaptive (Verifiers
    prefer reward-0 solutions, Correctors prefer reward-1 bug reports);
  * group-normalised advantages, Eq. 1 (population standard deviation, adv_eps added);
  * agentic pipeline parallelism and segment rollout (Sections 2.3, 3.3): decoding advances in stages of at most
    `segment` tokens; a sequence that finishes in a stage is handed back at the end of that stage, an unfinished one is
    carried into the next; a group becomes trainable when its last member is back (pipeline = 1) or only when its
    problem's whole trajectory has ended (pipeline = 0, the trajectory-level baseline).

Readings where the paper is silent: the pool a later agent samples from is all outputs of the preceding agent for the
problem (both groups); fewer candidates than n_select means fewer groups; Balanced fills from the other class when one is
empty; a stage lasts as long as its longest decode (at most `segment`); sequences wait first-in first-out for one of
`capacity` decode slots (0 = unlimited); every problem's Solver group is submitted at time 0.

Random numbers: every draw is SplitMix64 (Steele, Lea, Flood 2014: add 0x9E3779B97F4A7C15, two xor-shift-multiply rounds
with 0xBF58476D1CE4E5B9 and 0x94D049BB133111EB, final xor-shift by 31) of a key made from (seed, problem, role, group,
member, purpose), so that a draw does not depend on the order of events.  Probabilities are integers in units of 2^-24.
"""
from __future__ import annotations

import math
from typing import Dict, List

MASK = (1 << 64) - 1
ROLES = ("solver", "verifier1", "corrector1", "verifier2", "corrector2")
RANDOM, BALANCED, ADAPTIVE = 0, 1, 2
# purposes of a draw
P_LEN_CLASS, P_LEN, P_OUTCOME, P_PICK = 0, 1, 2, 3


def splitmix64(z: int) -> int:
    z = (z + 0x9E3779B97F4A7C15) & MASK
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK
    return z ^ (z >> 31)


def draw(seed: int, problem: int, role: int, group: int, member: int, purpose: int) -> int:
    key = ((((problem * 8 + role) * 4 + group) * 64 + member) * 8 + purpose) & MASK
    return splitmix64(splitmix64(seed & MASK) ^ key)


def bernoulli(u: int, p24: int) -> bool:
    return (u >> 40) < p24


def is_verifier(role: int) -> bool:
    return role in (1, 3)


def pick_distinct(cands: List[int], m: int, seed: int, problem: int, role: int, tag: int) -> List[int]:
    """m distinct elements of cands (all of them if fewer): partial Fisher-Yates, draw j of the pick keyed by member=tag*8+j."""
    pool = list(cands)
    out = []
    for j in range(min(m, len(pool))):
        u = draw(seed, problem, role, 3, tag * 8 + j, P_PICK)
        i = j + (u >> 11) % (len(pool) - j)
        pool[j], pool[i] = pool[i], pool[j]
        out.append(pool[j])
    return out


def select_inputs(cfg: Dict, items: List[Dict], cands: List[int], problem: int, role: int) -> List[int]:
    """The outputs of the preceding agent that `role` works on (indices into items), at most n_select."""
    n = cfg["n_select"]
    strat = cfg["strategy"]
    seed = cfg["seed"]
    pos = [i for i in cands if items[i]["reward"] == 1]
    neg = [i for i in cands if items[i]["reward"] == 0]
    if strat == RANDOM:
        return pick_distinct(cands, n, seed, problem, role, 0)
    if strat == BALANCED:
        half = n // 2
        a = pick_distinct(pos, half, seed, problem, role, 1)
        b = pick_distinct(neg, n - half, seed, problem, role, 2)
        rest = [i for i in cands if i not in a and i not in b]
        return a + b + pick_distinct(rest, n - len(a) - len(b), seed, problem, role, 3)
    # adaptive: Verifiers want incorrect solutions (reward 0), Correctors want correct bug reports (reward 1)
    first, second = (neg, pos) if is_verifier(role) else (pos, neg)
    a = pick_distinct(first, n, seed, problem, role, 1)
    return a + pick_distinct(second, n - len(a), seed, problem, role, 2)


def advantages(rewards: List[int], adv_eps: float) -> List[float]:
    """Eq. 1 on 0/1 rewards: mean k/G, population variance k (G - k) / G^2."""
    G = len(rewards)
    k = sum(rewards)
    mean = k / G
    std = math.sqrt((k * (G - k)) / (G * G))
    return [(r - mean) / (std + adv_eps) for r in rewards]


def simulate(cfg: Dict) -> Dict:
    """cfg keys: problems, group_size, n_select, segment, capacity, strategy, pipeline, seed, adv_eps, and per-role lists of
    five: short_lo, short_hi, long_hi (token ranges), p_long, and the 2^-24 probabilities p_correct (Solver/Correctors when
    the solution they start from is wrong or absent), p_keep (Correctors when it was right), p_flag_wrong (Verifiers: recall),
    p_flag_right (Verifiers: false alarms)."""
    P, G = cfg["problems"], cfg["group_size"]
    seed = cfg["seed"]
    items: List[Dict] = []
    groups: List[Dict] = []
    pending: List[int] = []          # item indices waiting for a decode slot, first in first out
    active: List[int] = []
    # per (problem, role): group ids still running
    open_groups = {}
    end_time = [None] * P            # when the problem's trajectory ended
    early_stop = [0] * 5

    def submit(problem: int, role: int, parents: List[int], now: int):
        gids = []
        for gi, parent in enumerate(parents):
            gid = len(groups)
            groups.append({"problem": problem, "role": role, "group": gi, "parent": parent, "members": [], "left": G,
                           "t_submit": now, "t_group": -1, "t_train": -1, "adv": None})
            for m in range(G):
                u = draw(seed, problem, role, gi, m, P_LEN_CLASS)
                v = draw(seed, problem, role, gi, m, P_LEN)
                if bernoulli(u, cfg["p_long"][role]):
                    lo, hi = cfg["short_hi"][role], cfg["long_hi"][role]
                else:
                    lo, hi = cfg["short_lo"][role], cfg["short_hi"][role]
                length = lo + (v >> 11) % (hi - lo + 1)
                w = draw(seed, problem, role, gi, m, P_OUTCOME)
                if is_verifier(role):
                    wrong = items[parent]["value"] == 0
                    value = int(bernoulli(w, cfg["p_flag_wrong"][role] if wrong else cfg["p_flag_right"][role]))   # 1 = flags an error
                    reward = int(value == int(wrong))
                else:
                    base_right = role != 0 and items[items[parent]["parent"]]["value"] == 1     # the solution under correction
                    value = int(bernoulli(w, cfg["p_keep"][role] if base_right else cfg["p_correct"][role]))   # 1 = correct
                    reward = value
                items.append({"problem": problem, "role": role, "group": gid, "member": m, "parent": parent, "length": length,
                              "left": length, "value": value, "reward": reward, "t_done": -1})
                groups[gid]["members"].append(len(items) - 1)
                pending.append(len(items) - 1)
            gids.append(gid)
        open_groups[(problem, role)] = set(gids)

    for p in range(P):
        submit(p, 0, [-1], 0)
    now = 0
    tokens = 0
    cap = cfg["capacity"]
    while pending or active:
        while pending and (cap == 0 or len(active) < cap):
            active.append(pending.pop(0))
        step = max(min(cfg["segment"], items[i]["left"]) for i in active)
        now += step
        still = []
        finished_groups = []
        for i in active:
            it = items[i]
            d = min(cfg["segment"], it["left"])
            it["left"] -= d
            tokens += d
            if it["left"] == 0:
                it["t_done"] = now
                g = groups[it["group"]]
                g["left"] -= 1
                if g["left"] == 0:
                    finished_groups.append(it["group"])
            else:
                still.append(i)
        active = still
        for gid in sorted(finished_groups):
            g = groups[gid]
            g["t_group"] = now
            g["adv"] = advantages([items[i]["reward"] for i in g["members"]], cfg["adv_eps"])
            key = (g["problem"], g["role"])
            open_groups[key].discard(gid)
            if open_groups[key]:
                continue
            # the agent is done for this problem: the next one picks its inputs
            problem, role = key
            if role == 4:
                end_time[problem] = now
                continue
            cands = [i for gg in groups if gg["problem"] == problem and gg["role"] == role for i in gg["members"]]
            if not is_verifier(role + 1):
                cands = [i for i in cands if items[i]["value"] == 1]        # Correctors only take reports that flag an error
            chosen = select_inputs(cfg, items, cands, problem, role + 1)
            if not chosen:
                end_time[problem] = now
                early_stop[role + 1] += 1
                continue
            submit(problem, role + 1, chosen, now)
    for g in groups:
        g["t_train"] = g["t_group"] if cfg["pipeline"] else end_time[g["problem"]]
    return {"items": items, "groups": groups, "makespan": now, "tokens": tokens, "early_stop": early_stop,
            "end_time": end_time, "sum_t_train": sum(g["t_train"] for g in groups),
            "sum_wait": sum(g["t_train"] - g["t_submit"] for g in groups)}
