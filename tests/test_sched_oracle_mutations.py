"""The scheduling oracle's pins must be able to fail: each plausible mistake planted in a copy of its source has to make
at least one of the pins in test_sched_oracle_pins.py fail.  CPU only; the mistakes are planted in the oracle, never in
the native simulator."""
import os
import types

import pytest

from oracle import sched_oracle as so
import test_sched_oracle_pins as pins

SRC = open(os.path.join(os.path.dirname(so.__file__), "sched_oracle.py")).read()
PIN_FUNCS = [getattr(pins, name) for name in sorted(dir(pins)) if name.startswith("test_")]

MUTATIONS = [
    ("SplitMix64 multiplier", "0xBF58476D1CE4E5B9) & MASK", "0xBF58476D1CE4E5B8) & MASK"),
    ("SplitMix64 final shift", "return z ^ (z >> 31)", "return z ^ (z >> 30)"),
    ("Bernoulli test inverted", "return (u >> 40) < p24", "return (u >> 40) >= p24"),
    ("sample standard deviation in Eq. 1", "std = math.sqrt((k * (G - k)) / (G * G))", "std = math.sqrt((k * (G - k)) / (G * (G - 1)))"),
    ("advantage not centred", "mean = k / G", "mean = 0.0"),
    ("Verifier rewarded for raising a flag", "reward = int(value == int(wrong))", "reward = value"),
    ("Correctors take the reports that raise no flag", 'cands = [i for i in cands if items[i]["value"] == 1]', 'cands = [i for i in cands if items[i]["value"] == 0]'),
    ("the pipeline ends one agent early", "if role == 4:", "if role == 3:"),
    ("pipeline and trajectory-level hand-over swapped", 'g["t_group"] if cfg["pipeline"] else end_time[g["problem"]]', 'end_time[g["problem"]] if cfg["pipeline"] else g["t_group"]'),
    ("a stage lasts as long as its shortest decode", 'step = max(min(cfg["segment"], items[i]["left"]) for i in active)', 'step = min(min(cfg["segment"], items[i]["left"]) for i in active)'),
    ("one decode slot too many", "len(active) < cap", "len(active) <= cap"),
    ("Adaptive preferences swapped", "first, second = (neg, pos) if is_verifier(role) else (pos, neg)", "first, second = (pos, neg) if is_verifier(role) else (neg, pos)"),
    ("Balanced takes positives only", "half = n // 2", "half = n"),
    ("the pick does not shuffle", "        pool[j], pool[i] = pool[i], pool[j]\n", ""),
    ("a Corrector keeps what its Verifier said, not what the solution was", 'base_right = role != 0 and items[items[parent]["parent"]]["value"] == 1', 'base_right = role != 0 and items[parent]["value"] == 1'),
    ("a group is handed back with its first member", 'if g["left"] == 0:', 'if g["left"] == G - 1:'),
    ("the long class drawn from the short range", 'lo, hi = cfg["short_hi"][role], cfg["long_hi"][role]', 'lo, hi = cfg["short_lo"][role], cfg["short_hi"][role]'),
    ("every later agent produces one group only", "chosen = select_inputs(cfg, items, cands, problem, role + 1)", "chosen = select_inputs(cfg, items, cands, problem, role + 1)[:1]"),
]


def caught(mod) -> bool:
    """True if some pin fails with `mod` in the oracle's place."""
    keep = pins.so
    pins.so = mod
    try:
        for f in PIN_FUNCS:
            try:
                f()
            except Exception:
                return True
        return False
    finally:
        pins.so = keep


def test_the_unmodified_oracle_passes():
    assert not caught(so)


@pytest.mark.parametrize("what,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(what, old, new):
    assert SRC.count(old) == 1, f"pattern for '{what}' must match the oracle source exactly once"
    mod = types.ModuleType("sched_oracle_mutant")
    exec(compile(SRC.replace(old, new), "sched_oracle_mutant", "exec"), mod.__dict__)
    assert caught(mod), f"the pins did not notice: {what}"
