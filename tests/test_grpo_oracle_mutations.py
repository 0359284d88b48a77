"""The GRPO oracle's pins must be able to fail: each plausible mistake planted in a copy of its source has to be caught
by a compact set of them (the hand-worked example of Eq. 1-3, scipy's logsumexp, the Bernoulli closed form of Eq. 1).
CPU only; the mistakes are planted in the oracle, never in the GPU path."""
import math
import os
import types

import numpy as np
import pytest
import scipy.special

from oracle import grpo_oracle as go

SRC = open(os.path.join(os.path.dirname(go.__file__), "grpo_oracle.py")).read()
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "grpo_example.txt")

MUTATIONS = [
    ("log-sum-exp without the maximum added back", "lse = m + np.log(", "lse = np.log("),
    ("log-prob sign", "return x[np.arange(x.shape[0]), t] - lse", "return lse - x[np.arange(x.shape[0]), t]"),
    ("sum over the wrong axis", "np.exp(x - m[:, None]).sum(axis=1))", "np.exp(x - m[:, None]).sum(axis=0)[:1].repeat(x.shape[0]))"),
    ("sample standard deviation", "(r.std() + adv_eps)", "(r.std(ddof=1) + adv_eps)"),
    ("advantage not centred", "return (r - r.mean()) /", "return r /"),
    ("ratio inverted", "ratio = np.exp(logp[sl] - old[sl])", "ratio = np.exp(old[sl] - logp[sl])"),
    ("clip range one-sided", "clipped = np.clip(ratio, 1.0 - clip_eps, 1.0 + clip_eps)", "clipped = np.clip(ratio, 0.0, 1.0 + clip_eps)"),
    ("max instead of min", "np.minimum(ratio * adv[i], clipped * adv[i])", "np.maximum(ratio * adv[i], clipped * adv[i])"),
    ("clipping applied after the advantage's sign is lost", "np.minimum(ratio * adv[i], clipped * adv[i])", "np.minimum(ratio, clipped) * adv[i]"),
    ("KL direction", "d = ref[sl] - logp[sl]", "d = logp[sl] - ref[sl]"),
    ("KL estimator without the linear term", "kl = np.exp(d) - d - 1.0", "kl = np.exp(d) - 1.0"),
    ("KL added instead of subtracted", "- beta * kl", "+ beta * kl"),
    ("token mean over all tokens instead of per response", "J = mean.mean() if G > 0 else 0.0", "J = term.mean() if G > 0 else 0.0"),
]


def pins_hold(mod) -> bool:
    try:
        # scipy's logsumexp, and -log V for uniform rows
        rng = np.random.default_rng(0)
        x = rng.standard_normal((7, 33)) * 3 + 50.0
        t = rng.integers(0, 33, 7)
        lp = mod.token_logprob(x, t)
        if not np.allclose(lp, x[np.arange(7), t] - scipy.special.logsumexp(x, axis=1), rtol=0, atol=1e-12):
            return False
        if not np.allclose(mod.token_logprob(np.zeros((3, 10)), [0, 4, 9]), -math.log(10.0)):
            return False
        # Eq. 1 on 0/1 rewards with k ones of G: (1 - p) / sqrt(p (1 - p)) for the ones
        adv = mod.group_advantage([1, 0, 0, 1, 0, 0, 0, 0], 0.0)
        p = 0.25
        if not np.allclose(adv[0], (1 - p) / math.sqrt(p * (1 - p))) or abs(adv.sum()) > 1e-12:
            return False
        # the hand-worked example
        want = {}
        for line in open(GOLDEN):
            if line.startswith("#") or not line.strip():
                continue
            k, *v = line.split()
            want[k] = np.array([float(z) for z in v])
        ln2 = math.log(2.0)
        logp = np.array([-1.0, -2.0, -1.0, -2.0, -3.0])
        old = logp - np.log([1.5, 0.5, 1.5, 0.5, 1.0])
        ref = logp + np.array([0.0, ln2, 0.0, -ln2, 0.0])
        a, term, mean, J = mod.objective(logp, old, ref, [1.0, 0.0], [0, 2, 5], 0.2, 0.5, 0.0)
        return (np.allclose(a, want["advantage"], atol=1e-9) and np.allclose(term, want["term"], atol=1e-9) and
                np.allclose(mean, want["mean"], atol=1e-9) and abs(J - want["objective"][0]) < 1e-9)
    except Exception:
        return False


def _load(src):
    mod = types.ModuleType("mutant")
    exec(compile(src, "mutant", "exec"), mod.__dict__)
    return mod


def test_the_unmutated_oracle_passes():
    assert pins_hold(_load(SRC))


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(name, old, new):
    assert SRC.count(old) >= 1, "the mutation's anchor is gone from the oracle source"
    assert not pins_hold(_load(SRC.replace(old, new))), name
