"""Pins of the GRPO oracle (CPU only): library routines, closed forms, invariants, a hand-worked example."""
import math
import os

import numpy as np
import scipy.special
import torch

from oracle import grpo_oracle as go

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "grpo_example.txt")


def test_logprob_is_the_library_log_softmax():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((7, 1000)) * 3.0
    x[2, 17] = 40.0                                         # one dominant entry
    t = rng.integers(0, 1000, 7)
    t[2] = 17
    got = go.token_logprob(x, t)
    ref = x[np.arange(7), t] - scipy.special.logsumexp(x, axis=1)
    np.testing.assert_allclose(got, ref, rtol=1e-13, atol=1e-13)
    ref2 = torch.log_softmax(torch.from_numpy(x), dim=1).numpy()[np.arange(7), t]
    np.testing.assert_allclose(got, ref2, rtol=1e-12, atol=1e-12)
    assert abs(got[2]) < 1e-12 and np.all(got <= 0)


def test_logprob_closed_forms_and_shift_invariance():
    V = 4096
    x = np.full((3, V), 1.75)
    np.testing.assert_allclose(go.token_logprob(x, [0, 5, V - 1]), -math.log(V), rtol=1e-14)
    rng = np.random.default_rng(1)
    y = rng.standard_normal((4, 64))
    t = [3, 0, 63, 10]
    np.testing.assert_allclose(go.token_logprob(y + np.array([[100.0], [-50.0], [0.5], [7.0]]), t), go.token_logprob(y, t),
                               rtol=1e-12, atol=1e-12)
    # two-entry row: log sigmoid
    z = np.array([[2.0, -1.0]])
    np.testing.assert_allclose(go.token_logprob(z, [0]), -math.log1p(math.exp(-3.0)), rtol=1e-14)
    # huge magnitudes must not overflow
    big = np.array([[1e4, 1e4 - 1.0, -1e4]])
    np.testing.assert_allclose(go.token_logprob(big, [1]), -1.0 - math.log1p(math.exp(-1.0)), rtol=1e-12)


def test_advantage_normalisation():
    r = np.array([1.0, 0.0, 0.0, 1.0, 1.0, 0.0, 1.0, 1.0])
    a = go.group_advantage(r, 0.0)
    assert abs(a.mean()) < 1e-15 and abs(a.std() - 1.0) < 1e-15
    assert np.all(np.sign(a) == np.sign(r - 0.5))
    np.testing.assert_allclose(a, (r - 0.625) / math.sqrt(0.625 * 0.375), rtol=1e-14)      # Bernoulli closed form
    assert np.all(go.group_advantage(np.ones(5), 1e-6) == 0.0)                             # equal rewards: 0, not 0/0


def test_hand_worked_example():
    vals = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        vals[k] = np.array([float(t) for t in v])
    ln2 = math.log(2.0)
    logp = np.array([-1.0, -2.0, -0.5, -3.0, -1.5])
    old = logp - np.array([math.log(1.5), -ln2, math.log(1.5), -ln2, 0.0])
    ref = logp + np.array([0.0, ln2, 0.0, -ln2, 0.0])
    adv, term, mean, J = go.objective(logp, old, ref, [1.0, 0.0], [0, 2, 5], 0.2, 0.5, 0.0)
    np.testing.assert_allclose(adv, vals["advantage"], rtol=1e-14)
    np.testing.assert_allclose(term, vals["term"], atol=2e-10)
    np.testing.assert_allclose(mean, vals["mean"], atol=2e-10)
    assert abs(J - vals["objective"][0]) < 2e-10
    # the same from closed forms, to full precision
    np.testing.assert_allclose(term, [1.2, 0.5 - 0.5 * (1.0 - ln2), -1.5, -0.8 - 0.5 * (ln2 - 0.5), -1.0], rtol=1e-13)


def test_objective_special_cases():
    rng = np.random.default_rng(2)
    N, G = 40, 4
    off = np.array([0, 7, 7, 25, 40])                       # response 1 has no tokens
    logp = -rng.random(N) * 3
    r = np.array([1.0, 0.0, 0.5, 0.25])
    # identical policies: ratio 1, kl 0 => every token term is its response's advantage
    adv, term, mean, J = go.objective(logp, logp, logp, r, off, 0.2, 0.3, 1e-6)
    for i in range(G):
        assert np.all(term[off[i]:off[i + 1]] == adv[i])
    assert mean[1] == 0.0 and abs(J - (adv[0] + adv[2] + adv[3]) / 4.0) < 1e-15
    # beta = 0 and a huge clip range: the plain importance-weighted objective
    old = logp + rng.standard_normal(N) * 0.1
    adv, term, mean, J = go.objective(logp, old, logp + 1.0, r, off, 1e9, 0.0, 1e-6)
    np.testing.assert_allclose(term, np.exp(logp - old) * np.repeat(adv, np.diff(off)), rtol=1e-13)
    # the KL estimator is non-negative and the clipped surrogate never exceeds the unclipped one
    adv, term, mean, J = go.objective(logp, old, logp + rng.standard_normal(N), r, off, 0.2, 1.0, 1e-6)
    _, term0, _, _ = go.objective(logp, old, logp, r, off, 0.2, 1.0, 1e-6)
    assert np.all(term <= term0 + 1e-15)
    assert np.all(term0 <= np.exp(logp - old) * np.repeat(adv, np.diff(off)) + 1e-15)
    # empty group
    assert go.objective(np.zeros(0), np.zeros(0), np.zeros(0), np.zeros(0), [0], 0.2, 0.1, 1e-6)[3] == 0.0
