"""CPU oracle of the token log-probability and GRPO objective step (Section 2.2, Eq. 1-3).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the benchmark's CPU-baseline leg, never by the
GPU library or its binding, with which it shares nothing.  Plain numpy in float64, one formula per line, no
blocking or fusion.

Readings where the paper is silent (it cites GRPO and prints Eq. 1-3 only):
  * std in Eq. 1 is the population standard deviation, and adv_eps is added to it (equal rewards give zero
    advantages instead of 0/0);
  * D_KL(pi_theta || pi_ref) in Eq. 2 is GRPO's per-token estimator exp(d) - d - 1 with
    d = log pi_ref(o_t) - log pi_theta(o_t);
  * a response without tokens contributes 0 to the mean over responses.

Pins (tests/test_grpo_oracle_pins.py): scipy logsumexp and torch log_softmax; uniform logits give -log V; shift
invariance; advantages have zero mean and unit population variance; hand-worked clip / KL cases
(tests/golden/grpo_example.txt); ratio 1 and equal policies reduce the objective to the mean advantage.
"""
from __future__ import annotations

import numpy as np


def token_logprob(logits, target):
    """log pi(o_t) = logit[o_t] - log sum_v exp(logit[v]), row by row."""
    x = np.asarray(logits, dtype=np.float64)
    t = np.asarray(target, dtype=np.int64)
    m = x.max(axis=1)
    lse = m + np.log(np.exp(x - m[:, None]).sum(axis=1))
    return x[np.arange(x.shape[0]), t] - lse


def group_advantage(rewards, adv_eps):
    """Eq. 1 with the population standard deviation."""
    r = np.asarray(rewards, dtype=np.float64)
    return (r - r.mean()) / (r.std() + adv_eps)


def objective(logp, logp_old, logp_ref, rewards, resp_offsets, clip_eps, beta, adv_eps):
    """Returns (advantage [G], token_term [N], resp_mean [G], J)."""
    logp = np.asarray(logp, dtype=np.float64)
    old = np.asarray(logp_old, dtype=np.float64)
    ref = np.asarray(logp_ref, dtype=np.float64)
    off = np.asarray(resp_offsets, dtype=np.int64)
    G = off.shape[0] - 1
    adv = group_advantage(rewards, adv_eps) if G > 0 else np.zeros(0)
    term = np.zeros_like(logp)
    mean = np.zeros(G)
    for i in range(G):
        sl = slice(off[i], off[i + 1])
        ratio = np.exp(logp[sl] - old[sl])                                   # Eq. 3
        clipped = np.clip(ratio, 1.0 - clip_eps, 1.0 + clip_eps)
        d = ref[sl] - logp[sl]
        kl = np.exp(d) - d - 1.0
        term[sl] = np.minimum(ratio * adv[i], clipped * adv[i]) - beta * kl  # Eq. 2, inner bracket
        if off[i + 1] > off[i]:
            mean[i] = term[sl].mean()
    J = mean.mean() if G > 0 else 0.0
    return adv, term, mean, float(J)


def logprob_objective(logits, target, logp_old, logp_ref, rewards, resp_offsets, clip_eps, beta, adv_eps):
    logp = token_logprob(logits, target)
    return (logp,) + objective(logp, logp_old, logp_ref, rewards, resp_offsets, clip_eps, beta, adv_eps)
