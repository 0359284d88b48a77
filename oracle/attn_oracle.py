"""Single-token (decode) grouped-query attention over a long context, plain numpy float64.

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and bench.py's cpu_baseline leg, never by the product
path, with which it shares no code.

The policy the paper trains (Section 4.1: a Qwen3-30B-A3B-class model, 32k-token inputs and 64k-token outputs) generates
every token with one pass of causal attention of the new token's queries over everything before it.  The paper does not
spell the operation out; what is computed is the textbook definition:

    for sequence b, query head j (its key/value head is j // (Hq / Hkv)), context length n_b:
        s[t]  = <q[b, j, :], k[b, t, h, :]> / sqrt(D)        t = 0 .. n_b - 1
        p     = softmax(s)
        out[b, j, :] = sum_t p[t] * v[b, t, h, :]

written out exactly like that: no blocking, no running maximum, no splitting of the context.
"""
from __future__ import annotations

import numpy as np


def decode_attention(q, k, v, seq_lens):
    """q [B, Hq, D]; k, v [B, L, Hkv, D] (positions >= seq_lens[b] are ignored); returns out [B, Hq, D] float64.
    A sequence of length 0 gives zeros."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    B, Hq, D = q.shape
    Hkv = k.shape[2]
    group = Hq // Hkv
    out = np.zeros((B, Hq, D))
    for b in range(B):
        n = int(seq_lens[b])
        if n == 0:
            continue
        for j in range(Hq):
            h = j // group
            s = k[b, :n, h, :] @ q[b, j] / np.sqrt(D)
            p = np.exp(s - s.max())
            p /= p.sum()
            out[b, j] = p @ v[b, :n, h, :]
    return out
