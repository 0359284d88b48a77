"""Dense brute force of the MoE FFN block, for tiny shapes only.

TEST INFRASTRUCTURE ONLY.  A second definition, independent of moe_oracle.c:
no grouping, no permutation, every expert is applied to every token and the
result is masked by a dense gate matrix.  Logits in extended precision,
selection by a full sort of (-logit, index) pairs.  It exists to catch a
mistake in the oracle's grouping / permutation / indexing logic.
"""
from __future__ import annotations

import numpy as np


def dense_gates(x, w_router, K, bias=None, renormalize=True):
    """G [T,E] float64 with the routing weight where an expert is selected, else 0;
    also returns the ordered selection [T,K]."""
    xl = np.asarray(x, dtype=np.longdouble)
    wl = np.asarray(w_router, dtype=np.longdouble)
    T, E = xl.shape[0], wl.shape[0]
    G = np.zeros((T, E), dtype=np.float64)
    sel = np.zeros((T, K), dtype=np.int32)
    for t in range(T):
        logit = []
        for e in range(E):
            s = np.longdouble(0)
            for h in range(xl.shape[1]):
                s += xl[t, h] * wl[e, h]
            if bias is not None:
                s += np.longdouble(bias[e])
            logit.append(float(np.float32(s)))      # the contract's single rounding to float
        order = sorted(range(E), key=lambda e: (-logit[e], e))
        chosen = order[:K]
        full = np.exp(np.array(logit, dtype=np.float64) - max(logit))
        full /= full.sum()                           # the full softmax ...
        denom = full[chosen].sum() if renormalize else 1.0
        for k, e in enumerate(chosen):               # ... renormalised over the selected K
            G[t, e] = full[e] / denom
            sel[t, k] = e
    return G, sel


def dense_forward(x, w_router, w_gate, w_up, w_down, K, bias=None, renormalize=True):
    x64 = np.asarray(x, dtype=np.float64)
    G, sel = dense_gates(x, w_router, K, bias, renormalize)
    T, H = x64.shape
    E = w_gate.shape[0]
    out = np.zeros((T, H), dtype=np.float64)
    for e in range(E):
        g = x64 @ np.asarray(w_gate[e], dtype=np.float64).T
        u = x64 @ np.asarray(w_up[e], dtype=np.float64).T
        act = g * (1.0 / (1.0 + np.exp(-g))) * u
        y = act @ np.asarray(w_down[e], dtype=np.float64).T
        out += G[:, e:e + 1] * y
    return out, sel, G
