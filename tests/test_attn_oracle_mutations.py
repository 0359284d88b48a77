"""The decode-attention oracle's pins must be able to fail: each plausible mistake planted in a copy of its source has to
be caught by a compact set of them (torch's scaled-dot-product attention on one sequence, the mean of the values for
zero queries, the head mapping).  CPU only; the mistakes are planted in the oracle, never in the GPU path."""
import os
import types

import numpy as np
import pytest
import torch

from oracle import attn_oracle as ao

SRC = open(os.path.join(os.path.dirname(ao.__file__), "attn_oracle.py")).read()

MUTATIONS = [
    ("no 1/sqrt(D)", "@ q[b, j] / np.sqrt(D)", "@ q[b, j]"),
    ("scaled by 1/D", "@ q[b, j] / np.sqrt(D)", "@ q[b, j] / D"),
    ("the last valid position dropped", "k[b, :n, h, :] @", "k[b, :max(n - 1, 1), h, :] @"),
    ("positions past the length included", "k[b, :n, h, :] @ q[b, j] / np.sqrt(D)\n            p = np.exp(s - s.max())\n            p /= p.sum()\n            out[b, j] = p @ v[b, :n, h, :]",
     "k[b, :, h, :] @ q[b, j] / np.sqrt(D)\n            p = np.exp(s - s.max())\n            p /= p.sum()\n            out[b, j] = p @ v[b, :, h, :]"),
    ("query heads interleaved over the key/value heads", "h = j // group", "h = j % Hkv"),
    ("every query head reads key/value head 0", "h = j // group", "h = 0"),
    ("softmax not normalised", "            p /= p.sum()\n", ""),
    ("normalised by the largest weight", "p /= p.sum()", "p /= p.max()"),
    ("exponent sign", "p = np.exp(s - s.max())", "p = np.exp(s.max() - s)"),
    ("values of the wrong head", "out[b, j] = p @ v[b, :n, h, :]", "out[b, j] = p @ v[b, :n, (h + 1) % Hkv, :]"),
    ("keys used as values", "out[b, j] = p @ v[b, :n, h, :]", "out[b, j] = p @ k[b, :n, h, :]"),
    ("another sequence's query", "@ q[b, j] / np.sqrt(D)", "@ q[(b + 1) % B, j] / np.sqrt(D)"),
]


def pins_hold(mod) -> bool:
    try:
        rng = np.random.default_rng(0)
        B, Hq, Hkv, D, L = 3, 8, 2, 16, 40
        q = rng.standard_normal((B, Hq, D))
        k = rng.standard_normal((B, L, Hkv, D))
        v = rng.standard_normal((B, L, Hkv, D))
        lens = np.array([40, 17, 1])
        got = mod.decode_attention(q, k, v, lens)
        group = Hq // Hkv
        for b in range(B):
            n = int(lens[b])
            tq = torch.tensor(q[b])[:, None, :]
            tk = torch.tensor(k[b, :n]).permute(1, 0, 2).repeat_interleave(group, dim=0)
            tv = torch.tensor(v[b, :n]).permute(1, 0, 2).repeat_interleave(group, dim=0)
            ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[:, 0, :].numpy()
            if not np.allclose(got[b], ref, rtol=1e-12, atol=1e-12):
                return False
        zero = mod.decode_attention(np.zeros_like(q), k, v, lens)             # equal scores: the mean of the values
        for b in range(B):
            for j in range(Hq):
                if not np.allclose(zero[b, j], v[b, :lens[b], j // group].mean(axis=0), atol=1e-13):
                    return False
        return True
    except Exception:
        return False


def test_the_unmodified_oracle_passes():
    assert pins_hold(ao)


@pytest.mark.parametrize("what,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(what, old, new):
    assert SRC.count(old) == 1, f"pattern for '{what}' must match the oracle source exactly once"
    mod = types.ModuleType("attn_oracle_mutant")
    exec(compile(SRC.replace(old, new), "attn_oracle_mutant", "exec"), mod.__dict__)
    assert not pins_hold(mod), f"the pins did not notice: {what}"
