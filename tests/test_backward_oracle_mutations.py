"""The backward oracle's pins must be able to fail: each plausible mistake planted in a copy of its source (a dropped
term, a wrong sign, a missing factor, swapped operands) has to be caught by the central-difference pin.  CPU only; the
mistakes are planted in the oracle, never in the GPU path."""
import os
import types

import numpy as np
import pytest

from oracle import moe_backward_oracle as bwd

SRC = open(os.path.join(os.path.dirname(bwd.__file__), "moe_backward_oracle.py")).read()

MUTATIONS = [
    ("silu' without its second term", "dg = da * u * (s * (1.0 + g * (1.0 - s)))", "dg = da * u * s"),
    ("silu' sign", "dg = da * u * (s * (1.0 + g * (1.0 - s)))", "dg = da * u * (s * (1.0 - g * (1.0 - s)))"),
    ("du without the gate value", "du = da * (g * s)", "du = da * s"),
    ("dWd without the up factor", "dwd = dy.T @ a ", "dwd = dy.T @ (g * s) "),
    ("dv drops the up path", "dv = dg @ wg + du @ wu", "dv = dg @ wg"),
    ("dWg and dWu swapped", "dwg = dg.T @ v ", "dwg = du.T @ v "),
    ("softmax backward without the mean", "dl = w * (dw - (w * dw).sum(axis=1, keepdims=True))", "dl = w * dw"),
    ("softmax backward sign", "dl = w * (dw - (w * dw).sum(axis=1, keepdims=True))", "dl = w * (dw + (w * dw).sum(axis=1, keepdims=True))"),
    ("softmax backward without w", "dl = w * (dw - (w * dw).sum(axis=1, keepdims=True))", "dl = dw - (w * dw).sum(axis=1, keepdims=True)"),
    ("router path to x dropped", "dx = dlogits @ wr", "dx = 0.0 * (dlogits @ wr)"),
    ("routing weight dropped from dy", "dy = w[tt, kk][:, None] * d_out[tt]", "dy = d_out[tt]"),
    ("dw from the wrong tensor", 'dw = np.einsum("th,tkh->tk", d_out, y)', 'dw = np.einsum("th,tkh->tk", x, y)'),
    ("bias gradient averaged", "dbias = dlogits.sum(axis=0)", "dbias = dlogits.mean(axis=0)"),
    ("full softmax backward without the mean", "dlogits = p * (dw_dense - (w * dw).sum(axis=1, keepdims=True))", "dlogits = p * dw_dense"),
    ("da through the transposed projection", "da = dy @ wd ", "da = dy @ wd[:, ::-1] "),
]


def _tiny(seed, T=5, H=6, E=4, K=2, I=3):
    rng = np.random.default_rng(seed)
    p = {"x": rng.standard_normal((T, H)), "w_router": rng.standard_normal((E, H)) * 0.7, "bias": rng.standard_normal(E) * 0.3,
         "w_gate": rng.standard_normal((E, I, H)) * 0.7, "w_up": rng.standard_normal((E, I, H)) * 0.7,
         "w_down": rng.standard_normal((E, H, I)) * 0.7}
    logits = p["x"] @ p["w_router"].T + p["bias"]
    idx = np.argsort(-logits, axis=1, kind="stable")[:, :K].astype(np.int32)
    return p, idx, rng.standard_normal((T, H))


GRAD_OF = {"x": "d_x", "w_router": "d_w_router", "bias": "d_router_bias", "w_gate": "d_w_gate", "w_up": "d_w_up", "w_down": "d_w_down"}


def pins_hold(mod) -> bool:
    """The central-difference pin (against the UNMUTATED un-rounded forward), both weight modes, every input."""
    for renorm in (True, False):
        p, idx, d_out = _tiny(3)
        try:
            got = mod.backward(p["x"], p["w_router"], p["bias"], p["w_gate"], p["w_up"], p["w_down"], idx, d_out, renorm)
        except Exception:
            return False

        def loss(q):
            return float((bwd.forward64(q["x"], q["w_router"], q["bias"], q["w_gate"], q["w_up"], q["w_down"], idx, renorm)["out"] * d_out).sum())
        for name, gname in GRAD_OF.items():
            g = np.asarray(got[gname], dtype=np.float64).reshape(-1)
            if g.size != p[name].size:
                return False
            for pos in range(p[name].size):
                qp = {k: v.copy() for k, v in p.items()}
                qm = {k: v.copy() for k, v in p.items()}
                qp[name].reshape(-1)[pos] += 1e-6
                qm[name].reshape(-1)[pos] -= 1e-6
                fd = (loss(qp) - loss(qm)) / 2e-6
                if abs(fd - g[pos]) > 2e-6 * max(1.0, abs(g[pos])):
                    return False
    return True


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
