"""Pins of the backward oracle to things other than itself (CPU only).

The paper prints no numbers for the layer's gradient (Section 2.2 only states the
objective that is differentiated), so the oracle is pinned by: central differences
of the un-rounded forward, reverse-mode differentiation by a library (torch autograd
over plain torch ops written independently here), closed forms of the SiLU
derivative, and invariants of the softmax (logit gradients of a token sum to zero,
a single selected expert carries no router gradient, linearity in d_out).
"""
import math

import numpy as np
import pytest
import torch

from oracle import moe_backward_oracle as bwd
from paper_2511_11373_amd import workloads as wl


def _tiny(seed, T=5, H=6, E=4, K=2, I=3, scale=0.7):
    rng = np.random.default_rng(seed)
    p = {
        "x": rng.standard_normal((T, H)),
        "w_router": rng.standard_normal((E, H)) * scale,
        "bias": rng.standard_normal(E) * 0.3,
        "w_gate": rng.standard_normal((E, I, H)) * scale,
        "w_up": rng.standard_normal((E, I, H)) * scale,
        "w_down": rng.standard_normal((E, H, I)) * scale,
    }
    logits = p["x"] @ p["w_router"].T + p["bias"]
    idx = np.argsort(-logits, axis=1, kind="stable")[:, :K].astype(np.int32)
    d_out = rng.standard_normal((T, H))
    return p, idx, d_out


def _loss(p, idx, d_out, renorm):
    f = bwd.forward64(p["x"], p["w_router"], p["bias"], p["w_gate"], p["w_up"], p["w_down"], idx, renorm)
    return float((f["out"] * d_out).sum())


GRAD_OF = {"x": "d_x", "w_router": "d_w_router", "bias": "d_router_bias", "w_gate": "d_w_gate",
           "w_up": "d_w_up", "w_down": "d_w_down"}


@pytest.mark.parametrize("renorm", [True, False])
@pytest.mark.parametrize("seed", [1, 2])
def test_backward_matches_central_differences(seed, renorm):
    p, idx, d_out = _tiny(seed)
    got = bwd.backward(p["x"], p["w_router"], p["bias"], p["w_gate"], p["w_up"], p["w_down"], idx, d_out, renorm)
    eps = 1e-6
    rng = np.random.default_rng(100 + seed)
    for name, gname in GRAD_OF.items():
        flat_n = p[name].size
        for pos in rng.choice(flat_n, size=min(flat_n, 12), replace=False):
            q_plus = {k: v.copy() for k, v in p.items()}
            q_minus = {k: v.copy() for k, v in p.items()}
            q_plus[name].reshape(-1)[pos] += eps
            q_minus[name].reshape(-1)[pos] -= eps
            fd = (_loss(q_plus, idx, d_out, renorm) - _loss(q_minus, idx, d_out, renorm)) / (2 * eps)
            an = got[gname].reshape(-1)[pos]
            assert abs(fd - an) <= 2e-6 * max(1.0, abs(an)), (name, pos, fd, an)


def _torch_block(p, idx, renorm):
    """The block in plain torch ops (float64), written from the definition, for autograd."""
    x, wr, b = p["x"], p["w_router"], p["bias"]
    logits = x @ wr.T + b
    sel = torch.as_tensor(idx.astype(np.int64))
    if renorm:
        w = torch.softmax(torch.gather(logits, 1, sel), dim=1)
    else:
        w = torch.gather(torch.softmax(logits, dim=1), 1, sel)
    out = torch.zeros_like(x)
    T, K = idx.shape
    for t in range(T):
        for k in range(K):
            e = int(idx[t, k])
            a = torch.nn.functional.silu(p["w_gate"][e] @ x[t]) * (p["w_up"][e] @ x[t])
            out[t] = out[t] + w[t, k] * (p["w_down"][e] @ a)
    return out


@pytest.mark.parametrize("renorm", [True, False])
def test_backward_matches_library_autograd(renorm):
    p, idx, d_out = _tiny(7, T=6, H=5, E=5, K=3, I=4)
    tp = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in p.items()}
    out = _torch_block(tp, idx, renorm)
    (out * torch.tensor(d_out)).sum().backward()
    got = bwd.backward(p["x"], p["w_router"], p["bias"], p["w_gate"], p["w_up"], p["w_down"], idx, d_out, renorm)
    f = bwd.forward64(p["x"], p["w_router"], p["bias"], p["w_gate"], p["w_up"], p["w_down"], idx, renorm)
    assert np.allclose(f["out"], out.detach().numpy(), rtol=1e-12, atol=1e-12)
    for name, gname in GRAD_OF.items():
        ref = tp[name].grad.numpy()
        assert np.allclose(got[gname], ref, rtol=1e-10, atol=1e-12), name


def test_forward64_agrees_with_the_forward_oracle(oracle_lib):
    # same function up to the forward oracle's single rounding of the logits to float
    cfg = wl.small_config(40, 32, 6, 2, 16, dtype=wl.F32, seed=5, sigma_w=0.2)
    d = wl.make_inputs(cfg)
    out, idx, w = oracle_lib.forward(d["x_f32"], d["w_router_f32"], d["w_gate_f32"], d["w_up_f32"], d["w_down_f32"], cfg.K)
    f = bwd.forward64(d["x_f32"], d["w_router_f32"], None, d["w_gate_f32"], d["w_up_f32"], d["w_down_f32"], idx, True)
    assert np.allclose(f["w"], w, rtol=0, atol=2e-6)
    assert np.allclose(f["out"], out, rtol=1e-5, atol=1e-6 * np.abs(out).max())


def test_grouped_swiglu_backward_is_the_blockwise_backward():
    # rows sorted by expert with unit routing weight: the grouped function must give what `backward` gives for K = 1
    # (a single selected expert has weight 1, so nothing flows to the router)
    p, idx, d_out = _tiny(3, T=9, H=6, E=4, K=1, I=3)
    full = bwd.backward(p["x"], p["w_router"], p["bias"], p["w_gate"], p["w_up"], p["w_down"], idx, d_out, True)
    assert np.abs(full["d_w_router"]).max() == 0.0 and np.abs(full["d_router_bias"]).max() == 0.0
    order = np.argsort(idx[:, 0], kind="stable")
    counts = np.bincount(idx[:, 0], minlength=4)
    off = np.concatenate([[0], np.cumsum(counts)])
    g = bwd.grouped_swiglu_backward(p["x"][order], off, p["w_gate"], p["w_up"], p["w_down"], d_out[order])
    dx = np.zeros_like(p["x"])
    dx[order] = g["d_x_perm"]
    assert np.allclose(dx, full["d_x"], rtol=1e-12, atol=1e-12)
    for n in ("d_w_gate", "d_w_up", "d_w_down"):
        assert np.allclose(g[n], full[n], rtol=1e-12, atol=1e-12)


def test_silu_derivative_closed_forms():
    # one expert, one row, H = I = 1, Wu = Wd = 1: out = silu(wg x) x, so d out / d wg = silu'(wg x) x^2
    # silu'(0) = 1/2;  silu'(z) = s + z s (1 - s) with s = 1 / (1 + e^-z)
    for z in (0.0, 1.0, -2.5, 6.0):
        x = np.array([[1.0]])
        wg = np.array([[[z]]]); wu = np.array([[[1.0]]]); wd = np.array([[[1.0]]])
        g = bwd.grouped_swiglu_backward(x, [0, 1], wg, wu, wd, np.array([[1.0]]))
        s = 1.0 / (1.0 + math.exp(-z))
        want = s + z * s * (1.0 - s)
        assert abs(g["d_w_gate"][0, 0, 0] - want) < 1e-15
        assert abs(g["d_w_up"][0, 0, 0] - z * s) < 1e-15          # d/d wu = silu(z) x
        assert abs(g["d_w_down"][0, 0, 0] - z * s) < 1e-15        # d/d wd = a
    g0 = bwd.grouped_swiglu_backward(np.array([[1.0]]), [0, 1], np.zeros((1, 1, 1)), np.ones((1, 1, 1)), np.ones((1, 1, 1)),
                                     np.array([[1.0]]))
    assert g0["d_w_gate"][0, 0, 0] == 0.5


@pytest.mark.parametrize("renorm", [True, False])
def test_softmax_invariants_and_linearity(renorm):
    p, idx, d_out = _tiny(11, T=7, H=6, E=6, K=3, I=4)
    a = bwd.backward(p["x"], p["w_router"], p["bias"], p["w_gate"], p["w_up"], p["w_down"], idx, d_out, renorm)
    # shifting every logit of a token changes nothing, so its logit gradients sum to zero
    assert np.abs(a["d_logits"].sum(axis=1)).max() < 1e-13
    if renorm:      # only the selected logits matter
        mask = np.ones_like(a["d_logits"], dtype=bool)
        np.put_along_axis(mask, idx.astype(np.int64), False, axis=1)
        assert np.abs(a["d_logits"][mask]).max() == 0.0
    # linear in d_out
    b = bwd.backward(p["x"], p["w_router"], p["bias"], p["w_gate"], p["w_up"], p["w_down"], idx, -2.5 * d_out, renorm)
    for n in GRAD_OF.values():
        assert np.allclose(b[n], -2.5 * a[n], rtol=1e-12, atol=1e-13)
    # experts that received no token get no gradient
    unused = sorted(set(range(6)) - set(idx.reshape(-1).tolist()))
    for e in unused:
        assert np.abs(a["d_w_gate"][e]).max() == 0.0 and np.abs(a["d_w_down"][e]).max() == 0.0
    # a zero down projection blocks everything below it
    z = bwd.backward(p["x"], p["w_router"], p["bias"], p["w_gate"], p["w_up"], np.zeros_like(p["w_down"]), idx, d_out, renorm)
    assert np.abs(z["d_w_gate"]).max() == 0.0 and np.abs(z["d_w_up"]).max() == 0.0 and np.abs(z["d_x"]).max() == 0.0
