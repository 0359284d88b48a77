"""Backward pass of the routed-expert MoE FFN block, in float64 numpy.

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg, never by the product path.  Shares no code with the
HIP kernels.

The block is the one the forward oracle defines (Section 4.1 names the model; the
trainer differentiates it when it maximises the objective of Section 2.2, Eq. 2-3):

    l[t,e]  = <x_t, Wr_e> + b_e
    S_t     = the K experts with the largest logits (held fixed: the selection is
              piecewise constant, so it carries no gradient)
    w[t,k]  = softmax of l[t, S_t] over the K selected experts (renormalize), or the
              selected entries of the softmax over all E experts
    g = Wg_e x_t,  u = Wu_e x_t,  a = silu(g) * u,  y = Wd_e a      for e = S_t[k]
    out_t   = sum_k w[t,k] * y[t,k]

Given d_out = dL/d_out, the functions below return dL/d(everything), every step the
chain rule written out on real numbers (no intermediate rounding, unlike the bf16
forward the library runs).  `forward64` is the same function without any rounding;
the tests pin it to the forward oracle and pin `backward` to central differences of it.
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np


def _sigmoid(g: np.ndarray) -> np.ndarray:
    return 1.0 / (1.0 + np.exp(-g))


def routing_weights(logits_sel: np.ndarray, logits_all: np.ndarray, renormalize: bool) -> np.ndarray:
    """w [T,K] from the selected logits [T,K] (and all logits [T,E] when not renormalised)."""
    if renormalize:
        m = logits_sel.max(axis=1, keepdims=True)
        p = np.exp(logits_sel - m)
        return p / p.sum(axis=1, keepdims=True)
    m = logits_all.max(axis=1, keepdims=True)
    z = np.exp(logits_all - m).sum(axis=1, keepdims=True)
    return np.exp(logits_sel - m) / z


def forward64(x, w_router, bias, w_gate, w_up, w_down, topk_idx, renormalize: bool = True) -> Dict[str, np.ndarray]:
    """The block on real numbers with the selection given.  Returns out [T,H] and what backward needs."""
    x = np.asarray(x, dtype=np.float64)
    wr = np.asarray(w_router, dtype=np.float64)
    T, H = x.shape
    E = wr.shape[0]
    K = topk_idx.shape[1]
    logits = x @ wr.T
    if bias is not None:
        logits = logits + np.asarray(bias, dtype=np.float64)[None, :]
    lsel = np.take_along_axis(logits, topk_idx.astype(np.int64), axis=1)
    w = routing_weights(lsel, logits, renormalize)
    I = w_gate.shape[1]
    g = np.zeros((T, K, I)); u = np.zeros((T, K, I)); y = np.zeros((T, K, H))
    for e in range(E):
        tt, kk = np.nonzero(topk_idx == e)
        if tt.size == 0:
            continue
        xe = x[tt]
        g[tt, kk] = xe @ np.asarray(w_gate[e], dtype=np.float64).T
        u[tt, kk] = xe @ np.asarray(w_up[e], dtype=np.float64).T
        a = g[tt, kk] * _sigmoid(g[tt, kk]) * u[tt, kk]
        y[tt, kk] = a @ np.asarray(w_down[e], dtype=np.float64).T
    out = np.einsum("tk,tkh->th", w, y)
    return {"out": out, "logits": logits, "w": w, "g": g, "u": u, "y": y}


def swiglu_backward_rows(v, wg, wu, wd, dy):
    """One expert, rows v [R,H] with upstream dy [R,H]: returns dv, dWg, dWu, dWd.
    a = silu(g) u;  da = dy Wd;  dg = da u silu'(g);  du = da silu(g);  silu'(g) = s (1 + g (1 - s))."""
    g = v @ wg.T
    u = v @ wu.T
    s = _sigmoid(g)
    a = g * s * u
    da = dy @ wd                      # [R,I]
    dwd = dy.T @ a                    # [H,I]
    dg = da * u * (s * (1.0 + g * (1.0 - s)))
    du = da * (g * s)
    dwg = dg.T @ v                    # [I,H]
    dwu = du.T @ v
    dv = dg @ wg + du @ wu            # [R,H]
    return dv, dwg, dwu, dwd


def grouped_swiglu_backward(x_perm, expert_offsets, w_gate, w_up, w_down, dy_perm) -> Dict[str, np.ndarray]:
    """Backward of the grouped SwiGLU FFN over expert-sorted rows: rows [off[e], off[e+1]) belong to expert e."""
    xp = np.asarray(x_perm, dtype=np.float64)
    dyp = np.asarray(dy_perm, dtype=np.float64)
    E, I, H = w_gate.shape
    dxp = np.zeros_like(xp)
    dwg = np.zeros((E, I, H)); dwu = np.zeros((E, I, H)); dwd = np.zeros((E, H, I))
    for e in range(E):
        r0, r1 = int(expert_offsets[e]), int(expert_offsets[e + 1])
        if r1 == r0:
            continue
        dv, dwg[e], dwu[e], dwd[e] = swiglu_backward_rows(
            xp[r0:r1], np.asarray(w_gate[e], dtype=np.float64), np.asarray(w_up[e], dtype=np.float64),
            np.asarray(w_down[e], dtype=np.float64), dyp[r0:r1])
        dxp[r0:r1] = dv
    return {"d_x_perm": dxp, "d_w_gate": dwg, "d_w_up": dwu, "d_w_down": dwd}


def backward(x, w_router, bias, w_gate, w_up, w_down, topk_idx, d_out, renormalize: bool = True) -> Dict[str, np.ndarray]:
    """dL/dx, dL/dWr, dL/db, dL/dWg, dL/dWu, dL/dWd for L with dL/d_out = d_out."""
    x = np.asarray(x, dtype=np.float64)
    wr = np.asarray(w_router, dtype=np.float64)
    d_out = np.asarray(d_out, dtype=np.float64)
    T, H = x.shape
    E, I = w_gate.shape[0], w_gate.shape[1]
    K = topk_idx.shape[1]
    f = forward64(x, w_router, bias, w_gate, w_up, w_down, topk_idx, renormalize)
    w, y, logits = f["w"], f["y"], f["logits"]
    idx = topk_idx.astype(np.int64)

    # out_t = sum_k w_k y_k:  dy_k = w_k d_out_t,  dw_k = <d_out_t, y_k>
    dw = np.einsum("th,tkh->tk", d_out, y)
    # routing weights -> logits
    dlogits = np.zeros((T, E))
    if renormalize:
        # softmax over the K selected logits: dl_k = w_k (dw_k - sum_j w_j dw_j)
        dl = w * (dw - (w * dw).sum(axis=1, keepdims=True))
        np.put_along_axis(dlogits, idx, dl, axis=1)
    else:
        # w_k = p_{e_k}, p the softmax over all E: dl_e = p_e ([e selected] dw_e - sum_k p_{e_k} dw_k)
        m = logits.max(axis=1, keepdims=True)
        p = np.exp(logits - m)
        p /= p.sum(axis=1, keepdims=True)
        dw_dense = np.zeros((T, E))
        np.put_along_axis(dw_dense, idx, dw, axis=1)
        dlogits = p * (dw_dense - (w * dw).sum(axis=1, keepdims=True))
    dx = dlogits @ wr
    dwr = dlogits.T @ x
    dbias = dlogits.sum(axis=0)

    dwg = np.zeros((E, I, H)); dwu = np.zeros((E, I, H)); dwd = np.zeros((E, H, I))
    for e in range(E):
        tt, kk = np.nonzero(idx == e)
        if tt.size == 0:
            continue
        dy = w[tt, kk][:, None] * d_out[tt]
        dv, dwg[e], dwu[e], dwd[e] = swiglu_backward_rows(
            x[tt], np.asarray(w_gate[e], dtype=np.float64), np.asarray(w_up[e], dtype=np.float64),
            np.asarray(w_down[e], dtype=np.float64), dy)
        np.add.at(dx, tt, dv)
    return {"d_x": dx, "d_w_router": dwr, "d_router_bias": dbias, "d_w_gate": dwg, "d_w_up": dwu,
            "d_w_down": dwd, "d_topk_w": dw, "d_logits": dlogits}
