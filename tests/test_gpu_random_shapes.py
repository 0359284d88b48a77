"""Randomly drawn valid shapes through the forward block, the backward block and decode attention, each against its
oracle.  The shapes are fixed by the seed below; they are there for what hand-picked cases miss: sizes that are not a
multiple of any tile, experts with no or a single row, batches on either side of every kernel-selection threshold."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import oracle
from oracle import moe_backward_oracle as bwd
from paper_2511_11373_amd import moe, moe_backward as mb, workloads as wl

from gpu_util import check_close, check_weights, host, shape_of, to_dev, upload
import test_attn_gpu as attn_cases
import test_backward_gpu as backward_cases

pytestmark = pytest.mark.gpu

N_CASES = 60


def _draw(case: int):
    """The case-th shape: (kind, parameters).  Every case has a generator of its own, so cases do not depend on each other."""
    rng = np.random.default_rng(7000 + case)
    pick = lambda vals: int(vals[rng.integers(0, len(vals))])
    kind = ("forward", "backward", "attention")[case % 3]
    if kind == "attention":
        B = int(rng.integers(1, 6))
        Hkv, group = pick([1, 2, 4, 8]), pick([1, 2, 3, 4, 8, 16])
        lens = [int(rng.integers(0, 6000)) if rng.random() < 0.8 else int(rng.integers(0, 70)) for _ in range(B)]
        return kind, (lens, Hkv * group, Hkv)
    E = pick([1, 2, 3, 5, 8, 16, 33, 64, 128])
    K = int(rng.integers(1, min(E, 8) + 1))
    H = 8 * int(rng.integers(1, 65)) if rng.random() < 0.5 else pick([64, 128, 192, 256, 512, 1024])
    I = 8 * int(rng.integers(1, 49)) if rng.random() < 0.5 else pick([64, 128, 256, 320, 384])
    T = int(rng.integers(1, 40)) if rng.random() < 0.3 else int(rng.integers(40, 2600))
    dtype = wl.BF16 if (kind == "backward" or rng.random() < 0.7) else wl.F32
    return kind, (T, H, E, K, I, dtype)


def _name(case: int) -> str:
    kind, p = _draw(case)
    if kind == "attention":
        return f"attention-{len(p[0])}seq-Hq{p[1]}-Hkv{p[2]}"
    return f"{kind}-T{p[0]}H{p[1]}E{p[2]}K{p[3]}I{p[4]}-{p[5]}"


@pytest.mark.parametrize("case", range(N_CASES), ids=[_name(c) for c in range(N_CASES)])
def test_random_shape(oracle_lib, case):
    kind, p = _draw(case)
    if kind == "attention":
        lens, Hq, Hkv = p
        attn_cases.run_case(9000 + case, lens, Hq, Hkv, poison=bool(case % 2))
        return
    T, H, E, K, I, dtype = p
    cfg = wl.small_config(T, H, E, K, I, dtype=dtype, seed=8000 + case, sigma_w=0.05)
    d = wl.make_inputs(cfg)
    g = upload(cfg, d)
    shp = shape_of(cfg)
    o_idx, o_w = oracle_lib.route_topk(d["x_f32"], d["w_router_f32"], K)
    if kind == "forward":
        ws = moe.alloc_workspace(shp)
        idx = torch.empty((T, K), dtype=torch.int32, device="cuda")
        w = torch.empty((T, K), dtype=torch.float32, device="cuda")
        out = moe.moe_forward(shp, g["x"], g["w_router"], None, g["w_gate"], g["w_up"], g["w_down"], ws, topk_idx_out=idx,
                              topk_w_out=w)
        o_out, _, _ = oracle_lib.forward(d["x_f32"], d["w_router_f32"], d["w_gate_f32"], d["w_up_f32"], d["w_down_f32"], K)
        assert np.array_equal(host(idx), o_idx)
        check_weights(host(w), o_w)
        check_close(host(out), o_out, "forward", max_abs=2e-2 * max(1.0, np.abs(o_out).max()))
        return
    rng = np.random.default_rng(8500 + case)
    do_bits = wl.f32_to_bf16_bits_numpy(rng.standard_normal((T, H)).astype(np.float32))
    ws = mb.alloc_workspace(shp)
    out = mb.moe_backward(shp, g["x"], g["w_router"], None, g["w_gate"], g["w_up"], g["w_down"], to_dev(do_bits, wl.BF16), ws)
    ref = bwd.backward(d["x_f32"], d["w_router_f32"], None, d["w_gate_f32"], d["w_up_f32"], d["w_down_f32"], o_idx,
                       wl.bf16_bits_to_f32(do_bits), True)
    backward_cases._cmp_bias(out["d_router_bias"], ref, o_idx, o_w)
    for name in ("d_x", "d_w_router", "d_w_gate", "d_w_up", "d_w_down"):
        backward_cases._cmp(out[name], ref[name], name)
