"""GPU parity of the backward pass against the float64 oracle, through the C ABI.

Tolerances: the library rounds g, u, d_out*Wd, dg, du and w*a to bf16 (relative 2^-9 each) and sums in float, so
every gradient carries a few independent roundings per term: relative L2 error of a few 1e-3 expected, bound 1e-2;
largest single deviation bounded by 2e-2 of the largest magnitude of the tensor.
"""
import numpy as np
import pytest
import torch

from oracle import moe_backward_oracle as bwd
from paper_2511_11373_amd import moe, moe_backward as mb
from paper_2511_11373_amd import workloads as wl
from gpu_util import check_close, host, shape_of, to_dev, upload

pytestmark = pytest.mark.gpu


def _bf16_normal(rng, shape, scale=1.0):
    bits = wl.f32_to_bf16_bits_numpy((rng.standard_normal(shape) * scale).astype(np.float32))
    return bits, wl.bf16_bits_to_f32(bits)


def _cmp(got, ref, what):
    ref = np.asarray(ref, dtype=np.float64)
    scale = max(np.abs(ref).max(), 1e-30)
    return check_close(host(got), ref, what, max_abs=2e-2 * scale, rel_l2=1e-2)


@pytest.mark.parametrize("counts,H,I,dtype", [([0, 70, 0, 33, 256, 1, 300, 0], 136, 72, wl.BF16),
                                              ([0, 700, 0, 257, 256, 1, 0, 900, 3, 0], 128, 64, wl.BF16),     # takes the LDS-pipelined kernels
                                              ([3, 0, 260, 41], 128, 64, wl.F32)],
                         ids=["small", "large", "float"])
def test_grouped_swiglu_backward_uneven_segments(oracle_lib, counts, H, I, dtype):
    n, E = sum(counts), len(counts)
    cfg = wl.small_config(n, H, E, 1, I, dtype=dtype, seed=41, sigma_w=0.1)
    d = wl.make_inputs(cfg)
    g = upload(cfg, d)
    rng = np.random.default_rng(41)
    dy_bits, dy = _bf16_normal(rng, (n, H))
    if dtype == wl.F32:
        dy_bits = dy
    off = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    shp = shape_of(cfg)
    ws = mb.alloc_workspace(shp)
    out = mb.moe_grouped_swiglu_backward(shp, g["x"], torch.from_numpy(off).cuda(), g["w_gate"], g["w_up"], g["w_down"],
                                         to_dev(dy_bits, dtype), ws)
    assert out["d_x_perm"].dtype == g["x"].dtype
    ref = bwd.grouped_swiglu_backward(d["x_f32"], off, d["w_gate_f32"], d["w_up_f32"], d["w_down_f32"], dy)
    for name in ("d_x_perm", "d_w_gate", "d_w_up", "d_w_down"):
        _cmp(out[name], ref[name], name)
    # experts without rows get exact zeros
    for e in [i for i, c in enumerate(counts) if c == 0]:
        assert torch.count_nonzero(out["d_w_gate"][e]).item() == 0 and torch.count_nonzero(out["d_w_down"][e]).item() == 0


CASES = [
    wl.small_config(37, 72, 5, 3, 40, dtype=wl.BF16, seed=42, sigma_w=0.1),          # nothing divides a tile
    wl.small_config(300, 256, 16, 4, 128, dtype=wl.BF16, seed=43, sigma_w=0.05),
    wl.small_config(64, 128, 40, 8, 64, dtype=wl.BF16, seed=44, sigma_w=0.1),         # most experts get one or two rows
    wl.small_config(1500, 256, 70, 4, 64, dtype=wl.BF16, seed=45, sigma_w=0.05),      # large-batch router, several row tiles
    wl.small_config(600, 256, 4, 2, 256, dtype=wl.BF16, seed=46, sigma_w=0.05),       # pre-activations by the forward pass's large-batch kernel
    wl.small_config(900, 192, 3, 2, 320, dtype=wl.BF16, seed=47, sigma_w=0.05),       # LDS-pipelined GEMMs, no dimension a multiple of 256
    wl.small_config(152, 64, 3, 2, 320, dtype=wl.BF16, seed=48, sigma_w=0.05),        # few experts: bias gradients cancel almost fully
    wl.small_config(700, 320, 4, 2, 384, dtype=wl.BF16, seed=50, sigma_w=0.05),       # rows of x and d_out through the token map, ragged last tiles in every GEMM
    wl.small_config(14, 512, 128, 2, 264, dtype=wl.BF16, seed=49, sigma_w=0.05),      # fewer assignments than experts
    # routing weights taken from the softmax over all experts (not renormalised): every logit of a token has a gradient
    wl.small_config(37, 72, 5, 3, 40, dtype=wl.BF16, seed=52, sigma_w=0.1, renormalize=False),
    wl.small_config(300, 256, 16, 4, 128, dtype=wl.BF16, seed=53, sigma_w=0.05, renormalize=False),     # with a bias (odd seed)
    wl.small_config(1500, 256, 70, 4, 64, dtype=wl.BF16, seed=54, sigma_w=0.05, renormalize=False),
    wl.small_config(40, 64, 300, 5, 16, dtype=wl.BF16, seed=55, sigma_w=0.1, renormalize=False),        # more than 256 experts
    # float storage: the router reads the floats, everything else is rounded to bf16 on the way in
    wl.small_config(130, 264, 6, 3, 136, dtype=wl.F32, seed=56, sigma_w=0.05),
    wl.small_config(300, 256, 16, 4, 128, dtype=wl.F32, seed=57, sigma_w=0.05),                         # with a bias, LDS-pipelined GEMMs
    wl.small_config(90, 128, 12, 2, 64, dtype=wl.F32, seed=58, sigma_w=0.1, renormalize=False),
]


def _cmp_bias(got, ref, o_idx, o_w, probs=None):
    """The bias gradient of an expert sums logit gradients of both signs, which largely cancel (those of one token sum to
    zero): besides the 2e-2 of the largest entry allowed to every tensor, its error grows with the magnitudes summed,
    w_k (|dw_k| + sum_j w_j |dw_j|) over the assignments of the expert, dw the gradient of the combine weights.  With
    un-renormalised weights every token contributes to every expert: p_e ([e selected] |dw_e| + sum_j w_j |dw_j|), p the
    softmax over all experts."""
    w = np.asarray(o_w, dtype=np.float64)
    adw = np.abs(ref["d_topk_w"])
    mean = (w * adw).sum(axis=1, keepdims=True)
    E = ref["d_router_bias"].shape[0]
    if probs is None:
        summed = np.zeros(E)
        np.add.at(summed, o_idx.reshape(-1), (w * (adw + mean)).reshape(-1))
    else:
        sel = np.zeros_like(probs)
        np.put_along_axis(sel, o_idx.astype(np.int64), adw, axis=1)
        summed = (probs * (sel + mean)).sum(axis=0)
    err = np.abs(host(got).astype(np.float64) - ref["d_router_bias"])
    tol = 2e-2 * np.abs(ref["d_router_bias"]).max() + 4e-3 * summed
    assert np.all(err <= tol), f"d_router_bias: worst error/tolerance {np.max(err / np.maximum(tol, 1e-300)):.3g}"


def _full_softmax(oracle_lib, d, bias):
    from scipy.special import softmax
    return softmax(oracle_lib.router_logits(d["x_f32"], d["w_router_f32"], bias).astype(np.float64), axis=1)


@pytest.mark.parametrize("cfg", CASES, ids=[c.name + ("" if c.renormalize else "-norenorm") + "-" + c.dtype for c in CASES])
def test_backward_against_oracle(oracle_lib, cfg):
    d = wl.make_inputs(cfg)
    g = upload(cfg, d)
    rng = np.random.default_rng(cfg.seed)
    bias = (rng.standard_normal(cfg.E) * 0.1).astype(np.float32) if cfg.seed % 2 else None
    do_bits, do = _bf16_normal(rng, (cfg.T, cfg.H))
    if cfg.dtype == wl.F32:       # float storage: d_out is float too (values a bf16 holds, so that the oracle sees what the GPU multiplies)
        do_bits = do
    shp = shape_of(cfg)
    ws = mb.alloc_workspace(shp)
    bias_dev = None if bias is None else torch.from_numpy(bias).cuda()
    out = mb.moe_backward(shp, g["x"], g["w_router"], bias_dev, g["w_gate"], g["w_up"], g["w_down"], to_dev(do_bits, cfg.dtype), ws)
    assert out["d_x"].dtype == g["x"].dtype
    o_idx, o_w = oracle_lib.route_topk(d["x_f32"], d["w_router_f32"], cfg.K, bias, cfg.renormalize)
    ref = bwd.backward(d["x_f32"], d["w_router_f32"], bias, d["w_gate_f32"], d["w_up_f32"], d["w_down_f32"], o_idx, do, cfg.renormalize)
    for name in ("d_x", "d_w_router", "d_w_gate", "d_w_up", "d_w_down"):
        _cmp(out[name], ref[name], name)
    _cmp_bias(out["d_router_bias"], ref, o_idx, o_w, None if cfg.renormalize else _full_softmax(oracle_lib, d, bias))
    # a second call gives the same bits
    out2 = mb.moe_backward(shp, g["x"], g["w_router"], bias_dev, g["w_gate"], g["w_up"], g["w_down"], to_dev(do_bits, cfg.dtype), ws)
    for name in out:
        assert torch.equal(out[name], out2[name]), name


def test_full_size_backward_every_element(oracle_lib):
    """The bench workload (16384 tokens, 128 experts) in the configuration bench.py times: every element of every
    gradient (d_x of all tokens, the router's and all 128 experts' weight gradients) against the float64 oracle."""
    cfg = wl.CONFIGS["prefill16k"]
    d = wl.make_inputs(cfg)
    g = upload(cfg, d)
    rng = np.random.default_rng(77)
    do_bits = wl.f32_to_bf16_bits(rng.standard_normal((cfg.T, cfg.H), dtype=np.float32))
    do = wl.bf16_bits_to_f32(do_bits)
    shp = shape_of(cfg)
    ws = mb.alloc_workspace(shp)
    out = mb.moe_backward(shp, g["x"], g["w_router"], None, g["w_gate"], g["w_up"], g["w_down"], to_dev(do_bits, wl.BF16), ws)
    # the pair that keeps the pre-activations gives the same bits at this size too
    _, g_rows, u_rows = mb.moe_forward_saving(shp, g["x"], g["w_router"], None, g["w_gate"], g["w_up"], g["w_down"], moe.alloc_workspace(shp))
    saved = mb.moe_backward_saved(shp, g["x"], g["w_router"], None, g["w_gate"], g["w_up"], g["w_down"], to_dev(do_bits, wl.BF16),
                                  g_rows, u_rows, mb.alloc_workspace(shp))
    for name in out:
        assert torch.equal(out[name], saved[name]), name
    del saved, g_rows, u_rows
    o_idx, o_w = oracle_lib.route_topk(d["x_f32"], d["w_router_f32"], cfg.K)
    ref = bwd.backward(d["x_f32"], d["w_router_f32"], None, d["w_gate_f32"], d["w_up_f32"], d["w_down_f32"], o_idx, do, True)
    for name in ("d_x", "d_w_router", "d_w_gate", "d_w_up", "d_w_down"):
        _cmp(out[name], ref[name], name)
    _cmp_bias(out["d_router_bias"], ref, o_idx, o_w)
    # no single token and no single expert may be far off either (one wrong row tile would hide in the norm of the rest)
    dx = host(out["d_x"])
    tok_rel = np.linalg.norm(dx - ref["d_x"], axis=1) / np.linalg.norm(ref["d_x"], axis=1)
    assert tok_rel.max() <= 3e-2, (int(tok_rel.argmax()), float(tok_rel.max()))
    for name in ("d_w_gate", "d_w_up", "d_w_down"):
        got = host(out[name]).reshape(cfg.E, -1)
        want = ref[name].reshape(cfg.E, -1)
        e_rel = np.linalg.norm(got - want, axis=1) / np.linalg.norm(want, axis=1)
        assert e_rel.max() <= 1e-2, (name, int(e_rel.argmax()), float(e_rel.max()))


SAVING_CASES = [
    wl.small_config(600, 256, 4, 2, 256, dtype=wl.BF16, seed=61, sigma_w=0.05),       # whole and ragged 256-row tiles
    wl.small_config(37, 256, 5, 3, 128, dtype=wl.BF16, seed=62, sigma_w=0.05),        # a handful of rows per expert
    wl.small_config(1100, 512, 16, 4, 384, dtype=wl.BF16, seed=63, sigma_w=0.05),     # with a router bias (odd seed)
]


@pytest.mark.parametrize("cfg", SAVING_CASES, ids=[c.name for c in SAVING_CASES])
def test_saved_pre_activations_pair(oracle_lib, cfg):
    """moe_forward_saving + moe_backward_saved: the output against the forward oracle, the gradients against the
    backward oracle, and bit for bit against moe_backward (whose recomputation yields the same g and u)."""
    d = wl.make_inputs(cfg)
    g = upload(cfg, d)
    rng = np.random.default_rng(cfg.seed)
    bias = (rng.standard_normal(cfg.E) * 0.1).astype(np.float32) if cfg.seed % 2 else None
    bias_dev = None if bias is None else torch.from_numpy(bias).cuda()
    do_bits, do = _bf16_normal(rng, (cfg.T, cfg.H))
    shp = shape_of(cfg)
    idx = torch.empty((cfg.T, cfg.K), dtype=torch.int32, device="cuda")
    wgt = torch.empty((cfg.T, cfg.K), dtype=torch.float32, device="cuda")
    out, g_rows, u_rows = mb.moe_forward_saving(shp, g["x"], g["w_router"], bias_dev, g["w_gate"], g["w_up"], g["w_down"],
                                                moe.alloc_workspace(shp), topk_idx_out=idx, topk_w_out=wgt)
    o_out, _, _ = oracle_lib.forward(d["x_f32"], d["w_router_f32"], d["w_gate_f32"], d["w_up_f32"], d["w_down_f32"], cfg.K, bias)
    check_close(host(out), o_out, "out", max_abs=2e-2 * max(1.0, np.abs(o_out).max()))
    ws = mb.alloc_workspace(shp)
    got = mb.moe_backward_saved(shp, g["x"], g["w_router"], bias_dev, g["w_gate"], g["w_up"], g["w_down"], to_dev(do_bits, wl.BF16),
                                g_rows, u_rows, ws)
    o_idx, o_w = oracle_lib.route_topk(d["x_f32"], d["w_router_f32"], cfg.K, bias)
    ref = bwd.backward(d["x_f32"], d["w_router_f32"], bias, d["w_gate_f32"], d["w_up_f32"], d["w_down_f32"], o_idx, do, True)
    for name in ("d_x", "d_w_router", "d_w_gate", "d_w_up", "d_w_down"):
        _cmp(got[name], ref[name], name)
    _cmp_bias(got["d_router_bias"], ref, o_idx, o_w)
    assert np.array_equal(host(idx), o_idx)
    again = mb.moe_backward(shp, g["x"], g["w_router"], bias_dev, g["w_gate"], g["w_up"], g["w_down"], to_dev(do_bits, wl.BF16), ws)
    for name in got:
        assert torch.equal(got[name], again[name]), name
    # ... and with the routing kept too
    kept = mb.moe_backward_saved(shp, g["x"], g["w_router"], bias_dev, g["w_gate"], g["w_up"], g["w_down"], to_dev(do_bits, wl.BF16),
                                 g_rows, u_rows, ws, topk_idx=idx, topk_w=wgt)
    for name in got:
        assert torch.equal(got[name], kept[name]), name


def test_saving_pair_restrictions():
    shp = moe.make_shape(8, 192, 4, 2, 128, moe.MOE_BF16)           # H not a multiple of 256
    z = lambda *s: torch.zeros(s, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(moe.MoeError) as e:
        mb.moe_forward_saving(shp, z(8, 192), z(4, 192), None, z(4, 128, 192), z(4, 128, 192), z(4, 192, 128), moe.alloc_workspace(shp))
    assert e.value.code == 2
    shp = moe.make_shape(8, 256, 4, 2, 128, moe.MOE_F32)
    f = lambda *s: torch.zeros(s, dtype=torch.float32, device="cuda")
    with pytest.raises(moe.MoeError) as e:
        mb.moe_forward_saving(shp, f(8, 256), f(4, 256), None, f(4, 128, 256), f(4, 128, 256), f(4, 256, 128), moe.alloc_workspace(shp),
                              out=z(8, 256))
    assert e.value.code == 3


def test_backward_restrictions_and_empty_batch():
    with pytest.raises(moe.MoeError) as e:
        mb.workspace_bytes(moe.make_shape(8, 64, 4, 2, 32, 7))        # no such storage type
    assert e.value.code == 3
    assert mb.workspace_bytes(moe.make_shape(8, 64, 4, 2, 32, moe.MOE_F32)) > mb.workspace_bytes(moe.make_shape(8, 64, 4, 2, 32, moe.MOE_BF16))
    assert mb.workspace_bytes(moe.make_shape(8, 64, 4, 2, 32, moe.MOE_BF16, renormalize=False)) > \
        mb.workspace_bytes(moe.make_shape(8, 64, 4, 2, 32, moe.MOE_BF16))      # room for the softmax over all experts
    shp = moe.make_shape(0, 64, 4, 2, 32, moe.MOE_BF16)
    ws = mb.alloc_workspace(shp)
    z = lambda *s: torch.zeros(s, dtype=torch.bfloat16, device="cuda")
    out = {k: torch.ones(v, dtype=torch.float32, device="cuda") for k, v in
           (("d_w_router", (4, 64)), ("d_router_bias", (4,)), ("d_w_gate", (4, 32, 64)), ("d_w_up", (4, 32, 64)), ("d_w_down", (4, 64, 32)))}
    out["d_x"] = z(1, 64)      # never written: there is no token (a zero-size tensor would have a NULL pointer)
    mb.moe_backward(shp, z(1, 64), z(4, 64), None, z(4, 32, 64), z(4, 32, 64), z(4, 64, 32), z(1, 64), ws, out=out)
    torch.cuda.synchronize()
    for name in ("d_w_router", "d_router_bias", "d_w_gate", "d_w_up", "d_w_down"):
        assert torch.count_nonzero(out[name]).item() == 0, name
