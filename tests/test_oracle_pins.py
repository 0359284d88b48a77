"""Pins of the CPU oracle to things other than itself (CPU only).

The paper gives no worked numbers for the MoE layer (Section 4.1 only names the
model), so the oracle is pinned by: closed forms, invariants of the definition,
special cases that reduce to library routines (numpy stable argsort, scipy
softmax, torch matmul + silu), exactly rounded sums (math.fsum), a hand-worked
example, and an independent dense brute force on tiny inputs.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.special
import torch

from oracle import bruteforce
from paper_2511_11373_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(cfg):
    d = wl.make_inputs(cfg)
    return d["x_f32"], d["w_router_f32"], d["w_gate_f32"], d["w_up_f32"], d["w_down_f32"]


# ---------------------------------------------------------------- router

def test_logits_are_the_correctly_rounded_exact_sum(oracle_lib):
    # bf16 x bf16 products and their sum are exact in double here, so the float
    # logit must equal the correctly rounded exact rational sum.
    cfg = wl.small_config(5, 96, 7, 2, 8, dtype=wl.BF16, seed=3)
    d = wl.make_inputs(cfg)
    x, wr = d["x_f32"], d["w_router_f32"]
    bias = np.linspace(-0.5, 0.5, cfg.E).astype(np.float32)
    got = oracle_lib.router_logits(x, wr, bias)
    for t in range(cfg.T):
        for e in range(cfg.E):
            exact = sum((Fraction(float(x[t, h])) * Fraction(float(wr[e, h])) for h in range(cfg.H)),
                        Fraction(float(bias[e])))
            assert got[t, e] == np.float32(float(exact)), (t, e)


def test_logits_fp32_inputs_match_fsum(oracle_lib):
    cfg = wl.small_config(4, 64, 5, 2, 8, dtype=wl.F32, seed=4)
    d = wl.make_inputs(cfg)
    x, wr = d["x_f32"], d["w_router_f32"]
    got = oracle_lib.router_logits(x, wr)
    for t in range(cfg.T):
        for e in range(cfg.E):
            ref = math.fsum(float(x[t, h]) * float(wr[e, h]) for h in range(cfg.H))
            assert abs(float(got[t, e]) - ref) <= 2.0 ** -24 * abs(ref) + 1e-30


def test_selection_matches_library_lexsort(oracle_lib):
    rng = np.random.default_rng(0)
    logits = rng.standard_normal((50, 16)).astype(np.float32)
    logits[:, 3] = logits[:, 9]          # planted ties
    logits[7, :] = 0.25
    idx, _ = oracle_lib.topk_from_logits(logits, 5)
    for t in range(logits.shape[0]):
        order = np.lexsort((np.arange(16), -logits[t].astype(np.float64)))
        assert idx[t].tolist() == order[:5].tolist()


def test_weights_sum_to_one_and_closed_form(oracle_lib):
    cfg = wl.CONFIGS["tiny"]
    x, wr, *_ = _rand(cfg)
    logits = oracle_lib.router_logits(x, wr)
    idx, w = oracle_lib.topk_from_logits(logits, cfg.K, True)
    assert np.all(np.abs(w.astype(np.float64).sum(axis=1) - 1.0) <= 1e-6)
    # renormalised top-K of the full softmax == softmax over the K selected logits
    full = scipy.special.softmax(logits.astype(np.float64), axis=1)
    sel = np.take_along_axis(full, idx.astype(np.int64), axis=1)
    np.testing.assert_allclose(w, sel / sel.sum(axis=1, keepdims=True), rtol=1e-6, atol=1e-7)
    # slot 0 is the arg-max and weights are non-increasing
    assert np.array_equal(idx[:, 0], logits.argmax(axis=1))
    assert np.all(np.diff(w, axis=1) <= 0)


def test_unnormalised_weights_are_full_softmax_entries(oracle_lib):
    rng = np.random.default_rng(1)
    logits = rng.standard_normal((20, 12)).astype(np.float32)
    idx, w = oracle_lib.topk_from_logits(logits, 4, False)
    full = scipy.special.softmax(logits.astype(np.float64), axis=1)
    np.testing.assert_allclose(w, np.take_along_axis(full, idx.astype(np.int64), axis=1), rtol=1e-6)


def test_k_equals_e_is_full_softmax_mixture(oracle_lib):
    cfg = wl.small_config(6, 32, 4, 4, 16, seed=5, sigma_w=0.3)
    x, wr, wg, wu, wd = _rand(cfg)
    out, idx, w = oracle_lib.forward(x, wr, wg, wu, wd, cfg.K)
    logits = oracle_lib.router_logits(x, wr)
    full = scipy.special.softmax(logits.astype(np.float64), axis=1)
    assert np.array_equal(np.sort(idx, axis=1), np.tile(np.arange(4), (cfg.T, 1)))
    np.testing.assert_allclose(np.take_along_axis(full, idx.astype(np.int64), axis=1), w, rtol=1e-6)
    ref = np.zeros_like(out)
    xt = torch.from_numpy(x).double()
    for e in range(cfg.E):
        g = xt @ torch.from_numpy(wg[e]).double().T
        u = xt @ torch.from_numpy(wu[e]).double().T
        y = (torch.nn.functional.silu(g) * u) @ torch.from_numpy(wd[e]).double().T
        ref += full[:, e:e + 1] * y.numpy()
    np.testing.assert_allclose(out, ref, rtol=1e-5, atol=1e-9)


def test_all_equal_logits_tie_break(oracle_lib):
    cfg = wl.small_config(9, 32, 8, 4, 16, seed=6)
    x, wr, wg, wu, wd = _rand(cfg)
    idx, w = oracle_lib.route_topk(x, np.zeros_like(wr), cfg.K)
    assert np.array_equal(idx, np.tile(np.arange(cfg.K, dtype=np.int32), (cfg.T, 1)))
    assert np.all(w == np.float32(1.0 / cfg.K))


# ---------------------------------------------------------------- permutation

def test_permute_is_the_stable_sort_and_round_trips(oracle_lib):
    rng = np.random.default_rng(2)
    T, K, E = 37, 3, 11
    idx = np.stack([rng.permutation(E)[:K] for _ in range(T)]).astype(np.int32)
    off, r2a, a2r = oracle_lib.permute(idx, E + 2)       # two experts certainly empty
    flat = idx.reshape(-1)
    n = T * K
    assert np.array_equal(r2a, np.argsort(flat, kind="stable").astype(np.int32))
    assert np.array_equal(off, np.concatenate([[0], np.cumsum(np.bincount(flat, minlength=E + 2))]))
    assert off[-1] == n and off[E + 1] == off[E] == n
    assert np.array_equal(r2a[a2r], np.arange(n)) and np.array_equal(a2r[r2a], np.arange(n))
    for e in range(E + 2):
        seg = r2a[off[e]:off[e + 1]]
        assert np.all(flat[seg] == e) and np.all(np.diff(seg) > 0)
    x = rng.standard_normal((T, 8)).astype(np.float32)
    xp = oracle_lib.gather_rows(x, r2a, K)
    assert np.array_equal(xp[a2r], np.repeat(x, K, axis=0))      # permute then un-permute = identity


def test_permute_rejects_out_of_range(oracle_lib):
    with pytest.raises(ValueError):
        oracle_lib.permute(np.array([[0, 9]], dtype=np.int32), 4)


# ---------------------------------------------------------------- expert FFN and the whole block

def test_single_expert_is_a_dense_swiglu_mlp(oracle_lib):
    cfg = wl.small_config(10, 48, 1, 1, 24, seed=7, sigma_w=0.25)
    x, wr, wg, wu, wd = _rand(cfg)
    out, idx, w = oracle_lib.forward(x, wr, wg, wu, wd, 1)
    assert np.all(idx == 0) and np.all(w == np.float32(1.0))
    xt = torch.from_numpy(x).double()
    ref = (torch.nn.functional.silu(xt @ torch.from_numpy(wg[0]).double().T)
           * (xt @ torch.from_numpy(wu[0]).double().T)) @ torch.from_numpy(wd[0]).double().T
    np.testing.assert_allclose(out, ref.numpy(), rtol=1e-10, atol=1e-13)
    # not symmetric in gate/up: swapping them must change the result
    out_sw, _, _ = oracle_lib.forward(x, wr, wu, wg, wd, 1)
    assert np.abs(out_sw - out).max() > 1e-3 * np.abs(out).max()


def test_grouped_swiglu_against_per_row_torch(oracle_lib):
    rng = np.random.default_rng(8)
    E, H, I = 5, 24, 16
    off = np.array([0, 3, 3, 4, 9, 9], dtype=np.int32)     # experts 1 and 4 empty
    xp = rng.standard_normal((9, H)).astype(np.float32)
    wg = rng.standard_normal((E, I, H)).astype(np.float32) * 0.3
    wu = rng.standard_normal((E, I, H)).astype(np.float32) * 0.3
    wd = rng.standard_normal((E, H, I)).astype(np.float32) * 0.3
    y = oracle_lib.grouped_swiglu(xp, off, wg, wu, wd)
    for e in range(E):
        for r in range(off[e], off[e + 1]):
            v = torch.from_numpy(xp[r]).double()
            a = torch.nn.functional.silu(torch.from_numpy(wg[e]).double() @ v) * (torch.from_numpy(wu[e]).double() @ v)
            np.testing.assert_allclose(y[r], (torch.from_numpy(wd[e]).double() @ a).numpy(), rtol=1e-10, atol=1e-13)


def test_combine_is_the_weighted_gather_sum(oracle_lib):
    rng = np.random.default_rng(9)
    T, K, H = 6, 3, 10
    y = rng.standard_normal((T * K, H))
    a2r = rng.permutation(T * K).astype(np.int32)
    w = rng.random((T, K)).astype(np.float32)
    out = oracle_lib.combine(y, a2r, w)
    ref = np.einsum("tk,tkh->th", w.astype(np.float64), y[a2r].reshape(T, K, H))
    np.testing.assert_allclose(out, ref, rtol=1e-13, atol=1e-15)


@pytest.mark.parametrize("shape", [(64, 256, 8, 2, 128), (13, 40, 6, 3, 24), (7, 16, 5, 5, 8), (3, 8, 4, 1, 8)])
def test_brute_force_agrees(oracle_lib, shape):
    cfg = wl.small_config(*shape, seed=11, sigma_w=0.02 if shape[1] >= 256 else 0.3)
    if shape == (64, 256, 8, 2, 128):
        cfg = wl.CONFIGS["tiny"]
    x, wr, wg, wu, wd = _rand(cfg)
    bias = None if shape[0] == 64 else np.linspace(0.3, -0.3, cfg.E).astype(np.float32)
    out, idx, w = oracle_lib.forward(x, wr, wg, wu, wd, cfg.K, bias=bias)
    ref, sel, G = bruteforce.dense_forward(x, wr, wg, wu, wd, cfg.K, bias=bias)
    assert np.array_equal(idx, sel)
    np.testing.assert_allclose(np.take_along_axis(G, idx.astype(np.int64), axis=1), w, rtol=2e-6)
    assert np.linalg.norm(out - ref) <= 1e-5 * np.linalg.norm(ref)
    np.testing.assert_allclose(out, ref, rtol=1e-4, atol=1e-6 * np.abs(ref).max())


def test_unfused_steps_compose_to_forward_and_sampled_tokens(oracle_lib):
    cfg = wl.small_config(21, 32, 6, 2, 16, seed=12, sigma_w=0.3)
    x, wr, wg, wu, wd = _rand(cfg)
    out, idx, w = oracle_lib.forward(x, wr, wg, wu, wd, cfg.K)
    idx2, w2 = oracle_lib.route_topk(x, wr, cfg.K)
    off, r2a, a2r = oracle_lib.permute(idx2, cfg.E)
    y = oracle_lib.grouped_swiglu(oracle_lib.gather_rows(x, r2a, cfg.K), off, wg, wu, wd)
    out2 = oracle_lib.combine(y, a2r, w2)
    assert np.array_equal(idx, idx2) and np.array_equal(w, w2) and np.array_equal(out, out2)
    tok = np.array([20, 0, 7], dtype=np.int32)
    rows = oracle_lib.forward_tokens(x, idx, w, wg, wu, wd, tok)
    np.testing.assert_allclose(rows, out[tok], rtol=1e-12, atol=1e-15)


def test_equivariance(oracle_lib):
    cfg = wl.small_config(12, 32, 6, 2, 16, seed=13, sigma_w=0.3)
    x, wr, wg, wu, wd = _rand(cfg)
    out, idx, w = oracle_lib.forward(x, wr, wg, wu, wd, cfg.K)
    rng = np.random.default_rng(14)
    pt = rng.permutation(cfg.T)
    out_p, idx_p, _ = oracle_lib.forward(x[pt], wr, wg, wu, wd, cfg.K)
    assert np.array_equal(idx_p, idx[pt]) and np.array_equal(out_p, out[pt])
    pe = rng.permutation(cfg.E)       # new expert j is old expert pe[j]
    out_e, idx_e, w_e = oracle_lib.forward(x, wr[pe], wg[pe], wu[pe], wd[pe], cfg.K)
    assert np.array_equal(pe[idx_e], idx) and np.array_equal(w_e, w)
    np.testing.assert_allclose(out_e, out, rtol=1e-12, atol=1e-15)


def test_zero_input_and_power_of_two_scaling(oracle_lib):
    cfg = wl.small_config(5, 32, 4, 2, 16, seed=15, sigma_w=0.3)
    x, wr, wg, wu, wd = _rand(cfg)
    out0, _, _ = oracle_lib.forward(np.zeros_like(x), wr, wg, wu, wd, cfg.K)
    assert np.all(out0 == 0.0)
    out, _, _ = oracle_lib.forward(x, wr, wg, wu, wd, cfg.K)
    out2, _, _ = oracle_lib.forward(x, wr, wg, wu, wd * np.float32(4.0), cfg.K)
    assert np.array_equal(out2, out * 4.0)


def test_hand_worked_example(oracle_lib):
    vals = {}
    with open(os.path.join(GOLDEN, "worked_example.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, *v = line.split()
            vals[k] = [float(t) for t in v]
    x = np.array([[1.0, 2.0]], dtype=np.float32)
    wr = np.eye(2, dtype=np.float32)
    wg = np.array([[[1.0, 0.0]], [[0.5, 0.5]]], dtype=np.float32)
    wu = np.array([[[0.0, 1.0]], [[1.0, -1.0]]], dtype=np.float32)
    wd = np.array([[[1.0], [1.0]], [[2.0], [-1.0]]], dtype=np.float32)
    s1 = 1.0 / (1.0 + math.exp(-1.0)) * 2.0
    s15 = -1.5 / (1.0 + math.exp(-1.5))
    y0, y1 = np.array([s1, s1]), np.array([2 * s15, -s15])
    out, idx, w = oracle_lib.forward(x, wr, wg, wu, wd, 1)
    assert idx.tolist() == [[int(vals["k1_idx"][0])]] and w.tolist() == [vals["k1_w"]]
    np.testing.assert_allclose(out[0], y1, rtol=1e-14)
    np.testing.assert_allclose(out[0], vals["k1_out"], rtol=0, atol=1e-9)
    out, idx, w = oracle_lib.forward(x, wr, wg, wu, wd, 2)
    w1 = 1.0 / (1.0 + math.exp(-1.0))
    assert idx.tolist() == [[int(v) for v in vals["k2_idx"]]]
    np.testing.assert_allclose(w[0], [w1, 1 - w1], rtol=1e-7)
    np.testing.assert_allclose(w[0], vals["k2_w"], rtol=0, atol=1e-7)
    np.testing.assert_allclose(out[0], float(w[0, 0]) * y1 + float(w[0, 1]) * y0, rtol=1e-14)
    np.testing.assert_allclose(out[0], vals["k2_out"], rtol=0, atol=1e-7)
