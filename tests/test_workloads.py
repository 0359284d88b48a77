"""The seeded input generators (CPU only): formats, determinism, distributions."""
import numpy as np
import torch

from paper_2511_11373_amd import workloads as wl


def test_bf16_rounding_matches_torch_and_round_trips():
    rng = np.random.default_rng(0)
    a = (rng.standard_normal(100000) * 10.0 ** rng.integers(-6, 4, 100000)).astype(np.float32)
    bits = wl.f32_to_bf16_bits(a)
    assert np.array_equal(bits, wl.f32_to_bf16_bits_numpy(a))
    ref = torch.from_numpy(a).to(torch.bfloat16)
    assert np.array_equal(bits, ref.view(torch.uint16).numpy())
    assert np.array_equal(wl.bf16_bits_to_f32(bits), ref.float().numpy())


def test_inputs_are_deterministic_and_distributed_as_stated():
    cfg = wl.CONFIGS["tiny"]
    a, b = wl.make_inputs(cfg), wl.make_inputs(cfg)
    for k in ("x", "w_router", "w_gate", "w_up", "w_down"):
        assert np.array_equal(a[k], b[k])
    assert a["x"].dtype == np.float32 and a["x"].shape == (64, 256)
    assert abs(a["x"].std() - 1.0) < 0.02 and abs(a["w_gate"].std() - 0.02) < 0.001
    assert a["router_bias"] is None
    c = wl.make_inputs(cfg, weight_set=1)
    assert np.array_equal(c["x"], a["x"]) and not np.array_equal(c["w_gate"], a["w_gate"])
    d = wl.make_inputs(wl.small_config(4, 64, 4, 2, 16, dtype=wl.BF16))
    assert d["x"].dtype == np.uint16 and np.array_equal(wl.bf16_bits_to_f32(d["x"]), d["x_f32"])


def test_zipf_target_and_bias():
    cfg = wl.CONFIGS["skew4k"]
    L = wl.zipf_target_load(cfg.T, cfg.K, cfg.E, cfg.zipf_s)
    assert abs(L.sum() - cfg.T * cfg.K) < 1e-3 * cfg.T and L.max() <= cfg.T and np.all(np.diff(L) <= 0)
    assert L[0] == cfg.T and L[1] == cfg.T and 2800 < L[2] < 3000 and 25 < L[-1] < 40
    b = wl.zipf_router_bias(cfg)
    assert b.shape == (cfg.E,) and b.dtype == np.float32 and np.array_equal(b, wl.zipf_router_bias(cfg))
    assert b.max() - b.min() > 2.0


def test_grpo_inputs():
    cfg = wl.GRPO_CONFIGS["logprob_small"]
    d = wl.make_grpo_inputs(cfg)
    assert d["logits"].shape == (cfg.N, cfg.V) and d["target"].min() >= 0 and d["target"].max() < cfg.V
    off = d["resp_offsets"]
    assert off[0] == 0 and off[-1] == cfg.N and np.all(np.diff(off) >= 0) and off.shape == (cfg.G + 1,)
    part = wl.make_grpo_inputs(cfg, rows=slice(100, 250))
    assert np.array_equal(part["logits"], d["logits"][100:250]) and np.array_equal(part["target"], d["target"])
    big = wl.GRPO_CONFIGS["logprob16k"]
    assert big.V % 8 == 0 and big.N == 16384 and big.G == 8
