"""Helpers for the GPU parity tests: upload seeded inputs, run the library, compare."""
from __future__ import annotations

import numpy as np
import torch

from paper_2511_11373_amd import moe
from paper_2511_11373_amd import workloads as wl

MAX_ABS_TOL = 2e-2     # bf16 products, float accumulation: bound on |out - oracle|
REL_L2_TOL = 1e-2      # bound on ||out - oracle||_2 / ||oracle||_2
W_ATOL, W_RTOL = 1e-6, 1e-5   # routing weights (float): |dw| <= atol + rtol * w


def to_dev(a: np.ndarray, dtype: str) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype == wl.BF16:
        t = t.view(torch.bfloat16)
    return t.cuda()


def upload(cfg: wl.MoEConfig, d: dict) -> dict:
    g = {k: to_dev(d[k], cfg.dtype) for k in ("x", "w_router", "w_gate", "w_up", "w_down")}
    g["router_bias"] = None if d["router_bias"] is None else torch.from_numpy(d["router_bias"]).cuda()
    return g


def shape_of(cfg: wl.MoEConfig) -> moe.MoeShape:
    return moe.make_shape(cfg.T, cfg.H, cfg.E, cfg.K, cfg.I, moe.MOE_BF16 if cfg.dtype == wl.BF16 else moe.MOE_F32,
                          cfg.renormalize)


def host(t: torch.Tensor) -> np.ndarray:
    torch.cuda.synchronize()
    if t.dtype == torch.bfloat16:
        return t.float().cpu().numpy().astype(np.float64)
    return t.cpu().numpy()


def check_close(got: np.ndarray, ref: np.ndarray, what: str, max_abs=MAX_ABS_TOL, rel_l2=REL_L2_TOL):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), what
    err = np.abs(got - ref).max() if got.size else 0.0
    nrm = np.linalg.norm(ref)
    rel = np.linalg.norm(got - ref) / nrm if nrm > 0 else np.linalg.norm(got - ref)
    assert err <= max_abs, f"{what}: max-abs error {err:.3e} > {max_abs}"
    assert rel <= rel_l2, f"{what}: relative L2 error {rel:.3e} > {rel_l2}"
    return err, rel


def check_weights(got: np.ndarray, ref: np.ndarray):
    assert np.all(np.abs(got.astype(np.float64) - ref.astype(np.float64)) <= W_ATOL + W_RTOL * np.abs(ref))
