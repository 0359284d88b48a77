"""GPU safety nets around the parity tests: routing under heavy cancellation, guard regions around every output and
the workspace, and bitwise repeatability of every kernel family."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2511_11373_amd import moe
from paper_2511_11373_amd import workloads as wl
from tests.gpu_util import check_weights, host, shape_of, to_dev, upload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lib():
    assert torch.cuda.is_available()
    return moe.load_library()


# ---- routing: near-equal exact logits from unrelated rows of large norm ---------------------------------------------
@pytest.mark.parametrize("T,H,E,K,amp,bias", [
    (1100, 2048, 128, 7, 4.0, False),     # matrix-core router with exact recheck; K odd: the boundary splits a twin pair
    (1030, 1024, 64, 8, 16.0, True),      # larger rows, with a bias
    (1200, 512, 96, 5, 1.0, False),
    (2048, 2048, 128, 8, 64.0, False),    # rows so large that nearly every expert has to be re-evaluated
    (300, 2048, 128, 7, 4.0, False),      # below 1024 tokens: the double-precision matrix-core path, k split over blocks
    (64, 1024, 64, 8, 16.0, True),
])
def test_router_under_heavy_cancellation(lib, oracle_lib, T, H, E, K, amp, bias):
    """Every router row carries large entries that cancel exactly in every token's logit, a different random set per
    row; rows e and e + E/2 then tie exactly or differ by far less than what float accumulation of the large entries
    leaves behind.  Only a selection made on exactly summed logits reproduces the oracle's ids."""
    xb, wb = wl.make_cancelling_router_inputs(T, H, E, seed=1000 + T + E, amp=amp)
    b = None
    if bias:
        b = (np.random.default_rng(T).standard_normal(E) * 1e-3).astype(np.float32)
        b[E // 2:] = b[:E // 2]                              # twins keep tying
    shp = moe.make_shape(T, H, E, K, 64, moe.MOE_BF16)
    ws = moe.alloc_workspace(shp)
    idx, w = moe.moe_route_topk(shp, to_dev(xb, wl.BF16), to_dev(wb, wl.BF16), None if b is None else torch.from_numpy(b).cuda(), ws)
    x32, w32 = wl.bf16_bits_to_f32(xb), wl.bf16_bits_to_f32(wb)
    o_idx, o_w = oracle_lib.route_topk(x32, w32, K, b)
    # the construction does what it says: in most tokens two of the K + 1 largest exact logits tie or nearly tie (with K
    # odd across the selection boundary, else between two slots), closer than the noise a float sum would carry
    logits = oracle_lib.router_logits(x32, w32, b)
    srt = -np.sort(-logits, axis=1)[:, :K + 1]
    assert np.mean(np.min(srt[:, :-1] - srt[:, 1:], axis=1) <= 1e-5 * amp) > 0.5
    assert np.array_equal(host(idx), o_idx)
    check_weights(host(w), o_w)


# ---- guard regions ---------------------------------------------------------------------------------------------------
GUARD = 4096
PATTERN = 0xA5


class Guarded:
    """A device buffer of `nbytes` with GUARD bytes of a known pattern before and after it."""

    def __init__(self, nbytes: int):
        self.nbytes = int(nbytes)
        pad = (-self.nbytes) % 256
        self.raw = torch.full((GUARD + self.nbytes + pad + GUARD,), PATTERN, dtype=torch.uint8, device="cuda")
        self.body = self.raw[GUARD:GUARD + self.nbytes]

    def view(self, dtype, shape):
        return self.body.view(dtype).view(shape)

    def intact(self) -> bool:
        torch.cuda.synchronize()
        return bool(torch.all(self.raw[:GUARD] == PATTERN).item() and torch.all(self.raw[GUARD + self.nbytes:] == PATTERN).item())


GUARD_SHAPES = [
    wl.small_config(37, 72, 5, 3, 40, dtype=wl.BF16, seed=2, sigma_w=0.1),        # tiled kernel, nothing divides a tile
    wl.small_config(61, 2048, 16, 2, 768, dtype=wl.BF16, seed=51),                # weight-streaming kernels
    wl.small_config(2100, 256, 8, 2, 128, dtype=wl.BF16, seed=11, sigma_w=0.05),  # large-batch GEMM, ragged tiles, fast router
    wl.small_config(601, 64, 1024, 16, 16, dtype=wl.F32, seed=13, sigma_w=0.1),   # multi-block permutation, float storage
]


@pytest.mark.parametrize("cfg", GUARD_SHAPES, ids=[c.name + "-" + c.dtype for c in GUARD_SHAPES])
def test_nothing_is_written_outside_outputs_and_workspace(lib, cfg):
    """Every output buffer and the workspace sit between guard regions filled with a byte pattern; the workspace is
    exactly moe_workspace_bytes() long.  After each entry point all guards must be untouched."""
    d = wl.make_inputs(cfg, want_f32=False)
    g = upload(cfg, d)
    shp = shape_of(cfg)
    elt = 2 if cfg.dtype == wl.BF16 else 4
    tdt = torch.bfloat16 if cfg.dtype == wl.BF16 else torch.float32
    T, K, H, E = cfg.T, cfg.K, cfg.H, cfg.E
    n = T * K
    ws = Guarded(moe.workspace_bytes(shp))
    idx, w = Guarded(n * 4), Guarded(n * 4)
    off, r2a, a2r = Guarded((E + 1) * 4), Guarded(n * 4), Guarded(n * 4)
    xp, y, out = Guarded(n * H * elt), Guarded(n * H * elt), Guarded(T * H * elt)
    bufs = dict(ws=ws, idx=idx, w=w, off=off, r2a=r2a, a2r=a2r, xp=xp, y=y, out=out)
    vp = ctypes.c_void_p

    def p(b):
        return vp(b.body.data_ptr())

    def t(x):
        return None if x is None else vp(x.data_ptr())

    def ok(what, rc):
        assert rc == 0, (what, rc)
        bad = [k for k, b in bufs.items() if not b.intact()]
        assert not bad, f"{what} wrote outside {bad}"

    st = vp(torch.cuda.current_stream().cuda_stream)
    sref = ctypes.byref(shp)
    ok("moe_route_topk", lib.moe_route_topk(sref, t(g["x"]), t(g["w_router"]), t(g["router_bias"]), p(idx), p(w), p(ws), ws.nbytes, st))
    ok("moe_permute", lib.moe_permute(sref, p(idx), t(g["x"]), p(off), p(r2a), p(a2r), p(xp), p(ws), ws.nbytes, st))
    ok("moe_grouped_swiglu", lib.moe_grouped_swiglu(sref, p(xp), p(off), t(g["w_gate"]), t(g["w_up"]), t(g["w_down"]), p(y), p(ws), ws.nbytes, st))
    ok("moe_combine", lib.moe_combine(sref, p(y), p(a2r), p(w), p(out), st))
    first = out.view(tdt, (T, H)).clone()
    ok("moe_forward", lib.moe_forward(sref, t(g["x"]), t(g["w_router"]), t(g["router_bias"]), t(g["w_gate"]), t(g["w_up"]), t(g["w_down"]),
                                     p(out), p(idx), p(w), p(ws), ws.nbytes, st))
    # the separate calls and the fused call agree closely (the fused call gathers inside the GEMM: same arithmetic)
    assert torch.allclose(out.view(tdt, (T, H)).float(), first.float(), rtol=0, atol=1e-6 + 2e-2 * float(first.float().abs().max()))


# ---- repeatability ------------------------------------------------------------------------------------------------------
FAMILIES = {
    "streaming GEMM, fp64 router, one-block permutation": wl.small_config(64, 2048, 16, 2, 768, dtype=wl.BF16, seed=61),
    "tiled GEMM": wl.small_config(333, 256, 24, 4, 128, dtype=wl.BF16, seed=9, sigma_w=0.05),
    "tiled GEMM, float storage, multi-block permutation": wl.small_config(600, 64, 1024, 16, 16, dtype=wl.F32, seed=13, sigma_w=0.1),
    "large-batch GEMM, fast router": wl.small_config(2100, 256, 8, 2, 128, dtype=wl.BF16, seed=11, sigma_w=0.05),
    "fast router, multi-block permutation, tiled GEMM": wl.small_config(2500, 256, 70, 4, 64, dtype=wl.BF16, seed=10, sigma_w=0.05),
}


@pytest.mark.parametrize("family", list(FAMILIES), ids=[k.replace(" ", "_").replace(",", "") for k in FAMILIES])
def test_twenty_runs_give_the_same_bits(lib, family):
    """Races in LDS, results that depend on the order of atomics or on which block finishes first would show up as bits
    that differ between runs.  Twenty runs of the whole block and of the separate permutation per kernel family."""
    cfg = FAMILIES[family]
    d = wl.make_inputs(cfg, want_f32=False)
    g = upload(cfg, d)
    shp = shape_of(cfg)
    ws = moe.alloc_workspace(shp)
    ref = None
    for run in range(20):
        idx = torch.empty((cfg.T, cfg.K), dtype=torch.int32, device="cuda")
        w = torch.empty((cfg.T, cfg.K), dtype=torch.float32, device="cuda")
        ws.fill_(run)                                     # whatever the last run left behind must not matter
        out = moe.moe_forward(shp, g["x"], g["w_router"], g["router_bias"], g["w_gate"], g["w_up"], g["w_down"], ws,
                              topk_idx_out=idx, topk_w_out=w)
        off, r2a, a2r, xp = moe.moe_permute(shp, idx, g["x"], ws)
        y = moe.moe_grouped_swiglu(shp, xp, off, g["w_gate"], g["w_up"], g["w_down"], ws)
        cur = (out, idx, w, off, r2a, a2r, y)
        torch.cuda.synchronize()
        if ref is None:
            ref = cur
        for a, b in zip(cur, ref):
            assert torch.equal(a, b), (family, run)


BW_FAMILIES = {
    "LDS-pipelined backward GEMMs": wl.small_config(300, 256, 16, 4, 128, dtype=wl.BF16, seed=43, sigma_w=0.05),
    "LDS-free backward GEMMs": wl.small_config(37, 72, 5, 3, 40, dtype=wl.BF16, seed=42, sigma_w=0.1),
}


@pytest.mark.parametrize("family", list(BW_FAMILIES), ids=[k.replace(" ", "_") for k in BW_FAMILIES])
def test_twenty_backward_runs_give_the_same_bits(lib, family):
    from paper_2511_11373_amd import moe_backward as mb
    cfg = BW_FAMILIES[family]
    d = wl.make_inputs(cfg, want_f32=False)
    g = upload(cfg, d)
    rng = np.random.default_rng(cfg.seed)
    d_out = to_dev(wl.f32_to_bf16_bits(rng.standard_normal((cfg.T, cfg.H)).astype(np.float32)), wl.BF16)
    shp = shape_of(cfg)
    ws = mb.alloc_workspace(shp)
    ref = None
    for run in range(20):
        ws.fill_(run)
        out = mb.moe_backward(shp, g["x"], g["w_router"], None, g["w_gate"], g["w_up"], g["w_down"], d_out, ws)
        torch.cuda.synchronize()
        if ref is None:
            ref = out
        for name in out:
            assert torch.equal(out[name], ref[name]), (family, run, name)


def test_forward_replays_from_a_hip_graph(lib, oracle_lib):
    """A serving loop captures the decode step once and replays it: every entry point only enqueues kernels on the caller's
    stream (no allocation, no synchronisation, no memset, no event), so the whole block records into a HIP graph.  Replays
    with the program's own eager work and synchronisations in between, on inputs changed in place, must give what an eager
    call gives; both the workspace form and the form on the library's static scratch."""
    cfg = wl.small_config(64, 2048, 16, 2, 768, dtype=wl.BF16, seed=71)
    d = wl.make_inputs(cfg, want_f32=False)
    g = upload(cfg, d)
    shp = shape_of(cfg)
    ws = moe.alloc_workspace(shp)
    x = g["x"].clone()
    outs = {"workspace": torch.empty_like(x), "static scratch": torch.empty_like(x)}
    idx = torch.empty((cfg.T, cfg.K), dtype=torch.int32, device="cuda")
    moe.moe_forward_noalloc(shp, x, g["w_router"], None, g["w_gate"], g["w_up"], g["w_down"], outs["static scratch"])   # symbol lookup happens here, not under capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        moe.moe_forward(shp, x, g["w_router"], None, g["w_gate"], g["w_up"], g["w_down"], ws, out=outs["workspace"], topk_idx_out=idx)
        moe.moe_forward_noalloc(shp, x, g["w_router"], None, g["w_gate"], g["w_up"], g["w_down"], outs["static scratch"])
    rng = np.random.default_rng(5)
    for replay in range(4):
        new_x = to_dev(wl.f32_to_bf16_bits(rng.standard_normal((cfg.T, cfg.H)).astype(np.float32)), wl.BF16)
        x.copy_(new_x)
        for o in outs.values():
            o.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        eager = moe.moe_forward(shp, new_x, g["w_router"], None, g["w_gate"], g["w_up"], g["w_down"], moe.alloc_workspace(shp))
        torch.cuda.synchronize()
        for name, o in outs.items():
            assert torch.equal(o, eager), (name, replay)
