"""GPU parity: every entry point of the C ABI against the CPU oracle, element by
element on the same seeded inputs.  Integer results (expert ids, offsets, both
permutation maps, gathered rows) must be identical; floating-point results must
stay within max-abs 2e-2 and relative L2 1e-2 of the (unrounded, double) oracle.
"""
import numpy as np
import pytest
import torch

from paper_2511_11373_amd import moe
from paper_2511_11373_amd import workloads as wl
from tests.gpu_util import check_close, check_weights, host, shape_of, to_dev, upload

pytestmark = pytest.mark.gpu

SMALL = [
    wl.CONFIGS["tiny"],
    wl.small_config(1, 64, 4, 2, 32, dtype=wl.BF16, seed=1, sigma_w=0.1),          # one token
    wl.small_config(37, 72, 5, 3, 40, dtype=wl.BF16, seed=2, sigma_w=0.1),         # nothing divides a tile
    wl.small_config(130, 264, 6, 6, 136, dtype=wl.F32, seed=3, sigma_w=0.05),      # K == E, float storage
    wl.small_config(200, 128, 1, 1, 64, dtype=wl.BF16, seed=4, sigma_w=0.1),       # a single expert
    wl.small_config(700, 256, 70, 4, 96, dtype=wl.BF16, seed=5, sigma_w=0.05),     # E not a multiple of 64, 2800 rows
    wl.small_config(96, 512, 300, 8, 64, dtype=wl.BF16, seed=6, sigma_w=0.05),     # many experts, most nearly empty
    wl.small_config(40, 64, 1024, 16, 16, dtype=wl.BF16, seed=12, sigma_w=0.1),      # the largest expert count the library takes
    wl.small_config(600, 64, 1024, 16, 16, dtype=wl.F32, seed=13, sigma_w=0.1),      # ... with the multi-block permutation (9600 rows)
    wl.small_config(1500, 256, 70, 4, 64, dtype=wl.BF16, seed=10, sigma_w=0.05),   # large batch: matrix-core router, big GEMM off
    wl.small_config(2100, 256, 8, 2, 128, dtype=wl.BF16, seed=11, sigma_w=0.05),   # 525 rows per expert: big GEMM with ragged tiles
    wl.small_config(420, 256, 8, 2, 128, dtype=wl.BF16, seed=14, sigma_w=0.05),     # ~105 rows per expert: big GEMM, short tiles only
    wl.small_config(260, 256, 16, 2, 128, dtype=wl.BF16, seed=7, renormalize=False, sigma_w=0.05),
]


def _ids(cfgs):
    return [c.name + ("" if c.renormalize else "-norenorm") + "-" + c.dtype for c in cfgs]


@pytest.fixture(scope="module")
def lib():
    assert torch.cuda.is_available()
    return moe.load_library()


def _oracle_all(oracle_lib, cfg, d):
    idx, w = oracle_lib.route_topk(d["x_f32"], d["w_router_f32"], cfg.K, d["router_bias"], cfg.renormalize)
    off, r2a, a2r = oracle_lib.permute(idx, cfg.E)
    return idx, w, off, r2a, a2r


@pytest.mark.parametrize("cfg", SMALL + [wl.CONFIGS["decode64"]], ids=_ids(SMALL + [wl.CONFIGS["decode64"]]))
def test_each_entry_point_against_oracle(lib, oracle_lib, cfg):
    d = wl.make_inputs(cfg)
    g = upload(cfg, d)
    shp = shape_of(cfg)
    ws = moe.alloc_workspace(shp)
    o_idx, o_w, o_off, o_r2a, o_a2r = _oracle_all(oracle_lib, cfg, d)
    # The named configurations are held to the absolute bound of 2e-2; the hand-made small shapes draw weights five
    # times as large to exercise the tails, so their bound scales with the largest reference magnitude above 1.
    named = cfg.name in wl.CONFIGS

    def bound(ref, base=2e-2):
        return base if named else base * max(1.0, np.abs(ref).max())

    # route
    idx, w = moe.moe_route_topk(shp, g["x"], g["w_router"], g["router_bias"], ws)
    assert np.array_equal(host(idx), o_idx)
    check_weights(host(w), o_w)
    if cfg.renormalize:
        assert np.all(np.abs(host(w).astype(np.float64).sum(axis=1) - 1.0) <= 1e-6)

    # permute, fed with the oracle's selection so the step is checked on its own
    off, r2a, a2r, xp = moe.moe_permute(shp, torch.from_numpy(o_idx).cuda(), g["x"], ws)
    assert np.array_equal(host(off), o_off)
    assert np.array_equal(host(r2a), o_r2a)
    assert np.array_equal(host(a2r), o_a2r)
    o_xp = oracle_lib.gather_rows(d["x_f32"], o_r2a, cfg.K)
    assert np.array_equal(host(xp).astype(np.float32), o_xp)
    # permute then un-permute is the identity
    assert torch.equal(xp[a2r.long()], g["x"].repeat_interleave(cfg.K, dim=0))

    # grouped SwiGLU on the oracle's rows and offsets
    o_y = oracle_lib.grouped_swiglu(o_xp, o_off, d["w_gate_f32"], d["w_up_f32"], d["w_down_f32"])
    y = moe.moe_grouped_swiglu(shp, to_dev(d["x"][o_r2a // cfg.K], cfg.dtype), torch.from_numpy(o_off).cuda(),
                               g["w_gate"], g["w_up"], g["w_down"], ws)
    check_close(host(y), o_y, "y_perm", max_abs=bound(o_y))

    # combine on the GPU's own y_perm against the same sum in double
    out = moe.moe_combine(shp, y, torch.from_numpy(o_a2r).cuda(), torch.from_numpy(o_w).cuda())
    o_out_of_gpu_y = oracle_lib.combine(host(y), o_a2r, o_w)
    check_close(host(out), o_out_of_gpu_y, "combine", max_abs=bound(o_out_of_gpu_y, 1e-2), rel_l2=4e-3)

    # fused forward against the oracle's forward
    o_out = oracle_lib.combine(o_y, o_a2r, o_w)
    idx2 = torch.empty_like(idx)
    w2 = torch.empty_like(w)
    out2 = moe.moe_forward(shp, g["x"], g["w_router"], g["router_bias"], g["w_gate"], g["w_up"], g["w_down"], ws,
                           topk_idx_out=idx2, topk_w_out=w2)
    assert np.array_equal(host(idx2), o_idx)
    check_weights(host(w2), o_w)
    err, rel = check_close(host(out2), o_out, "forward", max_abs=bound(o_out))
    assert rel <= 6e-3      # what bf16 rounding of x, W, act, y and out should cost
    # forward without the optional outputs gives the same bits
    out3 = moe.moe_forward(shp, g["x"], g["w_router"], g["router_bias"], g["w_gate"], g["w_up"], g["w_down"], ws)
    assert torch.equal(out3, out2)


def test_tie_break_and_zero_input(lib, oracle_lib):
    cfg = wl.small_config(50, 128, 40, 8, 64, dtype=wl.BF16, seed=8, sigma_w=0.1)
    d = wl.make_inputs(cfg)
    g = upload(cfg, d)
    shp = shape_of(cfg)
    ws = moe.alloc_workspace(shp)
    idx, w = moe.moe_route_topk(shp, g["x"], torch.zeros_like(g["w_router"]), None, ws)
    assert np.array_equal(host(idx), np.tile(np.arange(cfg.K, dtype=np.int32), (cfg.T, 1)))
    assert np.all(host(w) == np.float32(1.0 / cfg.K))
    # duplicated router rows: exact ties inside every token, lower id first
    wr = d["w_router"].copy()
    wr[5] = wr[2]
    wr[39] = wr[2]
    idx, w = moe.moe_route_topk(shp, g["x"], to_dev(wr, cfg.dtype), None, ws)
    o_idx, o_w = oracle_lib.route_topk(d["x_f32"], wl.bf16_bits_to_f32(wr), cfg.K)
    assert np.array_equal(host(idx), o_idx)
    out = moe.moe_forward(shp, torch.zeros_like(g["x"]), g["w_router"], None, g["w_gate"], g["w_up"], g["w_down"], ws)
    assert torch.count_nonzero(out).item() == 0


def test_near_ties_go_through_the_exact_recheck(lib, oracle_lib):
    """Router rows that differ from each other by one bf16 ulp in a few places, and exact duplicates: the
    logits of such experts differ by far less than float accumulation error, so only an exact re-evaluation
    can order them.  Shapes on both the matrix-core fast path (T >= 1024, H % 256 == 0, E <= 128) and the fp64 path."""
    for (T, H, E, K, seed) in ((1100, 512, 96, 8, 21), (1025, 2048, 128, 8, 22), (300, 512, 96, 8, 24), (64, 384, 40, 6, 23),
                               (1030, 1792, 64, 8, 25), (1200, 768, 33, 33, 26), (1027, 256, 5, 1, 27)):
        cfg = wl.small_config(T, H, E, K, 64, dtype=wl.BF16, seed=seed, sigma_w=0.02)
        d = wl.make_inputs(cfg)
        wr = d["w_router"].copy()
        rng = np.random.default_rng(seed)
        for e in range(1, E):
            if e % 3 == 0:
                continue                                   # keep a third of the rows independent
            wr[e] = wr[e - 1]                              # a chain of near-copies
            if e % 3 == 1:
                cols = rng.integers(0, H, 3)
                wr[e, cols] = wr[e, cols] ^ np.uint16(1)   # flip the last mantissa bit: one ulp
        bias = (rng.standard_normal(E) * 1e-4).astype(np.float32) if seed == 22 else None
        shp = moe.make_shape(T, H, E, K, 64, moe.MOE_BF16)
        ws = moe.alloc_workspace(shp)
        idx, w = moe.moe_route_topk(shp, to_dev(d["x"], wl.BF16), to_dev(wr, wl.BF16),
                                    None if bias is None else torch.from_numpy(bias).cuda(), ws)
        o_idx, o_w = oracle_lib.route_topk(d["x_f32"], wl.bf16_bits_to_f32(wr), K, bias)
        assert np.array_equal(host(idx), o_idx), (T, H, E)
        check_weights(host(w), o_w)


def test_grouped_gemm_uneven_experts(lib, oracle_lib):
    """The large-batch GEMM on hand-made expert segments: experts without rows at the start, in the middle and at
    the end, segments of 1, 3, 256 and 257 rows, segments around the row counts at which a tile changes from one main loop
    to another (64, 65, 128, 129, 255), and one expert that holds most of the rows and therefore spans several of the
    per-XCD shares of the row-tile list."""
    counts = [0, 700, 64, 257, 256, 1, 65, 2500, 3, 128, 512, 129, 255, 0]      # 64 / 65 / 128 / 129: around the short-tile loops' limits
    n, H, I, E = sum(counts), 256, 128, len(counts)
    cfg = wl.small_config(n, H, E, 1, I, dtype=wl.BF16, seed=31, sigma_w=0.05)
    d = wl.make_inputs(cfg)
    g = upload(cfg, d)
    shp = shape_of(cfg)
    ws = moe.alloc_workspace(shp)
    off = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    y = moe.moe_grouped_swiglu(shp, g["x"], torch.from_numpy(off).cuda(), g["w_gate"], g["w_up"], g["w_down"], ws)
    o_y = oracle_lib.grouped_swiglu(d["x_f32"], off, d["w_gate_f32"], d["w_up_f32"], d["w_down_f32"])
    check_close(host(y), o_y, "y_perm", max_abs=2e-2 * max(1.0, np.abs(o_y).max()))


@pytest.mark.parametrize("n_long,n_short", [(7, 7), (8, 1), (9, 0), (1, 15), (5, 6), (0, 9), (16, 16), (3, 5)])
def test_grouped_gemm_tile_shares_over_the_xcds(lib, oracle_lib, n_long, n_short):
    """The large-batch GEMM's row tiles are dealt out to 8 lists (one per XCD), long tiles (more than 128 rows) and short
    ones separately, the larger shares of the short ones starting where those of the long ones end.  Numbers of long and
    short tiles around the multiples of 8, including none of a kind and a wrap of the short tiles' larger shares past the
    last list: every row of every expert against the oracle (a tile dealt out twice or not at all would show as wrong rows)."""
    rng = np.random.default_rng(1000 * n_long + n_short)
    counts = [int(c) for c in rng.integers(129, 257, n_long)] + [int(c) for c in rng.integers(1, 129, n_short)]
    rng.shuffle(counts)
    n, H, I, E = sum(counts), 256, 128, len(counts)
    if n < 60 * E:                                      # keep the batch on the large-batch kernel: pad with one big expert
        counts.append(60 * (E + 1) - n + 256)
        n, E = sum(counts), len(counts)
    cfg = wl.small_config(n, H, E, 1, I, dtype=wl.BF16, seed=33, sigma_w=0.05)
    d = wl.make_inputs(cfg)
    g = upload(cfg, d)
    shp = shape_of(cfg)
    ws = moe.alloc_workspace(shp)
    off = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    y = moe.moe_grouped_swiglu(shp, g["x"], torch.from_numpy(off).cuda(), g["w_gate"], g["w_up"], g["w_down"], ws)
    o_y = oracle_lib.grouped_swiglu(d["x_f32"], off, d["w_gate_f32"], d["w_up_f32"], d["w_down_f32"])
    check_close(host(y), o_y, "y_perm", max_abs=2e-2 * max(1.0, np.abs(o_y).max()))


def test_streaming_gemm_uneven_experts(lib, oracle_lib):
    """The decode-sized (weight-streaming) kernels on hand-made expert segments at the shape they are built for: experts
    without rows, with one row, with exactly 16, and with 17 and 33 rows (two and three passes of 16 tokens)."""
    counts = [0, 1, 17, 0, 16, 33, 5, 0, 2]
    n, H, I, E = sum(counts), 2048, 768, len(counts)
    assert n <= 12 * E                                       # the batch size up to which these kernels are selected
    cfg = wl.small_config(n, H, E, 1, I, dtype=wl.BF16, seed=32, sigma_w=0.02)
    d = wl.make_inputs(cfg)
    g = upload(cfg, d)
    shp = shape_of(cfg)
    ws = moe.alloc_workspace(shp)
    off = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    y = moe.moe_grouped_swiglu(shp, g["x"], torch.from_numpy(off).cuda(), g["w_gate"], g["w_up"], g["w_down"], ws)
    o_y = oracle_lib.grouped_swiglu(d["x_f32"], off, d["w_gate_f32"], d["w_up_f32"], d["w_down_f32"])
    check_close(host(y), o_y, "y_perm", max_abs=2e-2 * max(1.0, np.abs(o_y).max()))


def test_empty_batch_and_bad_arguments(lib):
    shp = moe.make_shape(0, 64, 4, 2, 32, moe.MOE_BF16)
    ws = moe.alloc_workspace(shp)
    x = torch.empty((0, 64), dtype=torch.bfloat16, device="cuda")
    wr = torch.zeros((4, 64), dtype=torch.bfloat16, device="cuda")
    wg = torch.zeros((4, 32, 64), dtype=torch.bfloat16, device="cuda")
    wd = torch.zeros((4, 64, 32), dtype=torch.bfloat16, device="cuda")
    out = torch.full((1, 64), 7.0, dtype=torch.bfloat16, device="cuda")
    moe.moe_forward(shp, wr, wr, None, wg, wg, wd, ws, out=out)      # x pointer unused when T == 0
    torch.cuda.synchronize()
    assert torch.all(out == 7.0)                                       # nothing was enqueued
    shp = moe.make_shape(4, 64, 4, 2, 32, moe.MOE_BF16)
    small_ws = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(moe.MoeError) as ei:
        moe.moe_forward(shp, wr, wr, None, wg, wg, wd, small_ws)
    assert ei.value.code == 4


def test_repeated_runs_are_bitwise_identical(lib):
    cfg = wl.small_config(333, 256, 24, 4, 128, dtype=wl.BF16, seed=9, sigma_w=0.05)
    d = wl.make_inputs(cfg)
    g = upload(cfg, d)
    shp = shape_of(cfg)
    ws = moe.alloc_workspace(shp)
    ref = None
    for _ in range(10):
        idx = torch.empty((cfg.T, cfg.K), dtype=torch.int32, device="cuda")
        out = moe.moe_forward(shp, g["x"], g["w_router"], None, g["w_gate"], g["w_up"], g["w_down"], ws, topk_idx_out=idx)
        cur = (out.clone(), idx.clone())
        if ref is None:
            ref = cur
        assert torch.equal(cur[0], ref[0]) and torch.equal(cur[1], ref[1])


FULL = ["decode512", "skew4k", "prefill16k"]


@pytest.mark.parametrize("name", FULL)
def test_full_size_forward_every_element(lib, oracle_lib, name):
    """Full-size layer shapes, in the launch configuration the benchmark times: routing ids, routing weights, offsets
    and both permutation maps of every token are compared exactly, and EVERY element of the block output against the
    oracle's forward pass, at the absolute bound of 2e-2 and relative L2 of 1e-2 (no scaling by the magnitude)."""
    cfg = wl.CONFIGS[name]
    d = wl.make_inputs(cfg)
    g = upload(cfg, d)
    shp = shape_of(cfg)
    ws = moe.alloc_workspace(shp)
    idx = torch.empty((cfg.T, cfg.K), dtype=torch.int32, device="cuda")
    w = torch.empty((cfg.T, cfg.K), dtype=torch.float32, device="cuda")
    out = moe.moe_forward(shp, g["x"], g["w_router"], g["router_bias"], g["w_gate"], g["w_up"], g["w_down"], ws,
                          topk_idx_out=idx, topk_w_out=w)
    o_out, o_idx, o_w = oracle_lib.forward(d["x_f32"], d["w_router_f32"], d["w_gate_f32"], d["w_up_f32"], d["w_down_f32"],
                                           cfg.K, bias=d["router_bias"], renormalize=cfg.renormalize)
    assert np.array_equal(host(idx), o_idx)
    check_weights(host(w), o_w)
    o_off, o_r2a, o_a2r = oracle_lib.permute(o_idx, cfg.E)
    off, r2a, a2r, _ = moe.moe_permute(shp, idx, g["x"], ws, want_x_perm=False)
    assert np.array_equal(host(off), o_off) and np.array_equal(host(r2a), o_r2a) and np.array_equal(host(a2r), o_a2r)
    got = host(out)
    err, rel = check_close(got, o_out, f"forward[{name}], all {cfg.T} tokens")
    assert rel <= 6e-3
    # no single token may be far off either (a wrong row would hide in the norm of 16384 good ones)
    tok_rel = np.linalg.norm(got - o_out, axis=1) / np.linalg.norm(o_out, axis=1)
    assert tok_rel.max() <= 2e-2, (int(tok_rel.argmax()), float(tok_rel.max()))


def test_full_size_expert_rows_every_element(lib, oracle_lib):
    """The grouped SwiGLU alone on the skewed batch (experts of a few rows next to experts of thousands, and empty
    ones): every element of every expert-sorted output row against the oracle."""
    cfg = wl.CONFIGS["skew4k"]
    d = wl.make_inputs(cfg)
    g = upload(cfg, d)
    shp = shape_of(cfg)
    ws = moe.alloc_workspace(shp)
    o_idx, o_w, o_off, o_r2a, o_a2r = _oracle_all(oracle_lib, cfg, d)
    o_xp = oracle_lib.gather_rows(d["x_f32"], o_r2a, cfg.K)
    o_y = oracle_lib.grouped_swiglu(o_xp, o_off, d["w_gate_f32"], d["w_up_f32"], d["w_down_f32"])
    y = moe.moe_grouped_swiglu(shp, to_dev(d["x"][o_r2a // cfg.K], cfg.dtype), torch.from_numpy(o_off).cuda(),
                               g["w_gate"], g["w_up"], g["w_down"], ws)
    got = host(y)
    check_close(got, o_y, "y_perm[skew4k], all rows")
    row_rel = np.linalg.norm(got - o_y, axis=1) / np.maximum(np.linalg.norm(o_y, axis=1), 1e-30)
    assert row_rel.max() <= 2e-2, (int(row_rel.argmax()), float(row_rel.max()))


def test_rows_past_32_bit_element_indices(lib, oracle_lib):
    """131072 tokens at the layer shape: 1 048 576 expert-sorted rows, 2.1e9 elements of y_perm - past what a 32-bit element
    index holds - and 512 row tiles per expert.  Routing and permutation of every token exactly; the output on sampled tokens,
    among them the tokens whose rows are the last ones of the sorted order."""
    cfg = wl.MoEConfig("prefill128k", 131072, 2048, 128, 8, 768, wl.BF16, seed=3)
    d = wl.make_inputs(cfg)
    g = upload(cfg, d)
    shp = shape_of(cfg)
    ws = moe.alloc_workspace(shp)
    idx = torch.empty((cfg.T, cfg.K), dtype=torch.int32, device="cuda")
    w = torch.empty((cfg.T, cfg.K), dtype=torch.float32, device="cuda")
    out = moe.moe_forward(shp, g["x"], g["w_router"], None, g["w_gate"], g["w_up"], g["w_down"], ws, topk_idx_out=idx, topk_w_out=w)
    o_idx, o_w, o_off, o_r2a, o_a2r = _oracle_all(oracle_lib, cfg, d)
    assert np.array_equal(host(idx), o_idx)
    check_weights(host(w), o_w)
    off, r2a, a2r, _ = moe.moe_permute(shp, idx, g["x"], ws, want_x_perm=False)
    assert np.array_equal(host(off), o_off) and np.array_equal(host(r2a), o_r2a) and np.array_equal(host(a2r), o_a2r)
    rng = np.random.default_rng(9)
    tok = np.concatenate([[0, cfg.T - 1], rng.integers(0, cfg.T, 90), o_r2a[-32:] // cfg.K, o_r2a[:4] // cfg.K])
    tok = np.unique(tok).astype(np.int32)
    ref = oracle_lib.forward_tokens(d["x_f32"], o_idx, o_w, d["w_gate_f32"], d["w_up_f32"], d["w_down_f32"], tok)
    got = host(out[torch.from_numpy(tok).long().cuda()])
    check_close(got, ref, "forward at 131072 tokens, sampled tokens")
    assert bool(torch.isfinite(out.float()).all().item())
