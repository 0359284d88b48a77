#!/usr/bin/env python3
"""Benchmark of the routed-expert MoE FFN block on one MI355X.

One step = one moe_forward (router, permutation, grouped SwiGLU, combine) over one
synthetic batch at the Qwen3-30B-A3B layer shape, inputs resident in HBM.  Prints
ONE JSON line.  The default workload is the rollout decode step of 64 concurrent
responses; --workload selects the other shapes.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload decode64]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published
WEIGHT_SETS = 4                # expert-weight sets rotated between steps (4 x 1.2 GB > 256 MB last-level cache)
DEFAULT_STEPS = {"tiny": 200, "decode64": 400, "decode512": 300, "prefill16k": 40, "skew4k": 100}
HBM_BOUND = ("decode64", "decode512")
# HBM traffic of the gate/up kernel per launch, from `rocprofv3 --pmc FETCH_SIZE` and `--pmc WRITE_SIZE` runs of this
# script (KiB per dispatch, averaged), scaled by what the same counters read for a plain 393216 KiB copy kernel in
# the same runs (FETCH_SIZE 196652 -> x2.0, WRITE_SIZE 393216 -> x1.0).  Valid only for the kernel source whose
# hash is recorded; after any change to that file the bench reports null until the counters are taken again.
TRAFFIC = {
    "decode64": {"source": "grouped_swiglu_stream.hip", "sha256_16": "ba3da780065582d9",
                 "fetch_kib": 385073.1, "write_kib": 790.2, "fetch_scale": 2.0, "write_scale": 1.0},
    "decode512": {"source": "grouped_swiglu.hip", "sha256_16": "530109aef8ce97ee",
                  "fetch_kib": 398853.9, "write_kib": 6172.7, "fetch_scale": 2.0, "write_scale": 1.0},
    "skew4k": {"source": "grouped_swiglu_big.hip", "sha256_16": "c7946880602b4339",
               "fetch_kib": 636461.6, "write_kib": 49153.5, "fetch_scale": 2.0, "write_scale": 1.0},
    "attn64": {"source": "attn_decode.hip", "sha256_16": "e8bc56f296527f59",
               "fetch_kib": 4023095.8, "write_kib": 9335.4, "fetch_scale": 2.0, "write_scale": 1.0},
    "logprob16k": {"source": "grpo.hip", "sha256_16": "1d6b06c37e215813",
                   "fetch_kib": 2432523.5, "write_kib": 515.8, "fetch_scale": 2.0, "write_scale": 1.0},
    "prefill16k": {"source": "grouped_swiglu_big.hip", "sha256_16": "c7946880602b4339",
                   "fetch_kib": 1360715.3, "write_kib": 196609.2, "fetch_scale": 2.0, "write_scale": 1.0},
}


def measured_traffic(workload):
    """Bytes per launch from the recorded counters, or None when the kernel has changed since."""
    import hashlib
    rec = TRAFFIC.get(workload)
    if rec is None:
        return None
    src = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2511_11373_amd", "csrc", rec["source"])
    try:
        digest = hashlib.sha256(open(src, "rb").read()).hexdigest()[:16]
    except OSError:
        return None
    if digest != rec["sha256_16"]:
        return None
    return int((rec["fetch_kib"] * rec["fetch_scale"] + rec["write_kib"] * rec["write_scale"]) * 1024)



def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="decode64",
                    choices=["tiny", "decode64", "decode512", "prefill16k", "skew4k", "logprob16k", "backward16k", "sched", "attn64"])
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip timing the CPU oracle")
    ap.add_argument("--no-prefill-record", action="store_true",
                    help="decode64 only: skip the prefill16k sub-record (layer.prefill16k) measured in the same run")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    return ap.parse_args()


def bench_logprob(args):
    """The next row of the path: token log-probabilities + GRPO objective over one 16k-token group (Eq. 1-3).
    One step = one grpo_logprob_objective call; bound by reading the [N, V] logits once from HBM."""
    import torch
    from paper_2511_11373_amd import grpo
    from paper_2511_11373_amd import workloads as wl
    cfg = wl.GRPO_CONFIGS["logprob16k"]
    steps = args.steps if args.steps is not None else 50
    warmup = args.warmup if args.warmup is not None else 5
    d = wl.make_grpo_inputs(cfg, rows=slice(0, 512))          # everything but the logits; 512 host rows for the oracle
    dev = {k: torch.from_numpy(d[k]).cuda() for k in ("target", "resp_offsets", "rewards", "logp_old", "logp_ref")}
    # the 5 GB logits tensor is drawn on the device (same law as the host generator: N(0, s^2), target raised by 2s);
    # its first 512 rows are overwritten with the host generator's so that the oracle sees identical values
    gen = torch.Generator(device="cuda")
    gen.manual_seed(cfg.seed)
    logits = torch.empty((cfg.N, cfg.V), dtype=torch.bfloat16, device="cuda")
    for r0 in range(0, cfg.N, 1024):
        blk = torch.randn((1024, cfg.V), device="cuda", generator=gen) * cfg.logit_scale
        idx = dev["target"][r0:r0 + 1024].long()
        blk[torch.arange(1024, device="cuda"), idx] += 2.0 * cfg.logit_scale
        logits[r0:r0 + 1024] = blk.to(torch.bfloat16)
    logits[:512] = torch.from_numpy(d["logits"]).view(torch.bfloat16).cuda()
    shp = grpo.make_shape(cfg.N, cfg.V, cfg.G, logits.dtype, cfg.clip_eps, cfg.beta, cfg.adv_eps)
    out = grpo.grpo_logprob_objective(shp, logits, dev["target"], dev["logp_old"], dev["logp_ref"], dev["rewards"], dev["resp_offsets"])

    def step():
        grpo.grpo_logprob_objective(shp, logits, dev["target"], dev["logp_old"], dev["logp_ref"], dev["rewards"],
                                    dev["resp_offsets"], out=out)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    # the dominant kernel alone (grpo_token_logprob is exactly that kernel), HIP events on the launch stream
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    lp = grpo.grpo_token_logprob(shp, logits, dev["target"])
    torch.cuda.synchronize()
    e0.record()
    for _ in range(steps):
        grpo.grpo_token_logprob(shp, logits, dev["target"])
    e1.record()
    torch.cuda.synchronize()
    k_ms = e0.elapsed_time(e1) / steps
    nbytes = cfg.N * cfg.V * 2 + cfg.N * 8
    ach = nbytes / (k_ms * 1e-3) / 1e9
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import grpo_oracle as go
        n = 512
        c0 = time.perf_counter()
        reps = 0
        while time.perf_counter() - c0 < args.cpu_seconds:
            o_logp = go.token_logprob(d["logits_f32"], d["target"][:n])
            reps += 1
        dt = time.perf_counter() - c0
        err = float(np.abs(out[0][:n].cpu().numpy().astype(np.float64) - o_logp).max())
        cpu = {"value": round(n * reps / dt, 2), "unit": "tokens/s", "cores": 1, "kind": "oracle",
               "sample": f"log-probs of the first {n} of {cfg.N} rows, {reps} pass(es), {dt:.1f} s (numpy, float64)",
               "max_abs_logp_err_gpu_vs_oracle": err}
    rec = {
        "metric": "log-prob + GRPO-objective tokens/s + % HBM BW", "value": round(cfg.N / (ms_per_step * 1e-3), 1),
        "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": cfg.name, "tokens": cfg.N, "vocab": cfg.V, "responses": cfg.G, "logits_dtype": "bf16"},
        "roofline": {"bound": "hbm", "kernel": "logprob_kernel", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": measured_traffic("logprob16k"),
                     "bytes_per_launch": int(nbytes), "avg_launch_ms": round(k_ms, 5)},
        "cpu_baseline": cpu,
        "objective": float(out[4].item()),
    }
    print(json.dumps(rec))


def bench_backward(args):
    """Another row of the path: the block's backward pass at the trainer's batch (Section 4.1: the policy is
    optimised with AdamW, so every RL step differentiates this layer).  One step = one moe_backward call on the
    prefill16k inputs and a random upstream gradient; bound by the bf16 matrix cores."""
    import torch
    from paper_2511_11373_amd import moe, moe_backward as mb
    from paper_2511_11373_amd import workloads as wl
    cfg = wl.CONFIGS["prefill16k"]
    steps = args.steps if args.steps is not None else 10
    warmup = args.warmup if args.warmup is not None else 2
    want_cpu = not args.no_cpu_baseline
    d = wl.make_inputs(cfg, want_f32=want_cpu)

    def dev(a):
        return torch.from_numpy(a).view(torch.bfloat16).cuda()
    x, wr, wg, wu, wd = (dev(d[k]) for k in ("x", "w_router", "w_gate", "w_up", "w_down"))
    rng = np.random.default_rng(cfg.seed + 1000)
    do_f32 = rng.standard_normal((cfg.T, cfg.H), dtype=np.float32)
    do_bits = wl.f32_to_bf16_bits(do_f32)
    d_out = dev(do_bits)
    shp = moe.make_shape(cfg.T, cfg.H, cfg.E, cfg.K, cfg.I, moe.MOE_BF16, True)
    ws = mb.alloc_workspace(shp)
    out = mb.moe_backward(shp, x, wr, None, wg, wu, wd, d_out, ws)
    for _ in range(warmup):
        mb.moe_backward(shp, x, wr, None, wg, wu, wd, d_out, ws, out=out)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        mb.moe_backward(shp, x, wr, None, wg, wu, wd, d_out, ws, out=out)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    # the other choice: the forward pass keeps g and u, the backward pass reads them (same gradients, bit for bit)
    fws = moe.alloc_workspace(shp)
    k_idx = torch.empty((cfg.T, cfg.K), dtype=torch.int32, device="cuda")
    k_w = torch.empty((cfg.T, cfg.K), dtype=torch.float32, device="cuda")
    fout, g_rows, u_rows = mb.moe_forward_saving(shp, x, wr, None, wg, wu, wd, fws, topk_idx_out=k_idx, topk_w_out=k_w)
    fwd_plain = moe.moe_forward(shp, x, wr, None, wg, wu, wd, fws)
    pair = {}
    for name, fn in (("forward_ms", lambda: moe.moe_forward(shp, x, wr, None, wg, wu, wd, fws, out=fwd_plain)),
                     ("forward_saving_ms", lambda: mb.moe_forward_saving(shp, x, wr, None, wg, wu, wd, fws, out=fout, g_rows=g_rows, u_rows=u_rows,
                                                                         topk_idx_out=k_idx, topk_w_out=k_w)),
                     ("backward_saved_ms", lambda: mb.moe_backward_saved(shp, x, wr, None, wg, wu, wd, d_out, g_rows, u_rows, ws, out=out,
                                                                         topk_idx=k_idx, topk_w=k_w))):
        fn()
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        pair[name] = round((time.perf_counter() - c0) * 1e3 / steps, 5)
    stage = np.zeros(mb.NUM_STAGES)
    n_prof = max(3, min(steps, 10))
    for _ in range(n_prof):
        stage += np.array(mb.moe_backward_stage_times(shp, x, wr, None, wg, wu, wd, d_out, ws, out))
    stage /= n_prof
    stages_ms = {n: round(float(v), 5) for n, v in zip(mb.STAGE_NAMES, stage)}
    empty = stage[mb.STAGE_NAMES.index("empty_interval")]
    # the dominant kernel: the weight-gradient GEMM (three launches per step, each 2 * T*K * H * I flop)
    wg_ms = float(np.mean([stage[mb.STAGE_NAMES.index(k)] for k in ("d_w_down", "d_w_gate", "d_w_up")]) - empty)
    wg_flops = 2.0 * cfg.T * cfg.K * cfg.H * cfg.I
    ach = wg_flops / (wg_ms * 1e-3) / 1e12
    step_flops = 8 * wg_flops          # g, u, d_out Wd, two products for the row gradients, three weight gradients
    cpu = None
    if want_cpu:
        import oracle
        from oracle import moe_backward_oracle as bwd
        n = cfg.T
        c0 = time.perf_counter()
        o_idx, _ = oracle.route_topk(d["x_f32"][:n], d["w_router_f32"], cfg.K)
        ref = bwd.backward(d["x_f32"][:n], d["w_router_f32"], None, d["w_gate_f32"], d["w_up_f32"], d["w_down_f32"], o_idx,
                           wl.bf16_bits_to_f32(do_bits[:n]), True)
        dt = time.perf_counter() - c0
        try:
            from threadpoolctl import threadpool_info
            cores = max([1] + [int(p.get("num_threads", 1)) for p in threadpool_info()])      # numpy's BLAS threads
        except Exception:
            cores = 1
        cpu = {"value": round(n / dt, 2), "unit": "tokens/s", "cores": cores, "kind": "oracle",
               "sample": f"backward of the first {n} of {cfg.T} tokens as a batch of their own, 1 pass, {dt:.1f} s (numpy, float64)"}
        # sanity of the timed path on the same sample: d_x of a token does not depend on the other tokens of the batch
        got = out["d_x"][:n].float().cpu().numpy().astype(np.float64)
        cpu["rel_l2_dx_gpu_vs_oracle"] = round(float(np.linalg.norm(got - ref["d_x"]) / max(np.linalg.norm(ref["d_x"]), 1e-30)), 6)
    rec = {
        "metric": "MoE-layer backward tokens/s + % bf16 MFMA peak", "value": round(cfg.T / (ms_per_step * 1e-3), 1),
        "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "backward16k", "tokens": cfg.T, "hidden": cfg.H, "experts": cfg.E, "top_k": cfg.K,
                   "intermediate": cfg.I},
        "roofline": {"bound": "mfma", "kernel": "weight-gradient GEMM (bw_lds_kernel<true>)", "achieved": round(ach, 1), "peak": MFMA_BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(ach / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None,
                     "flops_per_launch": wg_flops, "avg_launch_ms": round(wg_ms, 5)},
        "cpu_baseline": cpu,
        "layer": {"algorithmic_GFLOP": round(step_flops / 1e9, 2),
                  "mfma_frac_whole_step": round(step_flops / (ms_per_step * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                  "stages_ms": stages_ms,
                  "with_saved_pre_activations": dict(pair, backward_recomputing_ms=round(ms_per_step, 5))},
    }
    print(json.dumps(rec))


def bench_attn(args):
    """Another row of the path: one decode step of attention for 64 sequences at the paper's context lengths (Section
    4.1: 32k-token inputs, outputs of up to 64k tokens), Qwen3-30B-A3B head geometry (32 query heads, 4 key/value heads,
    head size 128), paged bf16 cache.  One step = one attn_decode call; bound by reading the cache once from HBM."""
    import torch
    from paper_2511_11373_amd import attn
    from paper_2511_11373_amd import workloads as wl
    cfg = wl.ATTN_CONFIGS["attn64"]
    B, Hq, Hkv, D = cfg.B, cfg.Hq, cfg.Hkv, cfg.D
    steps = args.steps if args.steps is not None else 30
    warmup = args.warmup if args.warmup is not None else 3
    lens, table, n_pages = wl.attn_lengths_and_table(cfg)          # a 32k prompt plus an output somewhere on its way to 64k
    max_pages = table.shape[1]
    q, k_pages, v_pages = wl.attn_device_inputs(cfg, n_pages)
    shp = attn.make_shape(B, Hq, Hkv, max_pages, n_pages)
    ws = attn.alloc_workspace(shp)
    tab_d, len_d = torch.from_numpy(table).cuda(), torch.from_numpy(lens).cuda()
    out = attn.attn_decode(shp, q, k_pages, v_pages, tab_d, len_d, ws)
    for _ in range(warmup):
        attn.attn_decode(shp, q, k_pages, v_pages, tab_d, len_d, ws, out=out)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        attn.attn_decode(shp, q, k_pages, v_pages, tab_d, len_d, ws, out=out)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        attn.attn_decode(shp, q, k_pages, v_pages, tab_d, len_d, ws, out=out)
    e1.record()
    torch.cuda.synchronize()
    k_ms = e0.elapsed_time(e1) / steps          # all three kernels of the call; the streaming kernel is ~99 % of it
    nbytes = int(lens.astype(np.int64).sum()) * Hkv * D * 2 * 2 + B * Hq * D * 2 * 2
    ach = nbytes / (k_ms * 1e-3) / 1e9
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import attn_oracle as ao
        b = int(np.argmin(lens))
        n = int(lens[b])
        kb, vb = wl.attn_sequence_to_host(cfg, k_pages, v_pages, table, lens, b)
        qb = q[b].float().cpu().numpy()
        c0 = time.perf_counter()
        reps = 0
        while time.perf_counter() - c0 < args.cpu_seconds:
            ref = ao.decode_attention(qb[None], kb[None], vb[None], [n])
            reps += 1
        dt = time.perf_counter() - c0
        got = out[b].float().cpu().numpy().astype(np.float64)
        cpu = {"value": round(reps / dt, 3), "unit": "tokens/s", "cores": 1, "kind": "oracle",
               "sample": f"the shortest of the 64 sequences ({n} positions), {reps} pass(es), {dt:.1f} s (numpy, float64)",
               "rel_l2_gpu_vs_oracle": round(float(np.linalg.norm(got - ref[0]) / np.linalg.norm(ref[0])), 6)}
    print(json.dumps({
        "metric": "decode-attention tokens/s + % HBM BW", "value": round(B / (ms_per_step * 1e-3), 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "attn64", "sequences": B, "query_heads": Hq, "kv_heads": Hkv, "head_size": D,
                   "context_min": int(lens.min()), "context_mean": int(lens.mean()), "context_max": int(lens.max()), "cache_GB": round(nbytes / 1e9, 2)},
        "roofline": {"bound": "hbm", "kernel": "attn_stream_kernel", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": measured_traffic("attn64"), "bytes_per_launch": nbytes,
                     "avg_launch_ms": round(k_ms, 5)},
        "cpu_baseline": cpu}))


def bench_sched(args):
    """Host-only row: the agentic rollout scheduling simulator (Sections 2.3, 3.1-3.4) on a synthetic long-tailed length
    mix with the paper's settings (groups of 8, two picks per agent, 64k-token outputs).  One step = one simulation of
    512 problems; reported: simulated sequences per second of the native simulator, the Python oracle beside it, and
    what the simulation says about the schedules."""
    from paper_2511_11373_amd import sched
    one = 1 << 24
    cfg = dict(problems=512, group_size=8, n_select=2, segment=16384, capacity=2048, strategy=sched.ADAPTIVE, pipeline=1, seed=2511,
               adv_eps=1e-6, short_lo=[2000, 1000, 2000, 1000, 2000], short_hi=[16000, 8000, 16000, 8000, 16000],
               long_hi=[65536] * 5, p_long=[one // 8] * 5, p_correct=[one * 2 // 5, 0, one // 2, 0, one // 2],
               p_keep=[0, 0, one * 9 // 10, 0, one * 9 // 10], p_flag_wrong=[0, one * 7 // 10, 0, one * 3 // 4, 0],
               p_flag_right=[0, one // 5, 0, one // 6, 0])
    steps = args.steps if args.steps is not None else 20
    warmup = args.warmup if args.warmup is not None else 2
    for _ in range(warmup):
        r = sched.simulate(cfg, details=False)
    t0 = time.perf_counter()
    for _ in range(steps):
        r = sched.simulate(cfg, details=False)
    ms = (time.perf_counter() - t0) * 1e3 / steps
    variants = {}
    for name, kw in (("pipeline+segments", {}), ("pipeline, whole sequences", dict(segment=1 << 20)),
                     ("trajectory-level, segments", dict(pipeline=0)), ("trajectory-level, whole sequences", dict(pipeline=0, segment=1 << 20))):
        v = sched.simulate(dict(cfg, **kw), details=False)
        variants[name] = {"mean_tokens_until_trainable": round(v["sum_wait"] / v["n_groups"], 1), "makespan_tokens": v["makespan"]}
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import sched_oracle as so
        c0 = time.perf_counter()
        reps = 0
        while time.perf_counter() - c0 < args.cpu_seconds:
            o = so.simulate(cfg)
            reps += 1
        dt = time.perf_counter() - c0
        cpu = {"value": round(len(o["items"]) * reps / dt, 1), "unit": "sequences/s", "cores": 1, "kind": "oracle",
               "sample": f"the same 512 problems, {reps} simulation(s), {dt:.1f} s (pure Python)",
               "same_result_as_native": bool(r["makespan"] == o["makespan"] and r["sum_wait"] == o["sum_wait"] and r["n_items"] == len(o["items"]))}
    print(json.dumps({
        "metric": "simulated rollout sequences/s (host-only scheduling simulator)", "value": round(r["n_items"] / (ms * 1e-3), 1),
        "unit": "sequences/s", "n_gpus": 0, "steps": steps, "warmup": warmup, "ms_per_step": round(ms, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "int64", "data": "synthetic",
        "config": {"workload": "sched", "problems": cfg["problems"], "group_size": 8, "n_select": 2, "segment": cfg["segment"],
                   "decode_slots": cfg["capacity"], "strategy": "adaptive"},
        "roofline": None, "cpu_baseline": cpu,
        "simulation": {"sequences": r["n_items"], "groups": r["n_groups"], "tokens": r["tokens"], "early_stop_by_role": r["early_stop"],
                       "schedules": variants}}))


def main():
    args = parse()
    if args.gpus != 1:
        sys.stderr.write("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
                         "--gpus must be 1. See DESIGN.md for how the path would shard.\n")
        sys.exit(2)
    if args.workload == "sched":
        return bench_sched(args)
    import torch
    from paper_2511_11373_amd import moe
    from paper_2511_11373_amd import workloads as wl

    if not torch.cuda.is_available():
        sys.stderr.write("bench.py: no GPU visible\n")
        sys.exit(3)
    moe.load_library()          # raises if the HIP library is not built: there is no fallback
    if args.workload == "logprob16k":
        return bench_logprob(args)
    if args.workload == "backward16k":
        return bench_backward(args)
    if args.workload == "attn64":
        return bench_attn(args)
    cfg = wl.CONFIGS[args.workload]
    steps = args.steps if args.steps is not None else DEFAULT_STEPS[cfg.name]
    warmup = args.warmup if args.warmup is not None else max(5, steps // 10)

    want_cpu = not args.no_cpu_baseline
    d = wl.make_inputs(cfg, want_f32=want_cpu)
    bf16 = cfg.dtype == wl.BF16
    elt = 2 if bf16 else 4

    def dev(a):
        t = torch.from_numpy(a)
        return (t.view(torch.bfloat16) if bf16 else t).cuda()

    x, wr = dev(d["x"]), dev(d["w_router"])
    bias = None if d["router_bias"] is None else torch.from_numpy(d["router_bias"]).cuda()
    sets = [(dev(d["w_gate"]), dev(d["w_up"]), dev(d["w_down"]))]
    for s in range(1, WEIGHT_SETS):     # equally distributed sets at other addresses: experts rotated by s
        sets.append(tuple(torch.roll(w, shifts=s, dims=0).contiguous() for w in sets[0]))

    def measure(cfg, x, bias, steps, warmup):
        """Times `steps` forward passes of `cfg` over the rotating weight sets; then the per-stage event times and the
        realised routing of the same step.  Returns (ms_per_step, stage means [ms], load histogram, out, step)."""
        shp = moe.make_shape(cfg.T, cfg.H, cfg.E, cfg.K, cfg.I, moe.MOE_BF16 if bf16 else moe.MOE_F32, cfg.renormalize)
        ws = moe.alloc_workspace(shp)
        out = torch.empty((cfg.T, cfg.H), dtype=x.dtype, device="cuda")
        idx = torch.empty((cfg.T, cfg.K), dtype=torch.int32, device="cuda")

        def step(i, idx_out=None):
            wg, wu, wd = sets[i % WEIGHT_SETS]
            moe.moe_forward(shp, x, wr, bias, wg, wu, wd, ws, out=out, topk_idx_out=idx_out)

        for i in range(warmup):
            step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            step(i)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        # realised routing (after the timed region): active experts and load histogram
        step(0, idx_out=idx)
        torch.cuda.synchronize()
        load = np.bincount(idx.cpu().numpy().ravel(), minlength=cfg.E)
        # per-stage HIP-event times of the same step (the library records an event at every stage boundary)
        stage = np.zeros(moe.NUM_STAGES)
        n_prof = max(10, min(steps, 100))
        for i in range(n_prof):
            wg, wu, wd = sets[i % WEIGHT_SETS]
            _, sms = moe.moe_forward_stage_times(shp, x, wr, bias, wg, wu, wd, ws, out=out)
            stage += np.array(sms)
        return ms, stage / n_prof, load, out, step

    ms_per_step, stage, load, out, step = measure(cfg, x, bias, steps, warmup)
    tokens_per_s = cfg.T / (ms_per_step * 1e-3)
    e_act = int((load > 0).sum())
    stages_ms = {n: round(float(v), 5) for n, v in zip(moe.STAGE_NAMES, stage)}

    # roofline of the dominant kernel, the gate/up GEMM (2/3 of the weight bytes and of the flops)
    # a stage interval = the kernel plus what recording two events around it costs; the library also times an
    # empty interval, which is subtracted
    empty_ms = float(stage[moe.STAGE_NAMES.index("empty_interval")])
    gu_ms = float(stage[moe.STAGE_NAMES.index("gate_up_gemm")]) - empty_ms
    gu_bytes = e_act * 2 * cfg.I * cfg.H * elt + cfg.T * cfg.H * elt + cfg.T * cfg.K * cfg.I * 2
    gu_flops = 2.0 * cfg.T * cfg.K * 2 * cfg.I * cfg.H
    layer_bytes = e_act * 3 * cfg.I * cfg.H * elt + cfg.E * cfg.H * elt + 2 * cfg.T * cfg.H * elt
    layer_flops = 2.0 * cfg.T * cfg.K * 3 * cfg.I * cfg.H
    hbm_whole = layer_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS
    mfma_whole = layer_flops / (ms_per_step * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS
    traffic = measured_traffic(cfg.name)
    # `traffic` is not read in this run: it is the figure recorded from two rocprofv3 --pmc runs of this script, kept
    # with a hash of the kernel source it was taken for, and null once that source has changed
    traffic_note = None if traffic is None else (
        "recorded rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command (profiles/hbm_traffic.md), valid for "
        f"{TRAFFIC[cfg.name]['source']} sha256 {TRAFFIC[cfg.name]['sha256_16']}; not re-read in this run")
    if cfg.name in HBM_BOUND or cfg.name == "tiny":
        ach = gu_bytes / (gu_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": "gate_up_gemm", "scope": "dominant kernel only; whole step: whole_step_frac",
                    "achieved": round(ach, 1), "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4), "whole_step_frac": round(hbm_whole, 4),
                    "traffic": traffic, "traffic_source": traffic_note,
                    "bytes_per_launch": int(gu_bytes), "avg_launch_ms": round(gu_ms, 5)}
    else:
        ach = gu_flops / (gu_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "kernel": "gate_up_gemm", "scope": "dominant kernel only; whole step: whole_step_frac",
                    "achieved": round(ach, 1), "peak": MFMA_BF16_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(ach / MFMA_BF16_PEAK_TFLOPS, 4), "whole_step_frac": round(mfma_whole, 4),
                    "traffic": traffic, "traffic_source": traffic_note,
                    "flops_per_launch": gu_flops, "avg_launch_ms": round(gu_ms, 5)}
    layer = {"active_experts": e_act, "load_max": int(load.max()), "load_median": float(np.median(load)),
             "load_empty": int((load == 0).sum()),
             "algorithmic_GB": round(layer_bytes / 1e9, 4), "algorithmic_GFLOP": round(layer_flops / 1e9, 2),
             "hbm_frac_whole_step": round(hbm_whole, 4),
             "mfma_frac_whole_step": round(mfma_whole, 4),
             "stages_ms": stages_ms}

    # The metric has a prefill half (% of the bf16 matrix-core peak at 16384 tokens).  The default run measures it too,
    # in the same process, on the same weight sets and rotation: the layer shape is the same, only the batch differs.
    if cfg.name == "decode64" and not args.no_prefill_record:
        pcfg = wl.CONFIGS["prefill16k"]
        px = dev(wl.make_inputs(pcfg, want_f32=False, only=("x",))["x"])
        p_steps, p_warm = 40, 10
        p_ms, p_stage, p_load, p_out, _ = measure(pcfg, px, None, p_steps, p_warm)
        p_flops = 2.0 * pcfg.T * pcfg.K * 3 * pcfg.I * pcfg.H
        p_empty = float(p_stage[moe.STAGE_NAMES.index("empty_interval")])
        p_gu = float(p_stage[moe.STAGE_NAMES.index("gate_up_gemm")]) - p_empty
        p_dn = float(p_stage[moe.STAGE_NAMES.index("down_gemm")]) - p_empty
        layer["prefill16k"] = {
            "workload": "prefill16k", "tokens": pcfg.T, "steps": p_steps, "warmup": p_warm, "ms_per_step": round(p_ms, 5),
            "tokens_per_s": round(pcfg.T / (p_ms * 1e-3), 1), "algorithmic_GFLOP": round(p_flops / 1e9, 2),
            "mfma_frac_whole_step": round(p_flops / (p_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
            "gate_up_gemm": {"avg_launch_ms": round(p_gu, 5),
                             "mfma_frac": round(p_flops * (2.0 / 3.0) / (p_gu * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)},
            "down_gemm": {"avg_launch_ms": round(p_dn, 5),
                          "mfma_frac": round(p_flops / 3.0 / (p_dn * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)},
            "stages_ms": {n: round(float(v), 5) for n, v in zip(moe.STAGE_NAMES, p_stage)},
            "load_max": int(p_load.max()), "load_median": float(np.median(p_load)),
            "finite": bool(torch.isfinite(p_out.float()).all().item()),
        }
        del px, p_out

    cpu = None
    if want_cpu:
        import oracle                      # the CPU oracle, timed as it stands: a baseline, not the target
        xs, wrf = d["x_f32"], d["w_router_f32"]
        wgf, wuf, wdf = d["w_gate_f32"], d["w_up_f32"], d["w_down_f32"]
        def run_oracle(n):
            return oracle.forward(xs[:n], wrf, wgf, wuf, wdf, cfg.K, bias=d["router_bias"],
                                  renormalize=cfg.renormalize)
        n0 = min(cfg.T, 4)
        c0 = time.perf_counter()
        run_oracle(n0)
        per_tok = (time.perf_counter() - c0) / n0
        n = int(max(n0, min(cfg.T, args.cpu_seconds / max(per_tok, 1e-9))))
        reps = int(max(1, min(1000, args.cpu_seconds / max(per_tok * n, 1e-9))))   # small batches: repeat
        c0 = time.perf_counter()
        for _ in range(reps):
            o_out, _, _ = run_oracle(n)
        dt = time.perf_counter() - c0
        cpu = {"value": round(n * reps / dt, 2), "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"first {n} of {cfg.T} tokens of the same batch, {reps} oracle forward(s), {dt:.1f} s"}
        # the sample doubles as a sanity check of the timed path (rows of a batch are independent)
        step(0)
        torch.cuda.synchronize()
        got = out[:n].float().cpu().numpy().astype(np.float64)
        rel = float(np.linalg.norm(got - o_out) / max(np.linalg.norm(o_out), 1e-30))
        cpu["rel_l2_gpu_vs_oracle"] = round(rel, 6)

    rec = {
        "metric": "MoE-layer tokens/s + % HBM BW (decode) / % bf16 MFMA peak (prefill)",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": cfg.name, "tokens": cfg.T, "hidden": cfg.H, "experts": cfg.E, "top_k": cfg.K,
                   "intermediate": cfg.I, "weight_sets_rotated": WEIGHT_SETS,
                   "router_bias": "zipf(1.2)" if cfg.zipf_s else None},
        "roofline": roofline, "cpu_baseline": cpu, "layer": layer,
    }
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
