"""Seeded synthetic inputs for the routed-expert MoE FFN layer.

The layer shape is that of the policy model the paper trains (Section 4.1,
"Training Details": Qwen3-30B-A3B-Thinking-2507): hidden 2048, 128 routed
experts, 8 experts per token, expert intermediate size 768, SwiGLU experts.
Token counts stand in for the paper's workloads: a rollout decode step over a
batch of concurrent responses (Section 4.1: 128 prompts x 8 responses) and a
log-prob recompute chunk of one 16k-token segment (Section 2.3, segment
rollout; Eq. 3 needs the recomputed token probabilities).

This module only draws numbers.  It holds none of the layer's arithmetic and is
the one module both the CPU oracle's tests and the GPU path's tests draw their
inputs from; each tensor has its own independent random stream.

bf16 tensors are returned as numpy uint16 bit patterns (numpy has no bf16).
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, Optional

import numpy as np

BF16 = "bf16"
F32 = "f32"


@dataclasses.dataclass(frozen=True)
class MoEConfig:
    name: str
    T: int            # tokens
    H: int            # hidden size
    E: int            # routed experts
    K: int            # experts per token
    I: int            # expert intermediate size
    dtype: str        # BF16 or F32: storage type of x and of every weight
    renormalize: bool = True
    zipf_s: Optional[float] = None   # router-bias skew exponent, None = no bias
    seed: int = 0
    sigma_w: float = 0.02            # standard deviation of every weight


CONFIGS: Dict[str, MoEConfig] = {
    "tiny":        MoEConfig("tiny", 64, 256, 8, 2, 128, F32),
    "decode64":    MoEConfig("decode64", 64, 2048, 128, 8, 768, BF16),
    "decode512":   MoEConfig("decode512", 512, 2048, 128, 8, 768, BF16),
    "prefill16k":  MoEConfig("prefill16k", 16384, 2048, 128, 8, 768, BF16),
    "skew4k":      MoEConfig("skew4k", 4096, 2048, 128, 8, 768, BF16, zipf_s=1.2),
}


def f32_to_bf16_bits_numpy(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); returns uint16 bits.  Reference bit arithmetic."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Same rounding through torch's conversion (several times faster on large tensors; the two are tested equal)."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.uint16).numpy()


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to the fp32 values they denote (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


_CHUNK_ROWS = 1 << 22      # elements per independently seeded chunk (fixed: part of the recipe)


def _fill_chunk(args):
    seed, stream, j, view, sigma = args
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, stream, j])))
    rng.standard_normal(size=view.shape, dtype=np.float32, out=view)
    if sigma != 1.0:
        view *= np.float32(sigma)


def _normal(seed: int, stream: int, shape, sigma: float) -> np.ndarray:
    """N(0, sigma^2) float32 tensor; chunk j of the flattened tensor comes from
    the PCG64 stream seeded with (seed, stream, j), so the values do not depend
    on how many threads fill it."""
    n = int(np.prod(shape))
    flat = np.empty(n, dtype=np.float32)
    jobs = [(seed, stream, j, flat[o:o + _CHUNK_ROWS], sigma)
            for j, o in enumerate(range(0, n, _CHUNK_ROWS))]
    if len(jobs) == 1:
        _fill_chunk(jobs[0])
    else:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=8) as ex:
            list(ex.map(_fill_chunk, jobs))
    return flat.reshape(shape)


def zipf_target_load(T: int, K: int, E: int, s: float) -> np.ndarray:
    """Per-rank target row counts L_r = min(T, c * r^-s) with sum T*K.

    One expert can serve at most T of the T*K assignments (a token picks K
    distinct experts), so the head of the law is capped at T.
    """
    ranks = np.arange(1, E + 1, dtype=np.float64)
    lo, hi = 0.0, float(T) * K * E
    for _ in range(200):
        c = 0.5 * (lo + hi)
        tot = np.minimum(float(T), c * ranks ** (-s)).sum()
        if tot < T * K:
            lo = c
        else:
            hi = c
    return np.minimum(float(T), 0.5 * (lo + hi) * ranks ** (-s))


def zipf_router_bias(cfg: MoEConfig) -> np.ndarray:
    """Per-expert additive router bias whose realised load is roughly Zipf(s).

    Experts are ranked by a seeded permutation.  The bias starts from a
    Gumbel-matching guess and is then calibrated for a fixed number of steps
    against seeded i.i.d. Gaussian stand-in scores with the standard deviation
    the real logits have (sigma_w * sqrt(H) for x ~ N(0,1)); the inputs
    themselves are never looked at.  The realised load of a run is whatever the
    layer's own router then produces; benchmarks report that histogram.
    """
    assert cfg.zipf_s is not None
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([cfg.seed, 6])))
    perm = rng.permutation(cfg.E)                  # perm[r] = expert holding rank r+1
    target = zipf_target_load(cfg.T, cfg.K, cfg.E, cfg.zipf_s)
    sig = cfg.sigma_w * math.sqrt(cfg.H)
    beta = sig * math.sqrt(6.0) / math.pi
    n_mc = 4096
    z = rng.standard_normal(size=(n_mc, cfg.E)) * sig
    b_rank = -cfg.zipf_s * beta * np.log(np.arange(1, cfg.E + 1, dtype=np.float64))
    tgt = target * (n_mc / cfg.T)
    for _ in range(30):
        s = z + b_rank[None, :]
        top = np.argpartition(-s, cfg.K - 1, axis=1)[:, :cfg.K]
        real = np.bincount(top.ravel(), minlength=cfg.E).astype(np.float64)
        b_rank = b_rank + 0.5 * beta * (np.log(tgt) - np.log(np.maximum(real, 1.0)))
    bias = np.empty(cfg.E, dtype=np.float32)
    bias[perm] = b_rank.astype(np.float32)
    return bias


def make_inputs(cfg: MoEConfig, weight_set: int = 0, want_f32: bool = True, only=None) -> Dict[str, np.ndarray]:
    """Draw x, the router weight, the three expert weights and the router bias.

    Returns a dict with, for every tensor name in (x, w_router, w_gate, w_up,
    w_down): `<name>` in storage form (float32 array, or uint16 bf16 bits) and
    `<name>_f32`, the same values as float32 (what a CPU reference consumes;
    left out when `want_f32` is false).
    `router_bias` is float32 [E] or None.  `weight_set` > 0 draws a different,
    equally distributed set of expert weights (for cache-defeating rotation in
    benchmarks); x and the router are unchanged.  `only` restricts the tensors
    drawn to the names listed (each tensor has its own stream, so the values are
    the same as in a full draw).
    """
    T, H, E, I = cfg.T, cfg.H, cfg.E, cfg.I
    base = 16 * weight_set
    recipe = {
        "x": (1, (T, H), 1.0),
        "w_router": (2, (E, H), cfg.sigma_w),
        "w_gate": (3 + base, (E, I, H), cfg.sigma_w),
        "w_up": (4 + base, (E, I, H), cfg.sigma_w),
        "w_down": (5 + base, (E, H, I), cfg.sigma_w),
    }
    raw = {k: _normal(cfg.seed, stream, shape, sigma) for k, (stream, shape, sigma) in recipe.items()
           if only is None or k in only}
    out: Dict[str, np.ndarray] = {}
    for k, v in raw.items():
        if cfg.dtype == BF16:
            bits = f32_to_bf16_bits(v)
            out[k] = bits
            if want_f32:
                out[k + "_f32"] = bf16_bits_to_f32(bits)
        else:
            out[k] = v
            if want_f32:
                out[k + "_f32"] = v
    out["router_bias"] = zipf_router_bias(cfg) if cfg.zipf_s is not None else None
    return out


def small_config(T: int, H: int, E: int, K: int, I: int, dtype: str = F32, seed: int = 0,
                 renormalize: bool = True, sigma_w: float = 0.02) -> MoEConfig:
    return MoEConfig(f"T{T}H{H}E{E}K{K}I{I}", T, H, E, K, I, dtype, renormalize, None, seed, sigma_w)


def make_cancelling_router_inputs(T: int, H: int, E: int, seed: int, amp: float = 4.0, sigma_w: float = 0.02):
    """Token rows and router rows (bf16 bits) built so that unrelated router rows of LARGE norm get equal or nearly
    equal exact logits for every token, through heavy cancellation.

    Column j + H/4 of x repeats column j for j < H/4.  On those columns every router row carries +a at j and -a at
    j + H/4 with its own independent a ~ N(0, amp^2): the pairs contribute exactly zero to every exact logit, whatever
    the token, but the partners lie a quarter of the row apart, so an implementation that accumulates in a narrower type
    carries a partial sum of size amp * sqrt(H) through hundreds of additions and keeps rounding noise proportional to
    it, different for every row.  On the second half of the columns, rows e and e + E/2 ("twins") are the same
    N(0, sigma_w^2) draw, so twins tie exactly; every third twin then has the last mantissa bit of three entries
    flipped, which turns its ties into gaps far below that noise, of either sign depending on the token.  Only numbers
    are drawn here."""
    assert H % 4 == 0 and E % 2 == 0
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 77])))
    x = rng.standard_normal((T, H)).astype(np.float32)
    q, half = H // 4, H // 2
    x[:, q:half] = x[:, :q]
    xb = f32_to_bf16_bits(x)
    w = np.zeros((E, H), dtype=np.float32)
    base = (rng.standard_normal((E // 2, H - half)) * sigma_w).astype(np.float32)
    w[:E // 2, half:] = base
    w[E // 2:, half:] = base
    wb = f32_to_bf16_bits(w)
    a = f32_to_bf16_bits((rng.standard_normal((E, q)) * amp).astype(np.float32))
    wb[:, :q] = a
    wb[:, q:half] = a ^ np.uint16(0x8000)            # the same magnitude with the opposite sign
    for e in range(E // 2, E, 3):
        cols = half + rng.integers(0, H - half, 3)
        wb[e, cols] = wb[e, cols] ^ np.uint16(1)
    return xb, wb


# ---- token log-probability / GRPO objective step --------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class GrpoConfig:
    name: str
    N: int                 # response tokens of the group, concatenated
    V: int                 # vocabulary size
    G: int                 # responses in the group
    dtype: str             # storage type of the logits
    clip_eps: float = 0.2
    beta: float = 0.04
    adv_eps: float = 1e-6
    seed: int = 0
    logit_scale: float = 2.5


GRPO_CONFIGS: Dict[str, GrpoConfig] = {
    # one 16k-token segment of log-prob recompute over the group of 8 responses of a prompt (Section 4.1),
    # Qwen3 vocabulary
    "logprob16k": GrpoConfig("logprob16k", 16384, 151936, 8, BF16),
    "logprob_small": GrpoConfig("logprob_small", 300, 4096, 5, F32),
}


def make_grpo_inputs(cfg: GrpoConfig, rows: Optional[slice] = None) -> Dict[str, np.ndarray]:
    """Logits ~ N(0, logit_scale^2) with the target's logit raised so that targets are likely-ish tokens, old and
    reference log-probs near plausible values, 0/1 rewards, response lengths of a long-tailed mix.  `rows`
    restricts the (large) logits tensor to a row range; everything else is always complete."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([cfg.seed, 101])))
    target = rng.integers(0, cfg.V, cfg.N).astype(np.int32)
    # response lengths: a long-tailed split of N into G parts (some may be short, none negative)
    wts = rng.pareto(1.5, cfg.G) + 0.05 if cfg.G > 0 else np.zeros(0)
    lens = np.floor(wts / max(wts.sum(), 1e-30) * cfg.N).astype(np.int64) if cfg.G > 0 else np.zeros(0, np.int64)
    if cfg.G > 0:
        lens[-1] += cfg.N - lens.sum()
    offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    rewards = (rng.random(cfg.G) < 0.5).astype(np.float32)
    logp_old = (-rng.gamma(2.0, 0.8, cfg.N)).astype(np.float32)
    logp_ref = (logp_old + rng.standard_normal(cfg.N).astype(np.float32) * 0.2).astype(np.float32)
    r0, r1 = (0, cfg.N) if rows is None else (rows.start or 0, cfg.N if rows.stop is None else rows.stop)
    out = {"target": target, "resp_offsets": offsets, "rewards": rewards, "logp_old": logp_old, "logp_ref": logp_ref}
    n = r1 - r0
    chunks = []
    for c0 in range(r0, r1, 512):                       # row blocks of 512, each its own stream: any row range
        c1 = min(c0 + 512, r1)                          # of a 512-aligned start reproduces the same values
        blk = c0 // 512
        b0 = blk * 512
        a = _normal(cfg.seed, 1000 + blk, (min(512, cfg.N - b0), cfg.V), cfg.logit_scale)
        a[np.arange(a.shape[0]), target[b0:b0 + a.shape[0]]] += np.float32(2.0 * cfg.logit_scale)
        chunks.append(a[c0 - b0:c1 - b0])
    logits = np.concatenate(chunks, axis=0) if chunks else np.zeros((0, cfg.V), np.float32)
    assert logits.shape[0] == n
    if cfg.dtype == BF16:
        bits = f32_to_bf16_bits(logits)
        out["logits"] = bits
        out["logits_f32"] = bf16_bits_to_f32(bits)
    else:
        out["logits"] = logits
        out["logits_f32"] = logits
    return out


# ---- decode attention over a long paged context ----------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class AttnConfig:
    name: str
    B: int                 # sequences decoding one token each
    Hq: int
    Hkv: int
    prompt: int            # every context holds the prompt ...
    max_new: int           # ... plus a uniformly drawn part of the output budget
    seed: int = 4611
    D: int = 128
    page: int = 256


ATTN_CONFIGS: Dict[str, AttnConfig] = {
    # Section 4.1: inputs of 32k tokens, outputs of up to 64k; Qwen3-30B-A3B head geometry
    "attn64": AttnConfig("attn64", 64, 32, 4, 32768, 65536),
    "attn_small": AttnConfig("attn_small", 5, 32, 4, 300, 3000, seed=9),
}


def attn_lengths_and_table(cfg: AttnConfig):
    """Context lengths, a random page assignment and the pool size (16 spare pages): lens [B], table [B, max_pages], n_pages."""
    rng = np.random.default_rng(cfg.seed)
    lens = (cfg.prompt + rng.integers(0, cfg.max_new + 1, cfg.B)).astype(np.int32)
    pages_of = (lens + cfg.page - 1) // cfg.page
    max_pages, need = int(pages_of.max()), int(pages_of.sum())
    n_pages = need + 16
    ids = rng.permutation(n_pages)[:need].astype(np.int32)
    table = np.zeros((cfg.B, max_pages), dtype=np.int32)
    at = 0
    for b in range(cfg.B):
        table[b, :pages_of[b]] = ids[at:at + pages_of[b]]
        at += pages_of[b]
    return lens, table, n_pages


def attn_device_inputs(cfg: AttnConfig, n_pages: int):
    """q [B, Hq, D], k_pages [n_pages, Hkv, page, D], v_pages [n_pages, Hkv, D, page] (pages in storage order: what was
    drawn is whatever attn_untile_keys / attn_untile_values make of them): standard normal bf16 drawn on the device with
    torch's seeded generator (the full-size cache is several GB), 1024 pages at a time."""
    import torch
    gen = torch.Generator(device="cuda")
    gen.manual_seed(cfg.seed)
    q = torch.randn((cfg.B, cfg.Hq, cfg.D), device="cuda", generator=gen).bfloat16()
    k_pages = torch.empty((n_pages, cfg.Hkv, cfg.page, cfg.D), dtype=torch.bfloat16, device="cuda")
    v_pages = torch.empty((n_pages, cfg.Hkv, cfg.D, cfg.page), dtype=torch.bfloat16, device="cuda")
    for p0 in range(0, n_pages, 1024):
        p1 = min(n_pages, p0 + 1024)
        k_pages[p0:p1] = torch.randn((p1 - p0, cfg.Hkv, cfg.page, cfg.D), device="cuda", generator=gen).bfloat16()
        v_pages[p0:p1] = torch.randn((p1 - p0, cfg.Hkv, cfg.D, cfg.page), device="cuda", generator=gen).bfloat16()
    return q, k_pages, v_pages


# Storage order inside a cache page of one head (256 positions x 128 features), as include/attn_decode.h defines it: blocks
# of 64 positions; a block of keys is 16 tiles (t, i) of 16 rows x 32 features, row r of tile t being position
# 32 (t / 2) + 8 (r / 4) + 4 (t % 2) + r % 4 of the block; a block of values is 16 tiles (c8, u) of 16 features x 32
# positions.  These helpers only move elements (any array type with reshape / transpose: numpy or torch).
def _transpose(a, axes):
    return a.transpose(*axes) if isinstance(a, np.ndarray) else a.permute(*axes)


def attn_tile_keys(k):
    """[..., 256, 128] position-major -> the page's storage order, same shape."""
    lead = tuple(k.shape[:-2])
    n = len(lead)
    x = k.reshape(lead + (4, 2, 4, 2, 4, 4, 32))          # block, p/32, (p%32)/8, (p%8)/4, p%4, f/32, f%32
    x = _transpose(x, tuple(range(n)) + tuple(n + i for i in (0, 1, 3, 5, 2, 4, 6)))     # block, t = (p/32, (p%8)/4), i, r = ((p%32)/8, p%4), f%32
    return x.reshape(lead + (256, 128))


def attn_untile_keys(k):
    """Inverse of attn_tile_keys."""
    lead = tuple(k.shape[:-2])
    n = len(lead)
    x = k.reshape(lead + (4, 2, 2, 4, 4, 4, 32))
    x = _transpose(x, tuple(range(n)) + tuple(n + i for i in (0, 1, 4, 2, 5, 3, 6)))
    return x.reshape(lead + (256, 128))


def attn_tile_values(v):
    """[..., 128, 256] feature-major -> the page's storage order, same shape."""
    lead = tuple(v.shape[:-2])
    n = len(lead)
    x = v.reshape(lead + (8, 16, 4, 2, 32))               # f/16, f%16, block, (p%64)/32, p%32
    x = _transpose(x, tuple(range(n)) + tuple(n + i for i in (2, 0, 3, 1, 4)))
    return x.reshape(lead + (128, 256))


def attn_untile_values(v):
    """Inverse of attn_tile_values."""
    lead = tuple(v.shape[:-2])
    n = len(lead)
    x = v.reshape(lead + (4, 8, 2, 16, 32))
    x = _transpose(x, tuple(range(n)) + tuple(n + i for i in (1, 3, 0, 2, 4)))
    return x.reshape(lead + (128, 256))


def attn_sequence_to_host(cfg: AttnConfig, k_pages, v_pages, table, lens, b: int):
    """The logical cache of sequence b as float arrays k, v [n, Hkv, D] (copied back from the device pools)."""
    import torch
    n = int(lens[b])
    pg = torch.from_numpy(table[b, :(n + cfg.page - 1) // cfg.page].astype(np.int64)).to(k_pages.device)
    k = attn_untile_keys(k_pages[pg]).permute(0, 2, 1, 3).reshape(-1, cfg.Hkv, cfg.D)[:n].float().cpu().numpy()
    v = attn_untile_values(v_pages[pg]).permute(0, 3, 1, 2).reshape(-1, cfg.Hkv, cfg.D)[:n].float().cpu().numpy()
    return k, v
