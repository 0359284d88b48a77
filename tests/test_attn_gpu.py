"""GPU parity of decode attention against the numpy oracle, through the C ABI.

Tolerance: q, K, V are bf16 exactly on both sides; the library rounds the softmax numerators to bf16 before the second
product (relative 2^-9 each, averaged over the context by the weighted sum) and the result to bf16 (2^-9 relative):
max-abs <= 2e-2 * max|out|, relative L2 <= 1e-2 (measured ~3e-3).
"""
import numpy as np
import pytest
import torch

from oracle import attn_oracle as ao
from paper_2511_11373_amd import attn
from paper_2511_11373_amd import workloads as wl
from gpu_util import check_close, host

pytestmark = pytest.mark.gpu
PAGE, D = 256, 128


def paged(rng, lens, Hkv, k, v, extra_pages=3, poison=False):
    """Scatter logical caches k, v [B, L, Hkv, D] (bf16 bits) into page pools through a random block table."""
    B = len(lens)
    max_pages = max(1, max((int(n) + PAGE - 1) // PAGE for n in lens))
    need = sum((int(n) + PAGE - 1) // PAGE for n in lens)
    n_pages = need + extra_pages
    ids = rng.permutation(n_pages)[:need]
    table = np.full((B, max_pages), -12345 if poison else 0, dtype=np.int32)      # unused entries must never be followed
    fill = 0x7FC0 if poison else 0                                              # bf16 NaN in every unused position
    kp = np.full((n_pages, Hkv, PAGE, D), fill, dtype=np.uint16)
    vp = np.full((n_pages, Hkv, D, PAGE), fill, dtype=np.uint16)
    at = 0
    for b, n in enumerate(lens):
        for i in range((int(n) + PAGE - 1) // PAGE):
            pid = ids[at]; at += 1
            table[b, i] = pid
            m = min(PAGE, int(n) - i * PAGE)
            kp[pid, :, :m, :] = k[b, i * PAGE:i * PAGE + m].transpose(1, 0, 2)
            vp[pid, :, :, :m] = v[b, i * PAGE:i * PAGE + m].transpose(1, 2, 0)
    return wl.attn_tile_keys(kp), wl.attn_tile_values(vp), table, max_pages, n_pages        # the pages' storage order


def run_case(seed, lens, Hq, Hkv, poison=False, scale_q=1.0):
    rng = np.random.default_rng(seed)
    B, L = len(lens), max(1, int(max(lens)))
    qb = wl.f32_to_bf16_bits_numpy((rng.standard_normal((B, Hq, D)) * scale_q).astype(np.float32))
    kb = wl.f32_to_bf16_bits_numpy(rng.standard_normal((B, L, Hkv, D)).astype(np.float32))
    vb = wl.f32_to_bf16_bits_numpy(rng.standard_normal((B, L, Hkv, D)).astype(np.float32))
    kp, vp, table, max_pages, n_pages = paged(rng, lens, Hkv, kb, vb, poison=poison)
    shp = attn.make_shape(B, Hq, Hkv, max_pages, n_pages)
    ws = attn.alloc_workspace(shp)
    dev = lambda a: torch.from_numpy(a).view(torch.bfloat16).cuda()
    out = attn.attn_decode(shp, dev(qb), dev(kp), dev(vp), torch.from_numpy(table).cuda(),
                           torch.from_numpy(np.asarray(lens, dtype=np.int32)).cuda(), ws)
    ref = ao.decode_attention(wl.bf16_bits_to_f32(qb), wl.bf16_bits_to_f32(kb), wl.bf16_bits_to_f32(vb), lens)
    got = host(out)
    check_close(got, ref, f"attention seed {seed}", max_abs=2e-2 * max(np.abs(ref).max(), 1e-30), rel_l2=1e-2)
    return got, ref


@pytest.mark.parametrize("lens,Hq,Hkv", [
    ([1, 2, 63, 64, 65], 32, 4),                       # first step only, step boundary
    ([255, 256, 257, 1000], 32, 4),                    # page boundary
    ([2047, 2048, 2049, 5000], 32, 4),                 # 2048-position boundary (eight pages)
    ([0, 300, 0, 7], 32, 4),                           # sequences without context give zeros
    ([777, 4100], 8, 8),                               # one query head per key/value head
    ([900, 3333, 12], 16, 1),                          # a full group of 16
    ([1500], 12, 4),                                   # group of 3
], ids=["steps", "pages", "eight_pages", "empty", "mha", "group16", "group3"])
def test_decode_attention_against_oracle(lens, Hq, Hkv):
    got, ref = run_case(len(lens) * 100 + Hq, lens, Hq, Hkv)
    for b, n in enumerate(lens):
        if n == 0:
            assert np.all(got[b] == 0.0)


def _many_short(seed, B, longest):
    rng = np.random.default_rng(seed)
    lens = rng.integers(1, longest + 1, B)
    lens[rng.random(B) < 0.15] = 0
    return [int(n) for n in lens]


@pytest.mark.parametrize("lens,Hq,Hkv", [
    (_many_short(5, 1000, 192), 4, 4),                 # a wave's share of the steps runs over several sequences, empty ones among them
    (_many_short(6, 2500, 100), 2, 2),                 # more sequences than the step-counting kernel takes in one pass
    ([150000], 8, 1),                                  # one sequence shared by every wave: over a thousand partial results to merge
    ([40000, 3, 0, 129, 40000, 64, 0], 8, 2),          # shares that end inside, at the end of and just after a short sequence
], ids=["many_short", "many_sequences", "one_long", "mixed"])
def test_shares_of_the_step_list(lens, Hq, Hkv):
    """The split of the work into per-wave shares: the lengths decide where shares begin and end, so these cases put
    share boundaries in every kind of place."""
    got, ref = run_case(len(lens) + Hq, lens, Hq, Hkv, poison=True)
    for b, n in enumerate(lens):
        if n == 0:
            assert np.all(got[b] == 0.0)


@pytest.mark.parametrize("name", ["attn_small", "attn64"])
def test_bench_workload_on_sampled_sequences(name):
    """The bench workload in the configuration bench.py times (64 sequences of 34k-96k positions, 8 GB of cache drawn on the
    device): the shortest, the longest and one other sequence, every head, against the oracle on the copied-back cache."""
    cfg = wl.ATTN_CONFIGS[name]
    lens, table, n_pages = wl.attn_lengths_and_table(cfg)
    q, k_pages, v_pages = wl.attn_device_inputs(cfg, n_pages)
    shp = attn.make_shape(cfg.B, cfg.Hq, cfg.Hkv, table.shape[1], n_pages)
    ws = attn.alloc_workspace(shp)
    out = attn.attn_decode(shp, q, k_pages, v_pages, torch.from_numpy(table).cuda(), torch.from_numpy(lens).cuda(), ws)
    got = host(out)
    for b in sorted({int(np.argmin(lens)), int(np.argmax(lens)), cfg.B // 2}):
        k, v = wl.attn_sequence_to_host(cfg, k_pages, v_pages, table, lens, b)
        ref = ao.decode_attention(q[b].float().cpu().numpy()[None], k[None], v[None], [int(lens[b])])[0]
        check_close(got[b], ref, f"sequence {b}", max_abs=2e-2 * np.abs(ref).max(), rel_l2=1e-2)


def test_unused_positions_and_table_entries_are_never_followed():
    # NaN in every cache position past the sequence ends and invalid page ids in the unused table entries
    got, _ = run_case(5, [1, 70, 300, 2100], 32, 4, poison=True)
    assert np.all(np.isfinite(got))


def test_peaked_softmax_and_repeatability():
    got, ref = run_case(6, [4000, 100], 32, 4, scale_q=6.0)      # scores with a standard deviation of 6: a few positions dominate
    got2, _ = run_case(6, [4000, 100], 32, 4, scale_q=6.0)
    assert np.array_equal(got, got2)


def test_bad_arguments():
    for shp, code in ((attn.AttnShape(2, 32, 4, 64, 4, 8), 2), (attn.AttnShape(2, 30, 4, 128, 4, 8), 2),
                      (attn.AttnShape(2, 34, 2, 128, 4, 8), 2), (attn.AttnShape(2, 32, 4, 128, 0, 8), 2)):
        with pytest.raises(attn.AttnError) as e:
            attn.workspace_bytes(shp)
        assert e.value.code == code
    shp = attn.make_shape(0, 32, 4, 4, 8)
    z = torch.zeros(64, dtype=torch.bfloat16, device="cuda")
    zi = torch.zeros(16, dtype=torch.int32, device="cuda")
    attn.attn_decode(shp, z, z, z, zi, zi, attn.alloc_workspace(shp), out=z)          # an empty batch is fine
    shp = attn.make_shape(1, 32, 4, 4, 8)
    with pytest.raises(attn.AttnError) as e:
        attn.attn_decode(shp, z, z, z, zi, zi, torch.empty(256, dtype=torch.uint8, device="cuda"), out=z)
    assert e.value.code == 4
