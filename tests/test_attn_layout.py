"""The key/value page layout of include/attn_decode.h: the array reshapes in workloads.py (which the GPU tests and the
bench use to fill and to read back cache pages) against the element formulas the header states.  CPU only."""
import numpy as np
import torch

from paper_2511_11373_amd import workloads as wl


def _key_offset(p, f):
    """Element of position p (0..255), feature f in a page of one head, as the header defines it."""
    block, pb = divmod(p, 64)
    t = 2 * (pb // 32) + (pb % 8) // 4
    r = 4 * ((pb % 32) // 8) + pb % 4
    return block * 8192 + ((4 * t + f // 32) * 16 + r) * 32 + f % 32


def _value_offset(p, f):
    block, pb = divmod(p, 64)
    return block * 8192 + ((2 * (f // 16) + pb // 32) * 16 + f % 16) * 32 + pb % 32


def test_key_tiling_matches_the_header_formula():
    k = np.arange(256 * 128, dtype=np.int64).reshape(256, 128)
    tiled = wl.attn_tile_keys(k).reshape(-1)
    want = np.empty_like(tiled)
    for p in range(256):
        for f in range(128):
            want[_key_offset(p, f)] = k[p, f]
    assert np.array_equal(tiled, want)
    assert np.array_equal(wl.attn_untile_keys(wl.attn_tile_keys(k)), k)


def test_value_tiling_matches_the_header_formula():
    v = np.arange(128 * 256, dtype=np.int64).reshape(128, 256)          # [feature, position]
    tiled = wl.attn_tile_values(v).reshape(-1)
    want = np.empty_like(tiled)
    for p in range(256):
        for f in range(128):
            want[_value_offset(p, f)] = v[f, p]
    assert np.array_equal(tiled, want)
    assert np.array_equal(wl.attn_untile_values(wl.attn_tile_values(v)), v)


def test_the_maps_are_permutations_of_a_page():
    assert sorted(_key_offset(p, f) for p in range(256) for f in range(128)) == list(range(32768))
    assert sorted(_value_offset(p, f) for p in range(256) for f in range(128)) == list(range(32768))


def test_a_load_instruction_reads_one_contiguous_kilobyte():
    """Lane (c, q) of a wave reads 8 elements at row c, elements 8 q .. + 7 of a tile: for keys the tile (t, i) must hold the
    16 positions of score tile t with features 32 i .. + 31, for values the tile (c8, u) features 16 c8 .. + 15 with
    positions 32 u .. + 31 of the block, each as 512 consecutive elements."""
    for t in range(4):
        for i in range(4):
            offs = sorted(_key_offset(32 * (t // 2) + 8 * (r // 4) + 4 * (t % 2) + r % 4, 32 * i + e) for r in range(16) for e in range(32))
            assert offs == list(range((4 * t + i) * 512, (4 * t + i) * 512 + 512))
    for c8 in range(8):
        for u in range(2):
            offs = sorted(_value_offset(32 * u + e, 16 * c8 + c) for c in range(16) for e in range(32))
            assert offs == list(range((2 * c8 + u) * 512, (2 * c8 + u) * 512 + 512))


def test_leading_axes_and_torch_tensors():
    k = torch.arange(2 * 3 * 256 * 128).reshape(2, 3, 256, 128)
    assert torch.equal(wl.attn_untile_keys(wl.attn_tile_keys(k)), k)
    assert np.array_equal(wl.attn_tile_keys(k).numpy(), wl.attn_tile_keys(k.numpy()))
    v = torch.arange(2 * 3 * 128 * 256).reshape(2, 3, 128, 256)
    assert torch.equal(wl.attn_untile_values(wl.attn_tile_values(v)), v)
    assert np.array_equal(wl.attn_tile_values(v).numpy(), wl.attn_tile_values(v.numpy()))
