"""Pins of the decode-attention oracle to things other than itself (CPU only): the library's scaled-dot-product attention,
closed forms (zero queries average the values, a context of one returns its value, a dominant key returns its value),
and invariances of the definition (order of the context, common shift of the scores, grouped-query head mapping)."""
import numpy as np
import pytest
import torch

from oracle import attn_oracle as ao


def _rand(seed, B=3, Hq=8, Hkv=2, D=16, L=40):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((B, Hq, D))
    k = rng.standard_normal((B, L, Hkv, D))
    v = rng.standard_normal((B, L, Hkv, D))
    lens = rng.integers(1, L + 1, B)
    return q, k, v, lens


def test_matches_library_attention():
    q, k, v, lens = _rand(0)
    got = ao.decode_attention(q, k, v, lens)
    B, Hq, D = q.shape
    group = Hq // k.shape[2]
    for b in range(B):
        n = int(lens[b])
        tq = torch.tensor(q[b])[:, None, :]                                   # [Hq, 1, D]
        tk = torch.tensor(k[b, :n]).permute(1, 0, 2).repeat_interleave(group, dim=0)   # [Hq, n, D]
        tv = torch.tensor(v[b, :n]).permute(1, 0, 2).repeat_interleave(group, dim=0)
        ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[:, 0, :].numpy()
        assert np.allclose(got[b], ref, rtol=1e-12, atol=1e-12)


def test_closed_forms():
    q, k, v, lens = _rand(1)
    out = ao.decode_attention(np.zeros_like(q), k, v, lens)                   # equal scores: the mean of the values
    for b in range(q.shape[0]):
        n = int(lens[b])
        for j in range(q.shape[1]):
            assert np.allclose(out[b, j], v[b, :n, j // 4].mean(axis=0), atol=1e-13)
    one = ao.decode_attention(q, k, v, np.ones(3, dtype=int))                 # one position: its value, whatever the query
    assert np.allclose(one, np.repeat(v[:, 0], 4, axis=1), atol=1e-13)
    assert np.all(ao.decode_attention(q, k, v, np.zeros(3, dtype=int)) == 0.0)
    kk = k.copy()
    kk[0, 5, 0] = 1000.0 * q[0, 1] / np.dot(q[0, 1], q[0, 1])                 # score 1000/sqrt(D) for head 1 at position 5
    dom = ao.decode_attention(q, kk, v, np.full(3, 40))
    assert np.allclose(dom[0, 1], v[0, 5, 0], atol=1e-9)


def test_invariances_and_head_mapping():
    q, k, v, lens = _rand(2)
    lens[:] = 40
    base = ao.decode_attention(q, k, v, lens)
    perm = np.random.default_rng(3).permutation(40)
    assert np.allclose(ao.decode_attention(q, k[:, perm], v[:, perm], lens), base, atol=1e-12)     # a set, not a sequence
    # adding a multiple of q to every key shifts all scores of a head equally
    shifted = k + 0.0
    shifted[:, :, 0, :] += 3.0 * q[:, None, 0, :]
    assert np.allclose(ao.decode_attention(q, shifted, v, lens)[:, 0], base[:, 0], atol=1e-10)
    # query heads 0..3 read key/value head 0, heads 4..7 head 1: changing head 1 leaves heads 0..3 alone
    v2 = v.copy()
    v2[:, :, 1] += 1.0
    out2 = ao.decode_attention(q, k, v2, lens)
    assert np.array_equal(out2[:, :4], base[:, :4]) and np.allclose(out2[:, 4:], base[:, 4:] + 1.0, atol=1e-12)
    # positions past the length are ignored
    k3, v3 = k.copy(), v.copy()
    k3[:, 30:] = 99.0
    v3[:, 30:] = -99.0
    l30 = np.full(3, 30)
    assert np.array_equal(ao.decode_attention(q, k3, v3, l30), ao.decode_attention(q, k, v, l30))
