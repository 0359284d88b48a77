"""The pins must be able to fail: each plausible mistake planted in a copy of the oracle's C source (a dropped
term, a wrong sign, a swapped operand, an off-by-one, an unstable sort ...) has to be caught by at least one of a
compact set of pins.  CPU only; the mistakes are planted in the oracle, never in the GPU path."""
import ctypes
import math
import os
import subprocess

import numpy as np
import pytest
import scipy.special
import torch

import oracle
from oracle import bruteforce
from paper_2511_11373_amd import workloads as wl

SRC = os.path.join(os.path.dirname(oracle.__file__), "moe_oracle.c")

MUTATIONS = [
    ("logit bias dropped", "if (bias) s += (double)bias[e];", "if (0) s += (double)bias[e];"),
    ("router operand transposed", "(double)w_router[(size_t)e * H + h]", "(double)w_router[(size_t)(e * H + h) % ((size_t)E * H - 1)]"),
    ("ties go to the higher id", "if (best < 0 || l[e] > l[best]) best = e;", "if (best < 0 || l[e] >= l[best]) best = e;"),
    ("selects the smallest", "if (best < 0 || l[e] > l[best]) best = e;", "if (best < 0 || l[e] < l[best]) best = e;"),
    ("softmax sign", "(float)(exp((double)l[idx[(size_t)t * K + k]] - m) / denom)", "(float)(exp(m - (double)l[idx[(size_t)t * K + k]]) / denom)"),
    ("renormalise over all experts", "if (renormalize) {", "if (0) {"),
    ("offsets off by one", "off[idx[a] + 1] += 1;", "off[idx[a]] += 1;"),
    ("unstable placement", "int32_t r = next[idx[a]]++;", "int32_t r = off[idx[a] + 1] - 1 - (next[idx[a]]++ - off[idx[a]]);"),
    ("inverse map wrong", "assign_to_row[a] = r;", "assign_to_row[a] = a;"),
    ("gather ignores K", "(size_t)(row_to_assign[r] / K) * H", "(size_t)(row_to_assign[r] % (n / K)) * H"),
    ("silu without gate factor", "a[i] = g / (1.0 + exp(-g)) * u;", "a[i] = 1.0 / (1.0 + exp(-g)) * u;"),
    ("silu sign", "a[i] = g / (1.0 + exp(-g)) * u;", "a[i] = g / (1.0 + exp(g)) * u;"),
    ("gate and up swapped", "g += (double)v[h] * (double)wg[(size_t)i * H + h];\n            u += (double)v[h] * (double)wu[(size_t)i * H + h];",
     "u += (double)v[h] * (double)wg[(size_t)i * H + h];\n            g += (double)v[h] * (double)wu[(size_t)i * H + h];"),
    ("down projection transposed", "s += a[i] * (double)wd[(size_t)j * I + i];", "s += a[i] * (double)wd[((size_t)i * H + j) % ((size_t)H * I)];"),
    ("wrong expert's weights", "int e = row_expert[r];", "int e = row_expert[n - 1 - r];"),
    ("combine drops the weight", "s += (double)w[(size_t)t * K + k] * y_perm[", "s += y_perm["),
    ("combine skips a slot", "for (int k = 0; k < K; ++k)\n                s += (double)w[(size_t)t * K + k]", "for (int k = 0; k < K - (K > 1); ++k)\n                s += (double)w[(size_t)t * K + k]"),
]


class Lib:
    """The oracle's Python front end bound to another shared object."""

    def __init__(self, path):
        self.lib = ctypes.CDLL(path)

    def __getattr__(self, name):
        fn = getattr(oracle, name)

        def call(*a, **k):
            saved = oracle._lib
            oracle._lib = self.lib
            try:
                return fn(*a, **k)
            finally:
                oracle._lib = saved
        return call


def compact_pins(o):
    """A fast subset of the pins in test_oracle_pins.py; raises AssertionError on the first violation."""
    cfg = wl.small_config(9, 24, 6, 3, 16, seed=31, sigma_w=0.4)
    d = wl.make_inputs(cfg)
    x, wr, wg, wu, wd = (d[k + "_f32"] for k in ("x", "w_router", "w_gate", "w_up", "w_down"))
    bias = np.linspace(0.4, -0.4, cfg.E).astype(np.float32)
    out, idx, w = o.forward(x, wr, wg, wu, wd, cfg.K, bias=bias)
    ref, sel, G = bruteforce.dense_forward(x, wr, wg, wu, wd, cfg.K, bias=bias)
    assert np.array_equal(idx, sel)
    np.testing.assert_allclose(np.take_along_axis(G, idx.astype(np.int64), axis=1), w, rtol=2e-6)
    np.testing.assert_allclose(out, ref, rtol=1e-5, atol=1e-6 * np.abs(ref).max())     # w is stored as float
    # ties and un-normalised weights
    logits = np.array([[0.5, 0.5, -1.0, 0.5, 0.25]], dtype=np.float32)
    i2, w2 = o.topk_from_logits(logits, 2, False)
    assert i2.tolist() == [[0, 1]]
    full = scipy.special.softmax(logits.astype(np.float64), axis=1)
    np.testing.assert_allclose(w2, full[:, :2], rtol=1e-6)
    # permutation against the library stable sort
    rng = np.random.default_rng(5)
    tk = np.stack([rng.permutation(7)[:3] for _ in range(11)]).astype(np.int32)
    off, r2a, a2r = o.permute(tk, 7)
    assert np.array_equal(r2a, np.argsort(tk.reshape(-1), kind="stable"))
    assert np.array_equal(off, np.concatenate([[0], np.cumsum(np.bincount(tk.reshape(-1), minlength=7))]))
    assert np.array_equal(r2a[a2r], np.arange(33))
    xx = rng.standard_normal((11, 4)).astype(np.float32)
    assert np.array_equal(o.gather_rows(xx, r2a, 3)[a2r], np.repeat(xx, 3, axis=0))
    # a single expert is a dense SwiGLU MLP
    xt = torch.from_numpy(x).double()
    o1, _, _ = o.forward(x, wr[:1], wg[:1], wu[:1], wd[:1], 1)
    dense = (torch.nn.functional.silu(xt @ torch.from_numpy(wg[0]).double().T) * (xt @ torch.from_numpy(wu[0]).double().T)) \
        @ torch.from_numpy(wd[0]).double().T
    np.testing.assert_allclose(o1, dense.numpy(), rtol=1e-10, atol=1e-13)
    # combine against einsum
    y = rng.standard_normal((12, 5))
    p = rng.permutation(12).astype(np.int32)
    ww = rng.random((4, 3)).astype(np.float32)
    np.testing.assert_allclose(o.combine(y, p, ww), np.einsum("tk,tkh->th", ww.astype(np.float64), y[p].reshape(4, 3, 5)),
                               rtol=1e-13)


def test_the_unmodified_oracle_passes_the_compact_pins(oracle_lib):
    compact_pins(oracle_lib)


def _run_pins_in_child(so_path):
    """Runs compact_pins against a shared object in a child process (a mutant may also crash outright)."""
    import sys
    code = ("import sys; sys.path.insert(0, %r); sys.path.insert(0, %r)\n"
            "from tests.test_oracle_mutations import Lib, compact_pins\n"
            "compact_pins(Lib(%r))\n") % (os.path.dirname(os.path.dirname(os.path.abspath(__file__))),
                                           os.path.dirname(os.path.abspath(__file__)), so_path)
    return subprocess.run([sys.executable, "-c", code], stdout=subprocess.PIPE, stderr=subprocess.PIPE, timeout=120)


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(tmp_path, name, old, new):
    src = open(SRC).read()
    assert src.count(old) >= 1, f"mutation target not found: {name}"
    mutated = tmp_path / "mutant.c"
    mutated.write_text(src.replace(old, new, 1))
    so = tmp_path / "libmutant.so"
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-w", "-o", str(so), str(mutated), "-lm"])
    res = _run_pins_in_child(str(so))
    assert res.returncode != 0, f"the pins accepted an oracle with: {name}"


def test_child_runner_accepts_the_real_oracle():
    res = _run_pins_in_child(oracle.build())
    assert res.returncode == 0, res.stderr.decode()[-2000:]
