"""The C ABI without a GPU: the library loads, exports what include/moe_ffn.h declares, and rejects bad
arguments on the host before any HIP call (so none of this needs a device)."""
import ctypes
import os
import re

import pytest

from paper_2511_11373_amd import build as hip_build
from paper_2511_11373_amd import attn, grpo, moe, moe_backward

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(moe.LIB_PATH):
        hip_build.build()
    return moe.load_library()


def test_every_declared_symbol_is_exported(lib):
    hdr = open(os.path.join(ROOT, "include", "moe_ffn.h")).read()
    declared = set(re.findall(r"\b(moe_[a-z_]+)\s*\(", hdr))
    assert declared == set(moe.EXPORTS)
    hdr_b = open(os.path.join(ROOT, "include", "moe_ffn_backward.h")).read()
    declared_b = set(re.findall(r"\b(moe_[a-z_]+)\s*\(", hdr_b))
    assert declared_b == set(moe_backward.EXPORTS)
    declared |= declared_b
    for name in declared:
        assert getattr(lib, name) is not None
    assert lib.moe_status_string(0) == b"ok" and lib.moe_status_string(2) == b"unsupported shape"
    assert lib.moe_status_string(99) == b"unknown status"


def _call_forward(lib, shape, ptrs, ws=0x1000, ws_bytes=1 << 40):
    vp = ctypes.c_void_p
    x, wr, bias, wg, wu, wd, out, idx, w = [vp(p) if p else None for p in ptrs]
    return lib.moe_forward(ctypes.byref(shape), x, wr, bias, wg, wu, wd, out, idx, w, vp(ws) if ws else None,
                           ws_bytes, None)


GOOD = [0x1000, 0x2000, 0, 0x3000, 0x4000, 0x5000, 0x6000, 0, 0]      # fake, aligned, never dereferenced


@pytest.mark.parametrize("fields,code", [
    (dict(T=-1), 2), (dict(H=0), 2), (dict(E=0), 2), (dict(K=0), 2), (dict(K=9, E=8), 2), (dict(I=0), 2),
    (dict(H=100), 2), (dict(I=12), 2), (dict(E=1025, K=1), 2), (dict(dtype=7), 3),
    (dict(T=1 << 30, K=8, E=128), 2),
])
def test_bad_shapes_are_rejected_on_the_host(lib, fields, code):
    base = dict(T=4, H=64, E=8, K=2, I=32, dtype=0, renormalize=1)
    base.update(fields)
    shape = moe.MoeShape(*[base[k] for k in ("T", "H", "E", "K", "I", "dtype", "renormalize")])
    assert _call_forward(lib, shape, GOOD) == code
    out = ctypes.c_size_t(123)
    assert lib.moe_workspace_bytes(ctypes.byref(shape), ctypes.byref(out)) == code and out.value == 123


def test_null_alignment_and_workspace_errors(lib):
    shape = moe.make_shape(4, 64, 8, 2, 32, moe.MOE_BF16)
    for i in (0, 1, 3, 4, 5, 6):                      # every required pointer
        p = list(GOOD)
        p[i] = 0
        assert _call_forward(lib, shape, p) == 1
    p = list(GOOD)
    p[0] = 0x1008
    assert _call_forward(lib, shape, p) == 5
    p = list(GOOD)
    p[2] = 0x7004                                     # optional bias, misaligned
    assert _call_forward(lib, shape, p) == 5
    assert _call_forward(lib, shape, GOOD, ws=0) == 4
    assert _call_forward(lib, shape, GOOD, ws=0x1004) == 5
    need = moe.workspace_bytes(shape)
    assert need % 256 == 0 and need > 0
    assert _call_forward(lib, shape, GOOD, ws_bytes=need - 1) == 4
    assert lib.moe_workspace_bytes(ctypes.byref(shape), None) == 1
    assert lib.moe_workspace_bytes(None, None) == 1


def test_every_entry_point_validates_and_accepts_an_empty_batch(lib):
    vp = ctypes.c_void_p
    bad = moe.make_shape(4, 64, 8, 9, 32, moe.MOE_BF16)
    empty = moe.make_shape(0, 64, 8, 2, 32, moe.MOE_BF16)
    a = [vp(0x1000 * (i + 1)) for i in range(8)]
    big = 1 << 40
    for shape, code in ((bad, 2), (empty, 0)):
        s = ctypes.byref(shape)
        assert lib.moe_route_topk(s, a[0], a[1], None, a[2], a[3], a[4], big, None) == code
        assert lib.moe_permute(s, a[0], a[1], a[2], a[3], a[4], a[5], a[6], big, None) == code
        assert lib.moe_grouped_swiglu(s, a[0], a[1], a[2], a[3], a[4], a[5], a[6], big, None) == code
        assert lib.moe_combine(s, a[0], a[1], a[2], a[3], None) == code
        assert _call_forward(lib, shape, GOOD) == code
    s = ctypes.byref(empty)
    assert lib.moe_permute(s, a[0], None, a[2], a[3], a[4], a[5], a[6], big, None) == 1    # x_perm without x
    assert lib.moe_route_topk(s, None, a[1], None, a[2], a[3], a[4], big, None) == 1
    ms = (ctypes.c_float * moe.NUM_STAGES)()
    assert lib.moe_forward_stage_times(s, a[0], a[1], None, a[2], a[3], a[4], a[5], a[6], big, None, ms) == 0
    assert lib.moe_forward_stage_times(s, a[0], a[1], None, a[2], a[3], a[4], a[5], a[6], big, None, None) == 1


def test_binding_refuses_to_run_without_the_library(monkeypatch, tmp_path):
    monkeypatch.setattr(moe, "_lib", None)
    monkeypatch.setattr(moe, "LIB_PATH", str(tmp_path / "libmoe_ffn.so"))
    with pytest.raises(FileNotFoundError):
        moe.load_library()


def test_grpo_symbols_and_validation(lib):
    hdr = open(os.path.join(ROOT, "include", "grpo_loss.h")).read()
    declared = set(re.findall(r"\b(grpo_[a-z_]+)\s*\(", hdr))
    assert declared == set(grpo.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None
    vp = ctypes.c_void_p
    a = [vp(0x1000 * (i + 1)) for i in range(12)]
    good = grpo.GrpoShape(4, 64, 2, 0, 0.2, 0.04, 1e-6)
    for fields, code in ((dict(N=-1), 2), (dict(V=60), 2), (dict(V=0), 2), (dict(G=-1), 2), (dict(dtype=5), 3)):
        d = dict(N=4, V=64, G=2, dtype=0)
        d.update(fields)
        bad = grpo.GrpoShape(d["N"], d["V"], d["G"], d["dtype"], 0.2, 0.04, 1e-6)
        assert lib.grpo_token_logprob(ctypes.byref(bad), a[0], a[1], a[2], None) == code
        assert lib.grpo_objective(ctypes.byref(bad), *a[:9], None) == code
        assert lib.grpo_logprob_objective(ctypes.byref(bad), *a[:11], None) == code
    assert lib.grpo_token_logprob(ctypes.byref(good), None, a[1], a[2], None) == 1
    assert lib.grpo_token_logprob(ctypes.byref(good), vp(0x1004), a[1], a[2], None) == 5
    assert lib.grpo_objective(ctypes.byref(good), *a[:8], None, None) == 1
    assert lib.grpo_logprob_objective(ctypes.byref(good), *a[:10], None, None) == 1
    empty = grpo.GrpoShape(0, 64, 0, 0, 0.2, 0.04, 1e-6)
    assert lib.grpo_token_logprob(ctypes.byref(empty), a[0], a[1], a[2], None) == 0
    assert lib.grpo_logprob_objective(ctypes.byref(empty), *a[:11], None) == 0
    assert lib.grpo_token_logprob(None, a[0], a[1], a[2], None) == 1


def test_backward_validation_on_the_host(lib):
    vp = ctypes.c_void_p
    moe_backward._lib()
    a = [vp(0x1000 * (i + 1)) for i in range(14)]
    good = moe.make_shape(4, 64, 8, 2, 32, moe.MOE_BF16)
    need = ctypes.c_size_t(0)
    assert lib.moe_backward_workspace_bytes(ctypes.byref(good), ctypes.byref(need)) == 0
    assert need.value % 256 == 0 and need.value > moe.workspace_bytes(good)
    for shape, code in ((moe.make_shape(4, 64, 8, 2, 32, 7), 3),
                        (moe.make_shape(4, 60, 8, 2, 32, moe.MOE_BF16), 2), (moe.make_shape(4, 64, 8, 9, 32, moe.MOE_BF16), 2)):
        assert lib.moe_backward_workspace_bytes(ctypes.byref(shape), ctypes.byref(need)) == code
        assert lib.moe_backward(ctypes.byref(shape), *a, 1 << 40, None) == code
        assert lib.moe_grouped_swiglu_backward(ctypes.byref(shape), *a[:11], 1 << 40, None) == code
    # required pointers, alignment, workspace
    for i in (0, 1, 3, 4, 5, 6, 7, 8, 10, 11, 12):
        b = list(a)
        b[i] = None
        assert lib.moe_backward(ctypes.byref(good), *b, 1 << 40, None) == 1, i
    b = list(a)
    b[2] = None       # the bias and its gradient are optional
    b[9] = None
    b[13] = None      # ... the workspace is not
    assert lib.moe_backward(ctypes.byref(good), *b, 1 << 40, None) == 4
    b = list(a)
    b[6] = vp(0x7004)
    assert lib.moe_backward(ctypes.byref(good), *b, 1 << 40, None) == 5
    assert lib.moe_backward(ctypes.byref(good), *a, need.value - 1 if need.value else 0, None) in (4,)


def test_attention_symbols_and_validation(lib):
    hdr = open(os.path.join(ROOT, "include", "attn_decode.h")).read()
    declared = set(re.findall(r"\b(attn_decode[a-z_]*)\s*\(", hdr))
    assert declared == set(attn.EXPORTS)
    attn._lib()
    vp = ctypes.c_void_p
    a = [vp(0x1000 * (i + 1)) for i in range(7)]
    good = attn.make_shape(2, 32, 4, 8, 64)
    need = ctypes.c_size_t(0)
    assert lib.attn_decode_workspace_bytes(ctypes.byref(good), ctypes.byref(need)) == 0 and need.value % 256 == 0 and need.value > 0
    assert lib.attn_decode_workspace_bytes(ctypes.byref(good), None) == 1 and lib.attn_decode_workspace_bytes(None, None) == 1
    for bad in (attn.AttnShape(2, 32, 4, 64, 8, 64), attn.AttnShape(2, 32, 5, 128, 8, 64), attn.AttnShape(2, 64, 2, 128, 8, 64),
                attn.AttnShape(-1, 32, 4, 128, 8, 64), attn.AttnShape(2, 32, 4, 128, 8, 0)):
        assert lib.attn_decode(ctypes.byref(bad), *a, 1 << 40, None) == 2
    for i in range(6):
        b = list(a)
        b[i] = None
        assert lib.attn_decode(ctypes.byref(good), *b, 1 << 40, None) == 1
    b = list(a)
    b[6] = None
    assert lib.attn_decode(ctypes.byref(good), *b, 1 << 40, None) == 4
    assert lib.attn_decode(ctypes.byref(good), *a, need.value - 1, None) == 4
    b = list(a)
    b[1] = vp(0x2008)
    assert lib.attn_decode(ctypes.byref(good), *b, 1 << 40, None) == 5
    empty = attn.make_shape(0, 32, 4, 8, 64)
    assert lib.attn_decode(ctypes.byref(empty), *a, 1 << 40, None) == 0
