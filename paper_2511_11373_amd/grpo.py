"""Thin binding over include/grpo_loss.h (token log-probabilities and the GRPO objective): marshalling only."""
from __future__ import annotations

import ctypes

import torch

from . import moe

EXPORTS = ("grpo_token_logprob", "grpo_objective", "grpo_logprob_objective")


class GrpoShape(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int32), ("V", ctypes.c_int32), ("G", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("clip_eps", ctypes.c_float), ("beta", ctypes.c_float), ("adv_eps", ctypes.c_float)]


_ready = False


def _lib():
    global _ready
    lib = moe.load_library()
    if not _ready:
        vp = ctypes.c_void_p
        sp = ctypes.POINTER(GrpoShape)
        lib.grpo_token_logprob.argtypes = [sp, vp, vp, vp, vp]
        lib.grpo_objective.argtypes = [sp] + [vp] * 10
        lib.grpo_logprob_objective.argtypes = [sp] + [vp] * 12
        for n in EXPORTS:
            getattr(lib, n).restype = ctypes.c_int
        _ready = True
    return lib


def make_shape(N, V, G, logits_dtype, clip_eps=0.2, beta=0.04, adv_eps=1e-6) -> GrpoShape:
    code = moe.MOE_BF16 if logits_dtype == torch.bfloat16 else moe.MOE_F32
    return GrpoShape(N, V, G, code, clip_eps, beta, adv_eps)


def grpo_token_logprob(shape: GrpoShape, logits, target):
    logp = torch.empty(shape.N, dtype=torch.float32, device=logits.device)
    moe._check(_lib().grpo_token_logprob(ctypes.byref(shape), moe._ptr(logits), moe._ptr(target), moe._ptr(logp), moe._stream()))
    return logp


def _outputs(shape, device):
    f = dict(dtype=torch.float32, device=device)
    return (torch.empty(max(shape.G, 1), **f)[:shape.G], torch.empty(max(shape.N, 1), **f)[:shape.N],
            torch.empty(max(shape.G, 1), **f)[:shape.G], torch.zeros(1, **f))


def grpo_objective(shape: GrpoShape, logp, logp_old, logp_ref, rewards, resp_offsets):
    """Returns (advantage [G], token_term [N], resp_mean [G], objective [1])."""
    adv, term, mean, obj = _outputs(shape, logp.device)
    moe._check(_lib().grpo_objective(ctypes.byref(shape), moe._ptr(logp), moe._ptr(logp_old), moe._ptr(logp_ref), moe._ptr(rewards),
                                     moe._ptr(resp_offsets), moe._ptr(adv), moe._ptr(term), moe._ptr(mean), moe._ptr(obj),
                                     moe._stream()))
    return adv, term, mean, obj


def grpo_logprob_objective(shape: GrpoShape, logits, target, logp_old, logp_ref, rewards, resp_offsets, out=None):
    """Returns (logp [N], advantage [G], token_term [N], resp_mean [G], objective [1]); `out` may pass the same
    five tensors back in to avoid allocating."""
    if out is None:
        logp = torch.empty(max(shape.N, 1), dtype=torch.float32, device=logits.device)[:shape.N]
        out = (logp,) + _outputs(shape, logits.device)
    logp, adv, term, mean, obj = out
    moe._check(_lib().grpo_logprob_objective(ctypes.byref(shape), moe._ptr(logits), moe._ptr(target), moe._ptr(logp_old),
                                             moe._ptr(logp_ref), moe._ptr(rewards), moe._ptr(resp_offsets), moe._ptr(logp),
                                             moe._ptr(adv), moe._ptr(term), moe._ptr(mean), moe._ptr(obj), moe._stream()))
    return out
