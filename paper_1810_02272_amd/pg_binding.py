"""ctypes binding for the policy-gradient entry points of libmi355conv.so: the same names as
include/mi355pg.h, marshalling only (every compute step runs in the HIP kernels)."""
from __future__ import annotations

import ctypes

import torch

from . import binding as _b

_ready = False


def _load():
    global _ready
    lib = _b._load()
    if not _ready:
        vp, i32, fp = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float
        lib.pg_sigmoid_sample_action.argtypes = [vp, vp, vp, i32, vp]
        lib.pg_discount_rewards.argtypes = [vp, vp, i32, i32, fp, vp, vp]
        lib.pg_sigmoid_bottom_diff.argtypes = [vp, vp, vp, vp, vp, i32, vp]
        lib.pg_softmax_bottom_diff.argtypes = [vp, vp, vp, vp, vp, i32, i32, vp]
        for name in ("pg_sigmoid_sample_action", "pg_discount_rewards", "pg_sigmoid_bottom_diff",
                     "pg_softmax_bottom_diff"):
            getattr(lib, name).restype = ctypes.c_int
        _ready = True
    return lib


def _iptr(t, shape, name):
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name}: expected a CUDA/HIP tensor (there is no CPU path)")
    if t.dtype != torch.int32 or not t.is_contiguous():
        raise TypeError(f"{name}: expected a contiguous int32 tensor")
    if tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: expected shape {tuple(shape)}, got {tuple(t.shape)}")
    return t.data_ptr() or None


def pg_sigmoid_sample_action(aprob, random, action, stream=None) -> None:
    steps = aprob.numel()
    _b._check(_load().pg_sigmoid_sample_action(_b._ptr(aprob, (steps,), "aprob"), _b._ptr(random, (steps,), "random"),
                                               _iptr(action, (steps,), "action"), steps, _b._stream(stream)),
              "pg_sigmoid_sample_action")


def pg_discount_rewards(reward, episode_offsets, gamma, discounted, stream=None) -> None:
    steps, episodes = reward.numel(), episode_offsets.numel() - 1
    _b._check(_load().pg_discount_rewards(_b._ptr(reward, (steps,), "reward"),
                                          _iptr(episode_offsets, (episodes + 1,), "episode_offsets"), episodes, steps,
                                          float(gamma), _b._ptr(discounted, (steps,), "discounted"),
                                          _b._stream(stream)), "pg_discount_rewards")


def pg_sigmoid_bottom_diff(aprob, action, discounted, dlogps, bottom_diff, stream=None) -> None:
    steps = aprob.numel()
    _b._check(_load().pg_sigmoid_bottom_diff(_b._ptr(aprob, (steps,), "aprob"), _iptr(action, (steps,), "action"),
                                             _b._ptr(discounted, (steps,), "discounted"),
                                             _b._ptr(dlogps, (steps,), "dlogps"),
                                             _b._ptr(bottom_diff, (steps,), "bottom_diff"), steps, _b._stream(stream)),
              "pg_sigmoid_bottom_diff")


def pg_softmax_bottom_diff(logits, action, discounted, probs, bottom_diff, stream=None) -> None:
    steps, actions = logits.shape
    _b._check(_load().pg_softmax_bottom_diff(_b._ptr(logits, (steps, actions), "logits"),
                                             _iptr(action, (steps,), "action"),
                                             _b._ptr(discounted, (steps,), "discounted"),
                                             _b._ptr(probs, (steps, actions), "probs"),
                                             _b._ptr(bottom_diff, (steps, actions), "bottom_diff"), steps, actions,
                                             _b._stream(stream)), "pg_softmax_bottom_diff")
