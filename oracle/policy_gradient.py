"""CPU oracle for the policy-gradient loss arithmetic (paper Appendix A and B) -- TEST
INFRASTRUCTURE ONLY.  ctypes front end for ``pg_oracle.c`` (plain C, double precision, the
paper's steps in its order).  Nothing in the GPU package may import this module."""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pg_oracle.c")
_LIB = os.path.join(_HERE, "libpg_oracle.so")


def build(force: bool = False) -> str:
    """Compile pg_oracle.c with gcc into libpg_oracle.so next to it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.run(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"],
                       check=True, cwd=_HERE)
    return _LIB


def _f64(a):
    return np.ascontiguousarray(np.asarray(a), dtype=np.float64)


def _i64(a):
    return np.ascontiguousarray(np.asarray(a), dtype=np.int64)


def _dp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double)) if a is not None else None


def _ip(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"pg oracle {what}: invalid arguments")


class PgOracleLib:
    """One build of pg_oracle.c (the mutation tests load deliberately broken builds through this)."""

    def __init__(self, path: str):
        lib = ctypes.CDLL(path)
        dp, ip, i64 = ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64), ctypes.c_int64
        lib.oracle_pg_sigmoid_sample_action.argtypes = [dp, dp, i64, ip]
        lib.oracle_pg_sigmoid_dlogps.argtypes = [dp, ip, i64, dp]
        lib.oracle_pg_softmax_dlogps.argtypes = [dp, ip, i64, i64, dp, dp]
        lib.oracle_pg_discount_rewards.argtypes = [dp, ip, i64, ctypes.c_double, dp]
        lib.oracle_pg_bottom_diff.argtypes = [dp, dp, i64, i64, ctypes.c_int, dp]
        self.lib = lib

    def sigmoid_sample_action(self, aprob, random) -> np.ndarray:
        aprob, random = _f64(aprob).reshape(-1), _f64(random).reshape(-1)
        if aprob.shape != random.shape:
            raise ValueError("aprob and random differ in length")
        out = np.empty(aprob.shape, dtype=np.int64)
        _check(self.lib.oracle_pg_sigmoid_sample_action(_dp(aprob), _dp(random), aprob.size, _ip(out)), "sample_action")
        return out

    def sigmoid_dlogps(self, aprob, action) -> np.ndarray:
        aprob, action = _f64(aprob).reshape(-1), _i64(action).reshape(-1)
        if aprob.shape != action.shape:
            raise ValueError("aprob and action differ in length")
        out = np.empty(aprob.shape, dtype=np.float64)
        _check(self.lib.oracle_pg_sigmoid_dlogps(_dp(aprob), _ip(action), aprob.size, _dp(out)), "sigmoid_dlogps")
        return out

    def softmax_dlogps(self, logits, action):
        """Returns (probs, dlogps), both [steps][actions]."""
        logits, action = _f64(logits), _i64(action).reshape(-1)
        if logits.ndim != 2 or logits.shape[0] != action.size:
            raise ValueError("logits must be [steps][actions] with one action per step")
        probs, d = np.empty_like(logits), np.empty_like(logits)
        _check(self.lib.oracle_pg_softmax_dlogps(_dp(logits), _ip(action), logits.shape[0], logits.shape[1],
                                                 _dp(probs), _dp(d)), "softmax_dlogps")
        return probs, d

    def discount_rewards(self, reward, offsets, gamma: float) -> np.ndarray:
        reward, offsets = _f64(reward).reshape(-1), _i64(offsets).reshape(-1)
        if offsets.size < 1 or offsets[-1] != reward.size:
            raise ValueError("offsets must end at the number of steps")
        out = np.empty_like(reward)
        _check(self.lib.oracle_pg_discount_rewards(_dp(reward), _ip(offsets), offsets.size - 1, float(gamma), _dp(out)),
               "discount_rewards")
        return out

    def bottom_diff(self, dlogps, discounted, sigmoid_model: bool) -> np.ndarray:
        d = _f64(dlogps)
        if d.ndim not in (1, 2):
            raise ValueError("dlogps must be [steps] or [steps][actions]")
        steps, actions = d.shape[0], (1 if d.ndim == 1 else d.shape[1])
        d2 = d.reshape(steps, actions)
        r = _f64(discounted).reshape(-1) if discounted is not None else None
        if r is not None and r.size != steps:
            raise ValueError("one discounted reward per step")
        out = np.empty_like(d2)
        _check(self.lib.oracle_pg_bottom_diff(_dp(d2), _dp(r), steps, actions, 1 if sigmoid_model else 0, _dp(out)),
               "bottom_diff")
        return out.reshape(d.shape)


_default = None


def _load() -> PgOracleLib:
    global _default
    if _default is None:
        build()
        _default = PgOracleLib(_LIB)
    return _default


def sigmoid_sample_action(aprob, random):
    return _load().sigmoid_sample_action(aprob, random)


def sigmoid_dlogps(aprob, action):
    return _load().sigmoid_dlogps(aprob, action)


def softmax_dlogps(logits, action):
    return _load().softmax_dlogps(logits, action)


def discount_rewards(reward, offsets, gamma):
    return _load().discount_rewards(reward, offsets, gamma)


def bottom_diff(dlogps, discounted, sigmoid_model):
    return _load().bottom_diff(dlogps, discounted, sigmoid_model)
