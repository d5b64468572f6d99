"""CPU oracle for the InnerProduct layer (+ optional ReLU) -- TEST INFRASTRUCTURE ONLY.

ctypes front end for ``ip_oracle.c`` (plain C, double precision, direct loops from the layer's
definition; the paper names the layer in Table 1 and Appendix A/B and defers to C++ Caffe for its
meaning).  Nothing in the GPU package may import this module.  Inputs are widened to float64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ip_oracle.c")
_LIB = os.path.join(_HERE, "libip_oracle.so")
_FIELDS = ("m", "k", "num_output", "bias_term", "relu")


class _CParams(ctypes.Structure):
    _fields_ = [(f, ctypes.c_int64) for f in _FIELDS]


@dataclass(frozen=True)
class IpOracleParams:
    m: int
    k: int
    num_output: int
    bias_term: int = 1
    relu: int = 0

    def _c(self) -> _CParams:
        return _CParams(*[int(getattr(self, f)) for f in _FIELDS])


def build(force: bool = False) -> str:
    """Compile ip_oracle.c with gcc (OpenMP) into libip_oracle.so next to it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.run(["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC],
                       check=True, cwd=_HERE)
    return _LIB


def _f64(a, shape):
    a = np.ascontiguousarray(np.asarray(a), dtype=np.float64)
    if tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(a.shape)}")
    return a


def _dp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double)) if a is not None else None


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"ip oracle {what}: invalid parameters or arguments")


class IpOracleLib:
    """One build of ip_oracle.c (the module-level functions use the in-tree build; the mutation
    tests load deliberately broken builds through this class)."""

    def __init__(self, path: str):
        lib = ctypes.CDLL(path)
        dp, pp = ctypes.POINTER(ctypes.c_double), ctypes.POINTER(_CParams)
        lib.oracle_ip_forward.argtypes = [pp, dp, dp, dp, dp]
        lib.oracle_ip_relu_backward.argtypes = [pp, dp, dp, dp]
        lib.oracle_ip_backward_data.argtypes = [pp, dp, dp, dp]
        lib.oracle_ip_backward_filter.argtypes = [pp, dp, dp, dp, ctypes.c_double]
        lib.oracle_ip_backward_bias.argtypes = [pp, dp, dp, ctypes.c_double]
        lib.oracle_ip_num_threads.restype = ctypes.c_int
        self.lib = lib

    def num_threads(self) -> int:
        return int(self.lib.oracle_ip_num_threads())

    def forward(self, p: IpOracleParams, x, w, b=None) -> np.ndarray:
        x, w = _f64(x, (p.m, p.k)), _f64(w, (p.num_output, p.k))
        b = _f64(b, (p.num_output,)) if b is not None else None
        y = np.empty((p.m, p.num_output), dtype=np.float64)
        c = p._c()
        _check(self.lib.oracle_ip_forward(ctypes.byref(c), _dp(x), _dp(w), _dp(b), _dp(y)), "forward")
        return y

    def relu_backward(self, p: IpOracleParams, y, dy) -> np.ndarray:
        y = _f64(y, (p.m, p.num_output)) if y is not None else None
        dy = _f64(dy, (p.m, p.num_output))
        dz = np.empty_like(dy)
        c = p._c()
        _check(self.lib.oracle_ip_relu_backward(ctypes.byref(c), _dp(y), _dp(dy), _dp(dz)), "relu_backward")
        return dz

    def backward_data(self, p: IpOracleParams, w, dz) -> np.ndarray:
        w, dz = _f64(w, (p.num_output, p.k)), _f64(dz, (p.m, p.num_output))
        dx = np.empty((p.m, p.k), dtype=np.float64)
        c = p._c()
        _check(self.lib.oracle_ip_backward_data(ctypes.byref(c), _dp(w), _dp(dz), _dp(dx)), "backward_data")
        return dx

    def backward_filter(self, p: IpOracleParams, x, dz, dw=None, beta: float = 0.0) -> np.ndarray:
        x, dz = _f64(x, (p.m, p.k)), _f64(dz, (p.m, p.num_output))
        out = (np.zeros((p.num_output, p.k), dtype=np.float64) if dw is None
               else _f64(dw, (p.num_output, p.k)).copy())
        c = p._c()
        _check(self.lib.oracle_ip_backward_filter(ctypes.byref(c), _dp(x), _dp(dz), _dp(out), float(beta)),
               "backward_filter")
        return out

    def backward_bias(self, p: IpOracleParams, dz, db=None, beta: float = 0.0) -> np.ndarray:
        dz = _f64(dz, (p.m, p.num_output))
        out = np.zeros((p.num_output,), dtype=np.float64) if db is None else _f64(db, (p.num_output,)).copy()
        c = p._c()
        _check(self.lib.oracle_ip_backward_bias(ctypes.byref(c), _dp(dz), _dp(out), float(beta)), "backward_bias")
        return out


_default = None


def _load() -> IpOracleLib:
    global _default
    if _default is None:
        build()
        _default = IpOracleLib(_LIB)
    return _default


def num_threads() -> int:
    return _load().num_threads()


def forward(p, x, w, b=None):
    return _load().forward(p, x, w, b)


def relu_backward(p, y, dy):
    return _load().relu_backward(p, y, dy)


def backward_data(p, w, dz):
    return _load().backward_data(p, w, dz)


def backward_filter(p, x, dz, dw=None, beta: float = 0.0):
    return _load().backward_filter(p, x, dz, dw, beta)


def backward_bias(p, dz, db=None, beta: float = 0.0):
    return _load().backward_bias(p, dz, db, beta)
