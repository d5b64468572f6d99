"""CPU oracle for the Caffe-semantics ConvolutionLayer -- TEST INFRASTRUCTURE ONLY.

Thin ctypes front end for ``conv_oracle.c`` (plain C, double precision, direct
nested loops written from the layer's definition; the paper names the layer in
Table 1 and defers to C++ Caffe for its meaning).  Nothing in the GPU package may
import this module; it exists so that tests, the smoke check and the benchmark's
``cpu_baseline`` leg have something independent to compare against.

All inputs are widened to float64 before the C code sees them, so fp32 test
tensors give the exact double-precision result for those fp32 values.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv_oracle.c")
_LIB = os.path.join(_HERE, "libconv_oracle.so")

_FIELDS = ("n", "c", "h", "w", "num_output", "kernel_h", "kernel_w", "stride_h", "stride_w",
           "pad_h", "pad_w", "dilation_h", "dilation_w", "group", "bias_term")


class _CParams(ctypes.Structure):
    _fields_ = [(f, ctypes.c_int64) for f in _FIELDS]


@dataclass(frozen=True)
class OracleParams:
    n: int
    c: int
    h: int
    w: int
    num_output: int
    kernel_h: int
    kernel_w: int
    stride_h: int = 1
    stride_w: int = 1
    pad_h: int = 0
    pad_w: int = 0
    dilation_h: int = 1
    dilation_w: int = 1
    group: int = 1
    bias_term: int = 1

    def _c(self) -> _CParams:
        return _CParams(*[int(getattr(self, f)) for f in _FIELDS])


def build(force: bool = False) -> str:
    """Compile conv_oracle.c with gcc (OpenMP) into libconv_oracle.so next to it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True, cwd=_HERE)
    return _LIB


class OracleLib:
    """ctypes front end for one build of conv_oracle.c (the module-level functions use the in-tree build;
    the mutation tests load deliberately broken builds through this class)."""

    def __init__(self, path: str):
        lib = ctypes.CDLL(path)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int64)
        pp = ctypes.POINTER(_CParams)
        lib.oracle_conv_out_size.restype = ctypes.c_int64
        lib.oracle_conv_out_size.argtypes = [ctypes.c_int64] * 5
        lib.oracle_conv_output_shape.argtypes = [pp, ip, ip]
        lib.oracle_conv_forward.argtypes = [pp, dp, dp, dp, dp]
        lib.oracle_conv_backward_data.argtypes = [pp, dp, dp, dp]
        lib.oracle_conv_backward_filter.argtypes = [pp, dp, dp, dp, ctypes.c_double]
        lib.oracle_conv_backward_bias.argtypes = [pp, dp, dp, ctypes.c_double]
        lib.oracle_conv_forward_at.argtypes = [pp, dp, dp, dp, ip, ctypes.c_int64, dp]
        lib.oracle_conv_backward_data_at.argtypes = [pp, dp, dp, ip, ctypes.c_int64, dp]
        lib.oracle_conv_backward_filter_at.argtypes = [pp, dp, dp, ip, ctypes.c_int64, dp]
        lib.oracle_num_threads.restype = ctypes.c_int
        self.lib = lib

    def num_threads(self) -> int:
        return int(self.lib.oracle_num_threads())

    def out_size(self, in_size: int, kernel: int, stride: int = 1, pad: int = 0, dilation: int = 1) -> int:
        return int(self.lib.oracle_conv_out_size(in_size, kernel, stride, pad, dilation))

    def output_shape(self, p: OracleParams):
        oh, ow = ctypes.c_int64(), ctypes.c_int64()
        c = p._c()
        _check(self.lib.oracle_conv_output_shape(ctypes.byref(c), ctypes.byref(oh), ctypes.byref(ow)), "output_shape")
        return (p.n, p.num_output, int(oh.value), int(ow.value))

    def forward(self, p: OracleParams, x, w, b=None) -> np.ndarray:
        ys = self.output_shape(p)
        x, w = _f64(x, x_shape(p)), _f64(w, w_shape(p))
        b = _f64(b, (p.num_output,)) if b is not None else None
        y = np.empty(ys, dtype=np.float64)
        c = p._c()
        _check(self.lib.oracle_conv_forward(ctypes.byref(c), _dp(x), _dp(w), _dp(b), _dp(y)), "forward")
        return y

    def backward_data(self, p: OracleParams, w, dy) -> np.ndarray:
        w, dy = _f64(w, w_shape(p)), _f64(dy, self.output_shape(p))
        dx = np.empty(x_shape(p), dtype=np.float64)
        c = p._c()
        _check(self.lib.oracle_conv_backward_data(ctypes.byref(c), _dp(w), _dp(dy), _dp(dx)), "backward_data")
        return dx

    def backward_filter(self, p: OracleParams, x, dy, dw=None, beta: float = 0.0) -> np.ndarray:
        x, dy = _f64(x, x_shape(p)), _f64(dy, self.output_shape(p))
        out = np.zeros(w_shape(p), dtype=np.float64) if dw is None else _f64(dw, w_shape(p)).copy()
        c = p._c()
        _check(self.lib.oracle_conv_backward_filter(ctypes.byref(c), _dp(x), _dp(dy), _dp(out), float(beta)),
               "backward_filter")
        return out

    def backward_bias(self, p: OracleParams, dy, db=None, beta: float = 0.0) -> np.ndarray:
        dy = _f64(dy, self.output_shape(p))
        out = np.zeros((p.num_output,), dtype=np.float64) if db is None else _f64(db, (p.num_output,)).copy()
        c = p._c()
        _check(self.lib.oracle_conv_backward_bias(ctypes.byref(c), _dp(dy), _dp(out), float(beta)), "backward_bias")
        return out

    def forward_at(self, p: OracleParams, x, w, b, idx) -> np.ndarray:
        x, w = _f64(x, x_shape(p)), _f64(w, w_shape(p))
        b = _f64(b, (p.num_output,)) if b is not None else None
        idx, ip = _i64(idx)
        out = np.empty(idx.shape, dtype=np.float64)
        c = p._c()
        _check(self.lib.oracle_conv_forward_at(ctypes.byref(c), _dp(x), _dp(w), _dp(b), ip, idx.size, _dp(out)),
               "forward_at")
        return out

    def backward_data_at(self, p: OracleParams, w, dy, idx) -> np.ndarray:
        w, dy = _f64(w, w_shape(p)), _f64(dy, self.output_shape(p))
        idx, ip = _i64(idx)
        out = np.empty(idx.shape, dtype=np.float64)
        c = p._c()
        _check(self.lib.oracle_conv_backward_data_at(ctypes.byref(c), _dp(w), _dp(dy), ip, idx.size, _dp(out)),
               "backward_data_at")
        return out

    def backward_filter_at(self, p: OracleParams, x, dy, idx) -> np.ndarray:
        x, dy = _f64(x, x_shape(p)), _f64(dy, self.output_shape(p))
        idx, ip = _i64(idx)
        out = np.empty(idx.shape, dtype=np.float64)
        c = p._c()
        _check(self.lib.oracle_conv_backward_filter_at(ctypes.byref(c), _dp(x), _dp(dy), ip, idx.size, _dp(out)),
               "backward_filter_at")
        return out


def x_shape(p: OracleParams):
    return (p.n, p.c, p.h, p.w)


def w_shape(p: OracleParams):
    return (p.num_output, p.c // p.group, p.kernel_h, p.kernel_w)


def _f64(a, shape=None):
    a = np.ascontiguousarray(np.asarray(a), dtype=np.float64)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(a.shape)}")
    return a


def _dp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double)) if a is not None else None


def _i64(idx):
    idx = np.ascontiguousarray(np.asarray(idx), dtype=np.int64).reshape(-1)
    return idx, idx.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what}: invalid parameters or arguments")


_default = None


def _load() -> OracleLib:
    global _default
    if _default is None:
        build()
        _default = OracleLib(_LIB)
    return _default


def num_threads() -> int:
    return _load().num_threads()


def out_size(in_size: int, kernel: int, stride: int = 1, pad: int = 0, dilation: int = 1) -> int:
    return _load().out_size(in_size, kernel, stride, pad, dilation)


def output_shape(p: OracleParams):
    return _load().output_shape(p)


def forward(p: OracleParams, x, w, b=None) -> np.ndarray:
    return _load().forward(p, x, w, b)


def backward_data(p: OracleParams, w, dy) -> np.ndarray:
    return _load().backward_data(p, w, dy)


def backward_filter(p: OracleParams, x, dy, dw=None, beta: float = 0.0) -> np.ndarray:
    return _load().backward_filter(p, x, dy, dw, beta)


def backward_bias(p: OracleParams, dy, db=None, beta: float = 0.0) -> np.ndarray:
    return _load().backward_bias(p, dy, db, beta)


def forward_at(p: OracleParams, x, w, b, idx) -> np.ndarray:
    return _load().forward_at(p, x, w, b, idx)


def backward_data_at(p: OracleParams, w, dy, idx) -> np.ndarray:
    return _load().backward_data_at(p, w, dy, idx)


def backward_filter_at(p: OracleParams, x, dy, idx) -> np.ndarray:
    return _load().backward_filter_at(p, x, dy, idx)
