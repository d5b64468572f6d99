"""ctypes binding for libmi355conv.so: the same names as include/mi355conv.h, marshalling only.

Every compute step runs in the HIP kernels behind the C boundary.  PyTorch appears here only as
the owner of device memory and streams: tensors are checked (device, dtype, contiguity, size) and
their ``data_ptr()`` and the current stream handle are passed through.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass, fields

import torch  # imported before the library on purpose: both must share one HIP runtime

from . import build as _build

_lib = None

CONV_OK, CONV_EINVAL, CONV_ESHAPE, CONV_EWORKSPACE, CONV_EHIP = 0, -1, -2, -3, -4


class ConvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {conv_status_string(status)} (status {status})")


@dataclass(frozen=True)
class ConvParams:
    """Caffe convolution parameters plus the bottom blob shape (mirror of conv_params_t)."""
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


class _CParams(ctypes.Structure):
    _fields_ = [(f.name, ctypes.c_int32) for f in fields(ConvParams)]


def library_path() -> str:
    return _build.LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB):
        _build.build()  # nothing built yet: build once (raises if hipcc fails)
    lib = ctypes.CDLL(_build.LIB)
    vp, sz, fp = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_float
    lib.conv_desc_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(_CParams)]
    lib.conv_desc_destroy.argtypes = [vp]
    i32p = ctypes.POINTER(ctypes.c_int32)
    lib.conv_desc_output_shape.argtypes = [vp, i32p, i32p, i32p, i32p]
    lib.conv_desc_workspace_bytes.argtypes = [vp, ctypes.POINTER(sz)]
    lib.conv_forward.argtypes = [vp, vp, vp, vp, vp, vp, sz, vp]
    lib.conv_backward_data.argtypes = [vp, vp, vp, vp, vp, sz, vp]
    lib.conv_backward_filter.argtypes = [vp, vp, vp, vp, fp, vp, sz, vp]
    lib.conv_backward_bias.argtypes = [vp, vp, vp, fp, vp, sz, vp]
    lib.conv_backward_filter_bias.argtypes = [vp, vp, vp, vp, vp, fp, vp, sz, vp]
    lib.conv_backward_filter_bias.restype = ctypes.c_int
    lib.conv_backward_filter_static.argtypes = [vp, vp, vp, vp, fp, vp]
    lib.conv_backward_filter_static.restype = ctypes.c_int
    lib.conv_static_workspace_limit.argtypes = []
    lib.conv_static_workspace_limit.restype = sz
    dbl = ctypes.c_double
    lib.conv_desc_workspace_bytes_f64.argtypes = [vp, ctypes.POINTER(sz)]
    lib.conv_forward_f64.argtypes = [vp, vp, vp, vp, vp, vp, sz, vp]
    lib.conv_backward_data_f64.argtypes = [vp, vp, vp, vp, vp, sz, vp]
    lib.conv_backward_filter_f64.argtypes = [vp, vp, vp, vp, dbl, vp, sz, vp]
    lib.conv_backward_bias_f64.argtypes = [vp, vp, vp, dbl, vp, sz, vp]
    lib.conv_desc_kernel_names_f64.restype = ctypes.c_char_p
    lib.conv_desc_kernel_names_f64.argtypes = [vp]
    lib.conv_status_string.restype = ctypes.c_char_p
    lib.conv_status_string.argtypes = [ctypes.c_int]
    lib.conv_last_hip_error.restype = ctypes.c_int
    lib.conv_desc_kernel_names.restype = ctypes.c_char_p
    lib.conv_desc_kernel_names.argtypes = [vp]
    for name in ("conv_desc_create", "conv_desc_destroy", "conv_desc_output_shape", "conv_desc_workspace_bytes",
                 "conv_forward", "conv_backward_data", "conv_backward_filter", "conv_backward_bias",
                 "conv_desc_workspace_bytes_f64", "conv_forward_f64", "conv_backward_data_f64",
                 "conv_backward_filter_f64", "conv_backward_bias_f64"):
        getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def conv_status_string(status: int) -> str:
    return _load().conv_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != CONV_OK:
        raise ConvError(status, where)


class ConvDesc:
    """Owner of a conv_desc_t*; destroyed with the Python object (or conv_desc_destroy)."""

    def __init__(self, handle: int, params: ConvParams):
        self.handle = handle
        self.params = params

    def __del__(self):
        try:
            conv_desc_destroy(self)
        except Exception:
            pass


def conv_desc_create(params: ConvParams) -> ConvDesc:
    lib = _load()
    c = _CParams(*[int(getattr(params, f.name)) for f in fields(ConvParams)])
    out = ctypes.c_void_p()
    _check(lib.conv_desc_create(ctypes.byref(out), ctypes.byref(c)), "conv_desc_create")
    return ConvDesc(out.value, params)


def conv_desc_destroy(desc: ConvDesc) -> None:
    if desc.handle:
        _load().conv_desc_destroy(desc.handle)
        desc.handle = None


def conv_desc_output_shape(desc: ConvDesc):
    n, k, oh, ow = (ctypes.c_int32() for _ in range(4))
    _check(_load().conv_desc_output_shape(desc.handle, ctypes.byref(n), ctypes.byref(k), ctypes.byref(oh),
                                          ctypes.byref(ow)), "conv_desc_output_shape")
    return (n.value, k.value, oh.value, ow.value)


def conv_desc_workspace_bytes(desc: ConvDesc) -> int:
    b = ctypes.c_size_t()
    _check(_load().conv_desc_workspace_bytes(desc.handle, ctypes.byref(b)), "conv_desc_workspace_bytes")
    return int(b.value)


def conv_desc_kernel_names(desc: ConvDesc) -> str:
    return _load().conv_desc_kernel_names(desc.handle).decode()


def _x_shape(p):
    return (p.n, p.c, p.h, p.w)


def _w_shape(p):
    return (p.num_output, p.c // p.group, p.kernel_h, p.kernel_w)


def _ptr(t, shape, name, dtype=torch.float32):
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name}: expected a CUDA/HIP tensor (there is no CPU path)")
    if t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{name}: expected a contiguous {dtype} tensor")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: expected shape {tuple(shape)}, got {tuple(t.shape)}")
    return t.data_ptr() or None


def _ws(ws):
    if ws is None:
        return None, 0
    if not ws.is_cuda or not ws.is_contiguous():
        raise TypeError("workspace: expected a contiguous device tensor")
    return ws.data_ptr(), ws.numel() * ws.element_size()


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def conv_forward(desc, x, w, bias, y, ws=None, stream=None) -> None:
    p = desc.params
    wp, wb = _ws(ws)
    _check(_load().conv_forward(desc.handle, _ptr(x, _x_shape(p), "x"), _ptr(w, _w_shape(p), "w"),
                                _ptr(bias, (p.num_output,), "bias"), _ptr(y, conv_desc_output_shape(desc), "y"),
                                wp, wb, _stream(stream)), "conv_forward")


def conv_backward_data(desc, w, dy, dx, ws=None, stream=None) -> None:
    p = desc.params
    wp, wb = _ws(ws)
    _check(_load().conv_backward_data(desc.handle, _ptr(w, _w_shape(p), "w"),
                                      _ptr(dy, conv_desc_output_shape(desc), "dy"), _ptr(dx, _x_shape(p), "dx"),
                                      wp, wb, _stream(stream)), "conv_backward_data")


def conv_backward_filter(desc, x, dy, dw, beta=0.0, ws=None, stream=None) -> None:
    p = desc.params
    wp, wb = _ws(ws)
    _check(_load().conv_backward_filter(desc.handle, _ptr(x, _x_shape(p), "x"),
                                        _ptr(dy, conv_desc_output_shape(desc), "dy"), _ptr(dw, _w_shape(p), "dw"),
                                        float(beta), wp, wb, _stream(stream)), "conv_backward_filter")


def conv_backward_filter_bias(desc, x, dy, dw, db, beta=0.0, ws=None, stream=None) -> None:
    p = desc.params
    wp, wb = _ws(ws)
    _check(_load().conv_backward_filter_bias(desc.handle, _ptr(x, _x_shape(p), "x"),
                                             _ptr(dy, conv_desc_output_shape(desc), "dy"), _ptr(dw, _w_shape(p), "dw"),
                                             _ptr(db, (p.num_output,), "db"), float(beta), wp, wb, _stream(stream)),
           "conv_backward_filter_bias")


def conv_backward_filter_static(desc, x, dy, dw, beta=0.0, stream=None) -> None:
    """conv_backward_filter without a workspace argument: the library's own fixed device array holds the
    split partials; nothing is allocated."""
    p = desc.params
    _check(_load().conv_backward_filter_static(desc.handle, _ptr(x, _x_shape(p), "x"),
                                               _ptr(dy, conv_desc_output_shape(desc), "dy"),
                                               _ptr(dw, _w_shape(p), "dw"), float(beta), _stream(stream)),
           "conv_backward_filter_static")


def conv_static_workspace_limit() -> int:
    return int(_load().conv_static_workspace_limit())


def conv_backward_bias(desc, dy, db, beta=0.0, ws=None, stream=None) -> None:
    p = desc.params
    wp, wb = _ws(ws)
    _check(_load().conv_backward_bias(desc.handle, _ptr(dy, conv_desc_output_shape(desc), "dy"),
                                      _ptr(db, (p.num_output,), "db"), float(beta), wp, wb, _stream(stream)),
           "conv_backward_bias")


# ---- double base type: the same calls on float64 tensors ----
_F64 = torch.float64


def conv_desc_workspace_bytes_f64(desc: ConvDesc) -> int:
    b = ctypes.c_size_t()
    _check(_load().conv_desc_workspace_bytes_f64(desc.handle, ctypes.byref(b)), "conv_desc_workspace_bytes_f64")
    return int(b.value)


def conv_desc_kernel_names_f64(desc: ConvDesc) -> str:
    return _load().conv_desc_kernel_names_f64(desc.handle).decode()


def conv_forward_f64(desc, x, w, bias, y, ws=None, stream=None) -> None:
    p = desc.params
    wp, wb = _ws(ws)
    _check(_load().conv_forward_f64(desc.handle, _ptr(x, _x_shape(p), "x", _F64), _ptr(w, _w_shape(p), "w", _F64),
                                    _ptr(bias, (p.num_output,), "bias", _F64),
                                    _ptr(y, conv_desc_output_shape(desc), "y", _F64), wp, wb, _stream(stream)),
           "conv_forward_f64")


def conv_backward_data_f64(desc, w, dy, dx, ws=None, stream=None) -> None:
    p = desc.params
    wp, wb = _ws(ws)
    _check(_load().conv_backward_data_f64(desc.handle, _ptr(w, _w_shape(p), "w", _F64),
                                          _ptr(dy, conv_desc_output_shape(desc), "dy", _F64),
                                          _ptr(dx, _x_shape(p), "dx", _F64), wp, wb, _stream(stream)),
           "conv_backward_data_f64")


def conv_backward_filter_f64(desc, x, dy, dw, beta=0.0, ws=None, stream=None) -> None:
    p = desc.params
    wp, wb = _ws(ws)
    _check(_load().conv_backward_filter_f64(desc.handle, _ptr(x, _x_shape(p), "x", _F64),
                                            _ptr(dy, conv_desc_output_shape(desc), "dy", _F64),
                                            _ptr(dw, _w_shape(p), "dw", _F64), float(beta), wp, wb, _stream(stream)),
           "conv_backward_filter_f64")


def conv_backward_bias_f64(desc, dy, db, beta=0.0, ws=None, stream=None) -> None:
    p = desc.params
    wp, wb = _ws(ws)
    _check(_load().conv_backward_bias_f64(desc.handle, _ptr(dy, conv_desc_output_shape(desc), "dy", _F64),
                                          _ptr(db, (p.num_output,), "db", _F64), float(beta), wp, wb,
                                          _stream(stream)), "conv_backward_bias_f64")
