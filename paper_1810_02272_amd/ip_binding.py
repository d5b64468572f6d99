"""ctypes binding for the InnerProduct entry points of libmi355conv.so: the same names as
include/mi355ip.h, marshalling only (every compute step runs in the HIP kernels)."""
from __future__ import annotations

import ctypes
from dataclasses import dataclass, fields

from . import binding as _b

_ready = False


@dataclass(frozen=True)
class IpParams:
    """Mirror of ip_params_t."""
    m: int
    k: int
    num_output: int
    bias_term: int = 1
    relu: int = 0


class _CParams(ctypes.Structure):
    _fields_ = [(f.name, ctypes.c_int32) for f in fields(IpParams)]


def _load():
    global _ready
    lib = _b._load()
    if not _ready:
        vp, sz, fp = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_float
        lib.ip_desc_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(_CParams)]
        lib.ip_desc_destroy.argtypes = [vp]
        lib.ip_desc_workspace_bytes.argtypes = [vp, ctypes.POINTER(sz)]
        lib.ip_desc_kernel_names.argtypes = [vp]
        lib.ip_desc_kernel_names.restype = ctypes.c_char_p
        lib.ip_forward.argtypes = [vp, vp, vp, vp, vp, vp, sz, vp]
        lib.ip_relu_backward.argtypes = [vp, vp, vp, vp, vp]
        lib.ip_backward_data.argtypes = [vp, vp, vp, vp, vp, sz, vp]
        lib.ip_backward_filter.argtypes = [vp, vp, vp, vp, fp, vp, sz, vp]
        lib.ip_backward_bias.argtypes = [vp, vp, vp, fp, vp, sz, vp]
        for name in ("ip_desc_create", "ip_desc_destroy", "ip_desc_workspace_bytes", "ip_forward", "ip_relu_backward",
                     "ip_backward_data", "ip_backward_filter", "ip_backward_bias"):
            getattr(lib, name).restype = ctypes.c_int
        _ready = True
    return lib


class IpDesc:
    """Owner of an ip_desc_t*; destroyed with the Python object (or ip_desc_destroy)."""

    def __init__(self, handle: int, params: IpParams):
        self.handle = handle
        self.params = params

    def __del__(self):
        try:
            ip_desc_destroy(self)
        except Exception:
            pass


def ip_desc_create(params: IpParams) -> IpDesc:
    c = _CParams(*[int(getattr(params, f.name)) for f in fields(IpParams)])
    out = ctypes.c_void_p()
    _b._check(_load().ip_desc_create(ctypes.byref(out), ctypes.byref(c)), "ip_desc_create")
    return IpDesc(out.value, params)


def ip_desc_destroy(desc: IpDesc) -> None:
    if desc.handle:
        _load().ip_desc_destroy(desc.handle)
        desc.handle = None


def ip_desc_workspace_bytes(desc: IpDesc) -> int:
    b = ctypes.c_size_t()
    _b._check(_load().ip_desc_workspace_bytes(desc.handle, ctypes.byref(b)), "ip_desc_workspace_bytes")
    return int(b.value)


def ip_desc_kernel_names(desc: IpDesc) -> str:
    return _load().ip_desc_kernel_names(desc.handle).decode()


def ip_forward(desc, x, w, bias, y, ws=None, stream=None) -> None:
    p = desc.params
    wp, wb = _b._ws(ws)
    _b._check(_load().ip_forward(desc.handle, _b._ptr(x, (p.m, p.k), "x"), _b._ptr(w, (p.num_output, p.k), "w"),
                                 _b._ptr(bias, (p.num_output,), "bias"), _b._ptr(y, (p.m, p.num_output), "y"),
                                 wp, wb, _b._stream(stream)), "ip_forward")


def ip_relu_backward(desc, y, dy, dz, stream=None) -> None:
    p = desc.params
    _b._check(_load().ip_relu_backward(desc.handle, _b._ptr(y, (p.m, p.num_output), "y"),
                                       _b._ptr(dy, (p.m, p.num_output), "dy"), _b._ptr(dz, (p.m, p.num_output), "dz"),
                                       _b._stream(stream)), "ip_relu_backward")


def ip_backward_data(desc, w, dz, dx, ws=None, stream=None) -> None:
    p = desc.params
    wp, wb = _b._ws(ws)
    _b._check(_load().ip_backward_data(desc.handle, _b._ptr(w, (p.num_output, p.k), "w"),
                                       _b._ptr(dz, (p.m, p.num_output), "dz"), _b._ptr(dx, (p.m, p.k), "dx"),
                                       wp, wb, _b._stream(stream)), "ip_backward_data")


def ip_backward_filter(desc, x, dz, dw, beta=0.0, ws=None, stream=None) -> None:
    p = desc.params
    wp, wb = _b._ws(ws)
    _b._check(_load().ip_backward_filter(desc.handle, _b._ptr(x, (p.m, p.k), "x"),
                                         _b._ptr(dz, (p.m, p.num_output), "dz"), _b._ptr(dw, (p.num_output, p.k), "dw"),
                                         float(beta), wp, wb, _b._stream(stream)), "ip_backward_filter")


def ip_backward_bias(desc, dz, db, beta=0.0, ws=None, stream=None) -> None:
    p = desc.params
    wp, wb = _b._ws(ws)
    _b._check(_load().ip_backward_bias(desc.handle, _b._ptr(dz, (p.m, p.num_output), "dz"),
                                       _b._ptr(db, (p.num_output,), "db"), float(beta), wp, wb, _b._stream(stream)),
              "ip_backward_bias")
