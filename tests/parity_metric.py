"""The error metric of the parity tests.

max|gpu - ref| / max|ref| per output tensor.  The rounding error of a sum is proportional to the
magnitude of its terms, not to the magnitude of its result: a tensor of one or a few elements whose
terms happen to cancel can have max|ref| thousands of times below that magnitude, and then no
summation in the working precision, in any order, lands within the bar of the cancelled value.
Such a tensor -- and only a tensor of at most SMALL_TENSOR elements -- is measured against the scale
of its terms instead (never a smaller denominator than the plain metric, so a tensor that passes the
plain metric passes this one).  Every time that happens it is recorded in FALLBACKS, and the test
session prints the records at its end (conftest.py), so a change in how often it fires is visible.
"""
import numpy as np
import torch

import oracle

SMALL_TENSOR = 64   # the term-scale denominator applies to tensors of at most this many elements
FALLBACKS = []      # dicts: case, tensor, elements, plain (the plain metric), scaled (what was gated)


def nerr(gpu: torch.Tensor, ref: np.ndarray, floor: float = 0.0) -> float:
    """Largest absolute difference over the tensor, divided by the largest reference magnitude
    (and by no less than `floor`)."""
    g = gpu.detach().cpu().double().numpy().reshape(ref.shape)
    denom = max(float(np.max(np.abs(ref))), floor, 1e-30) if ref.size else 1.0
    return float(np.max(np.abs(g - ref))) / denom if ref.size else 0.0


def term_scale(op, which, xn, wn, bn, dyn) -> float:
    """Largest root-sum-square of the terms of an output element of one pass (the pass applied to the
    squared inputs): the magnitude an output has when its terms do not cancel."""
    sq = lambda a: None if a is None else np.square(np.asarray(a, dtype=np.float64))
    r = {"y": lambda: oracle.forward(op, sq(xn), sq(wn), sq(bn)),
         "dx": lambda: oracle.backward_data(op, sq(wn), sq(dyn)),
         "dw": lambda: oracle.backward_filter(op, sq(xn), sq(dyn)),
         "db": lambda: oracle.backward_bias(op, sq(dyn))}[which]()
    return float(np.sqrt(np.max(r))) if r.size else 0.0


def record_fallback(case, tensor, elements, plain, scaled):
    FALLBACKS.append(dict(case=case, tensor=tensor, elements=int(elements), plain=float(plain), scaled=float(scaled)))


def small_tensor_error(v, ref, tol, scale_fn, case, tensor):
    """`v` is the plain metric of a tensor with reference `ref`.  Returns v, or -- for a tensor of at
    most SMALL_TENSOR elements that misses `tol` -- v re-normalised by no less than scale_fn() (the
    term scale), recording that this happened."""
    if not (np.isfinite(v) and v > tol and 0 < ref.size <= SMALL_TENSOR):
        return v
    top = float(np.max(np.abs(ref)))
    scaled = v * top / max(top, scale_fn(), 1e-300)
    record_fallback(case, tensor, ref.size, v, scaled)
    return scaled


def gated_error(op, which, gpu, ref, tol, xn, wn, bn, dyn, case=None) -> float:
    """The normalised maximum error of one output tensor of a convolution pass (see the module text
    for the small-tensor rule)."""
    return small_tensor_error(nerr(gpu, ref), ref, tol, lambda: term_scale(op, which, xn, wn, bn, dyn), case, which)
