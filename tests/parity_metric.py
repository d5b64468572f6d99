"""The error metric of the convolution parity tests.

max|gpu - ref| / max|ref| per output tensor.  The rounding error of a sum is proportional to the
magnitude of its terms, not to the magnitude of its result: a tensor of one or a few elements whose
terms happen to cancel can have max|ref| thousands of times below that magnitude, and then no
summation in the working precision, in any order, lands within the bar of the cancelled value.
Such a tensor is measured against the scale of its terms instead (never a smaller denominator than
the plain metric, so a tensor that passes the plain metric passes this one).
"""
import numpy as np
import torch

import oracle


def nerr(gpu: torch.Tensor, ref: np.ndarray, floor: float = 0.0) -> float:
    """Largest absolute difference over the tensor, divided by the largest reference magnitude
    (and by no less than `floor`)."""
    g = gpu.detach().cpu().double().numpy().reshape(ref.shape)
    denom = max(float(np.max(np.abs(ref))), floor, 1e-30) if ref.size else 1.0
    return float(np.max(np.abs(g - ref))) / denom if ref.size else 0.0


def term_scale(op, which, xn, wn, bn, dyn) -> float:
    """Largest root-sum-square of the terms of an output element of one pass (the pass applied to the
    squared inputs): the magnitude an output has when its terms do not cancel.  A tensor of one or
    a few elements can cancel to far below it, and then no summation in the working precision is
    within the bar of the cancelled value; the bar is taken against this scale instead."""
    sq = lambda a: None if a is None else np.square(np.asarray(a, dtype=np.float64))
    r = {"y": lambda: oracle.forward(op, sq(xn), sq(wn), sq(bn)),
         "dx": lambda: oracle.backward_data(op, sq(wn), sq(dyn)),
         "dw": lambda: oracle.backward_filter(op, sq(xn), sq(dyn)),
         "db": lambda: oracle.backward_bias(op, sq(dyn))}[which]()
    return float(np.sqrt(np.max(r))) if r.size else 0.0


def gated_error(op, which, gpu, ref, tol, xn, wn, bn, dyn) -> float:
    """The normalised maximum error of one output tensor; where it misses the bar, the same error
    normalised by no less than the tensor's term scale (see term_scale)."""
    v = nerr(gpu, ref)
    if np.isfinite(v) and v > tol:
        v = nerr(gpu, ref, floor=term_scale(op, which, xn, wn, bn, dyn))
    return v
