"""The error metric of the parity tests, checked on the CPU: an input whose bias gradient cancels
to 2e-5 of its terms, summed in fp32 in two ordinary orders, misses the plain 1e-4 bar although both
sums are as accurate as fp32 allows; measured against the scale of the terms both pass, and planted
mistakes still fail by orders of magnitude."""
import numpy as np
import torch

import oracle
from oracle import OracleParams
from paper_1810_02272_amd import workloads
from parity_metric import gated_error, nerr, term_scale

# found by the extended random sweep: one output channel, 2200 gradient elements
PD = dict(n=4, c=1, h=48, w=46, num_output=1, kernel_h=7, kernel_w=3, stride_h=4, stride_w=1, pad_h=1, pad_w=4,
          dilation_h=1, dilation_w=2, group=1, bias_term=1)
SEED = 947633


def inputs():
    op = OracleParams(**PD)
    x, w, b, dy = workloads.random_inputs(oracle.x_shape(op), oracle.w_shape(op), oracle.output_shape(op), SEED)
    return op, x.numpy(), w.numpy(), b.numpy(), dy.numpy()


def test_cancelled_bias_gradient_fp32_sums_miss_the_plain_bar_but_not_the_term_scale():
    op, xn, wn, bn, dyn = inputs()
    ref = oracle.backward_bias(op, dyn)
    assert ref.shape == (1,) and abs(ref[0]) < 0.05 and np.abs(dyn).sum() > 1500.0   # cancels to 2e-5 of its terms
    scale = term_scale(op, "db", xn, wn, bn, dyn)
    assert abs(scale - np.sqrt(np.sum(dyn.astype(np.float64) ** 2))) < 1e-9 * scale
    flat = dyn.astype(np.float32).ravel()
    sequential = np.float32(0)
    for v in flat:
        sequential = np.float32(sequential + v)
    pairwise = flat.sum(dtype=np.float32)
    missed = 0
    for s in (sequential, pairwise):
        got = torch.tensor([float(s)], dtype=torch.float64)
        missed += nerr(got, ref) > 1e-4
        # accurate to a few units of fp32 rounding of the terms' scale all the same
        assert nerr(got, ref, floor=scale) < 1e-6
        assert gated_error(op, "db", got, ref, 1e-4, xn, wn, bn, dyn) < 1e-6
    assert missed >= 1


def test_term_scale_does_not_hide_mistakes():
    op, xn, wn, bn, dyn = inputs()
    ref = oracle.backward_bias(op, dyn)
    d = dyn.astype(np.float64)
    dropped_term = torch.tensor([d.sum() - d[1, 0, 3, 7]])
    dropped_image = torch.tensor([d[:3].sum()])
    for wrong in (dropped_term, dropped_image):
        assert gated_error(op, "db", wrong, ref, 1e-4, xn, wn, bn, dyn) > 1e-3
    # forward: a missing bias, a missing tap
    y = oracle.forward(op, xn, wn, bn)
    assert gated_error(op, "y", torch.from_numpy(y - bn[0]), y, 1e-4, xn, wn, bn, dyn) > 1e-3
    w2 = wn.copy()
    w2[0, 0, 6, 2] = 0.0
    assert gated_error(op, "y", torch.from_numpy(oracle.forward(op, xn, w2, bn)), y, 1e-4, xn, wn, bn, dyn) > 1e-3


def test_floor_never_lowers_the_denominator():
    ref = np.array([3.0, -4.0])
    got = torch.tensor([3.0, -4.5], dtype=torch.float64)
    assert nerr(got, ref) == nerr(got, ref, floor=1.0) == 0.125   # a floor below max|ref| changes nothing
    assert nerr(got, ref, floor=8.0) == 0.0625
    assert nerr(torch.zeros(0), np.zeros(0)) == 0.0


def test_only_small_tensors_take_the_term_scale_and_every_use_is_recorded():
    import parity_metric

    before = len(parity_metric.FALLBACKS)
    ref = np.full(parity_metric.SMALL_TENSOR + 1, 1e-3)
    got = torch.from_numpy(ref + 1e-6)                       # 1e-3 of the plain scale: misses 1e-4
    scale = lambda: 1e3                                      # a term scale that would hide it
    v = parity_metric.small_tensor_error(nerr(got, ref), ref, 1e-4, scale, "big", "y")
    assert v > 1e-4 and len(parity_metric.FALLBACKS) == before          # too many elements: plain metric, no record
    small = ref[:parity_metric.SMALL_TENSOR]
    v = parity_metric.small_tensor_error(nerr(got[:len(small)], small), small, 1e-4, scale, "small", "y")
    assert v < 1e-8 and len(parity_metric.FALLBACKS) == before + 1
    rec = parity_metric.FALLBACKS[-1]
    assert rec["case"] == "small" and rec["tensor"] == "y" and rec["plain"] > 1e-4 and rec["scaled"] == v
    # a tensor that meets the plain bar is never re-normalised or recorded
    ok = torch.from_numpy(small * (1 + 1e-6))
    assert parity_metric.small_tensor_error(nerr(ok, small), small, 1e-4, scale, "ok", "y") == nerr(ok, small)
    assert len(parity_metric.FALLBACKS) == before + 1
