"""conv_backward_filter_static -- the filter gradient with the library's fixed device array in place
of a caller workspace -- against conv_backward_filter on the same inputs: the two run the same
kernels, so the results must agree bit for bit (and so meet the 1e-4 bar against the oracle that
conv_backward_filter is held to).  Two calls in a row, the second on a smaller layer, whose
partials then overwrite only the start of what the first call left in the array."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_1810_02272_amd as conv
from oracle import OracleParams
from paper_1810_02272_amd import binding, workloads
from parity_cases import P
from parity_metric import nerr

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
NAN = float("nan")


def both_ways(pd, seed, beta):
    op = OracleParams(**pd)
    x, w, _, dy = workloads.random_inputs(oracle.x_shape(op), oracle.w_shape(op), oracle.output_shape(op), seed)
    d = conv.conv_desc_create(conv.ConvParams(**pd))
    ws = torch.full((max(conv.conv_desc_workspace_bytes(d) // 4, 1),), NAN, device=DEV)
    xd, dyd = x.to(DEV), dy.to(DEV)
    start = workloads.draw(tuple(w.shape), "normal", seed + 1).to(DEV) if beta else torch.full(tuple(w.shape), NAN, device=DEV)
    dw_ws, dw_static = start.clone(), start.clone()
    conv.conv_backward_filter(d, xd, dyd, dw_ws, beta, ws)
    # through the C boundary itself: plain pointers, no workspace argument
    rc = binding._load().conv_backward_filter_static(d.handle, xd.data_ptr(), dyd.data_ptr(), dw_static.data_ptr(),
                                                     ctypes.c_float(beta), None)
    assert rc == 0, conv.conv_status_string(rc)
    torch.cuda.synchronize()
    assert torch.equal(dw_ws, dw_static), (pd, conv.conv_desc_kernel_names(d))
    ref = oracle.backward_filter(op, x.numpy(), dy.numpy(), dw=start.cpu().numpy() if beta else None, beta=beta)
    assert nerr(dw_static, ref) <= 1e-4
    return d


def test_static_workspace_matches_caller_workspace_twice_in_a_row_second_call_smaller():
    assert conv.conv_static_workspace_limit() == 32 << 20
    big = both_ways(P(6, 24, 29, 31, 40, 5, 5, 1, 1, 2, 2, 1, 1, 2), 8100, 0.0)      # S > 1: many partial slices
    small = both_ways(P(2, 3, 9, 11, 4, 3, 3, 2, 2, 1, 1), 8200, 1.0)                 # fewer, shorter slices; beta = 1
    assert conv.conv_desc_workspace_bytes(small) < conv.conv_desc_workspace_bytes(big)
    both_ways(P(4, 6, 13, 12, 6, 3, 3, 1, 1, 1, 1, 1, 1, 6), 8300, 0.0)               # thin groups: direct kernels
