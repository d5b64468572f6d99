"""Randomised parameter sweep on the GPU: seeded random layer parameters (every field, including
the corners the hand-picked sweep may miss -- stride larger than the kernel, padding beyond the
kernel extent, dilation with stride, non-square everything, groups) against the CPU oracle, fp32
and fp64 paths, plus random InnerProduct shapes.  Same gates as the other parity tests."""
import numpy as np
import pytest
import torch

import oracle
import paper_1810_02272_amd as conv
from oracle import OracleParams
from paper_1810_02272_amd import workloads
from test_f64_parity_gpu import check_full64
from test_ip_parity_gpu import run_case as run_ip_case
from test_parity_gpu import check_full

pytestmark = pytest.mark.gpu


def random_params(rng):
    """One random, valid parameter set with a small oracle cost."""
    while True:
        g = int(rng.choice([1, 1, 1, 2, 3, 4]))
        c = g * int(rng.integers(1, 9))
        k = g * int(rng.integers(1, 13))
        kh, kw = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        sh, sw = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        dh, dw = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        ph, pw = int(rng.integers(0, 5)), int(rng.integers(0, 5))
        h, w = int(rng.integers(1, 24)), int(rng.integers(1, 24))
        n = int(rng.integers(1, 6))
        pd = dict(n=n, c=c, h=h, w=w, num_output=k, kernel_h=kh, kernel_w=kw, stride_h=sh, stride_w=sw, pad_h=ph,
                  pad_w=pw, dilation_h=dh, dilation_w=dw, group=g, bias_term=int(rng.integers(0, 2)))
        if (oracle.out_size(h, kh, sh, ph, dh) >= 1 and oracle.out_size(w, kw, sw, pw, dw) >= 1):
            return pd


@pytest.mark.parametrize("block", range(6))
def test_random_conv_parameters_fp32_and_fp64(block):
    rng = np.random.default_rng(20260 + block)
    for i in range(12):
        pd = random_params(rng)
        print("random case", block, i, pd, flush=True)
        seed = 31000 + 100 * block + i
        check_full(pd, seed=seed, bias=bool(pd["bias_term"]))
        op = OracleParams(**pd)
        x, w, b, dy = workloads.random_inputs(oracle.x_shape(op), oracle.w_shape(op), oracle.output_shape(op), seed,
                                              bias=bool(pd["bias_term"]))
        check_full64(pd, x.double(), w.double(), b.double() if b is not None else None, dy.double())


def random_thin_group_params(rng):
    """Random depthwise-like parameter sets: many groups of one or two channels, 3x3 and 5x5 kernels
    (the four-rows kernels) and arbitrary ones (the general direct kernels)."""
    while True:
        g = int(rng.integers(2, 13))
        c, k = g * int(rng.integers(1, 3)), g * int(rng.integers(1, 4))
        kh, kw = [(3, 3), (5, 5), (int(rng.integers(1, 8)), int(rng.integers(1, 8)))][int(rng.integers(0, 3))]
        sh, sw = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        if rng.integers(0, 2):
            sh = sw = 1
        dh, dw = int(rng.integers(1, 3)), int(rng.integers(1, 3))
        ph, pw = int(rng.integers(0, 5)), int(rng.integers(0, 5))
        h, w = int(rng.integers(1, 30)), int(rng.integers(1, 30))
        pd = dict(n=int(rng.integers(1, 7)), c=c, h=h, w=w, num_output=k, kernel_h=kh, kernel_w=kw, stride_h=sh,
                  stride_w=sw, pad_h=ph, pad_w=pw, dilation_h=dh, dilation_w=dw, group=g,
                  bias_term=int(rng.integers(0, 2)))
        if (oracle.out_size(h, kh, sh, ph, dh) >= 1 and oracle.out_size(w, kw, sw, pw, dw) >= 1):
            return pd


@pytest.mark.parametrize("block", range(4))
def test_random_thin_group_parameters_fp32_and_fp64(block):
    rng = np.random.default_rng(50500 + block)
    direct = 0
    for i in range(12):
        pd = random_thin_group_params(rng)
        print("random thin-group case", block, i, pd, flush=True)
        direct += "direct" in conv.conv_desc_kernel_names(conv.conv_desc_create(conv.ConvParams(**pd)))
        seed = 52000 + 100 * block + i
        check_full(pd, seed=seed, bias=bool(pd["bias_term"]))
        op = OracleParams(**pd)
        x, w, b, dy = workloads.random_inputs(oracle.x_shape(op), oracle.w_shape(op), oracle.output_shape(op), seed,
                                              bias=bool(pd["bias_term"]))
        check_full64(pd, x.double(), w.double(), b.double() if b is not None else None, dy.double())
    assert direct >= 6, direct  # most of these shapes take the direct kernels


def test_random_inner_product_shapes():
    rng = np.random.default_rng(777)
    for i in range(16):
        m, k, o = int(rng.integers(1, 200)), int(rng.integers(1, 700)), int(rng.integers(1, 300))
        relu, bias = int(rng.integers(0, 2)), bool(rng.integers(0, 2))
        x, w, b, dy = workloads.ip_random_inputs(m, k, o, seed=41000 + i, bias=bias)
        run_ip_case(m, k, o, bias, relu, x, w, b, dy, beta=float(rng.integers(0, 2)),
                    dw0=workloads.draw((o, k), "normal", 42000 + i), db0=workloads.draw((o,), "normal", 43000 + i))
