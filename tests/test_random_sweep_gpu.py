"""Randomised parameter sweep on the GPU: seeded random layer parameters (every field, including
the corners the hand-picked sweep may miss -- stride larger than the kernel, padding beyond the
kernel extent, dilation with stride, non-square everything, groups) against the CPU oracle, fp32
and fp64 paths, plus random InnerProduct shapes.  Same gates as the other parity tests."""
import os
import re
import time

import numpy as np
import pytest
import torch

import oracle
import paper_1810_02272_amd as conv
from oracle import OracleParams
from paper_1810_02272_amd import workloads
from parity_cases import (IP_RANDOM, MANY_CHANNEL, MULTI_TILE, RANDOM_BLOCKS, THIN_BLOCKS, THIN_ROW, draw_block,
                          random_ip_case, random_multi_tile_params, random_params, random_thin_group_params,
                          random_thin_row_params)
from test_f64_parity_gpu import check_full64
from test_ip_parity_gpu import run_case as run_ip_case
from test_parity_gpu import check_full
from test_pg_parity_gpu import check_batch as check_pg_batch

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("block", range(6))
def test_random_conv_parameters_fp32_and_fp64(block):
    for i, pd in enumerate(draw_block(*RANDOM_BLOCKS[block])):
        print("random case", block, i, pd, flush=True)
        seed = 31000 + 100 * block + i
        check_full(pd, seed=seed, bias=bool(pd["bias_term"]))
        op = OracleParams(**pd)
        x, w, b, dy = workloads.random_inputs(oracle.x_shape(op), oracle.w_shape(op), oracle.output_shape(op), seed,
                                              bias=bool(pd["bias_term"]))
        check_full64(pd, x.double(), w.double(), b.double() if b is not None else None, dy.double())


@pytest.mark.parametrize("block", range(4))
def test_random_thin_group_parameters_fp32_and_fp64(block):
    direct = 0
    for i, pd in enumerate(draw_block(*THIN_BLOCKS[block])):
        print("random thin-group case", block, i, pd, flush=True)
        direct += "direct" in conv.conv_desc_kernel_names(conv.conv_desc_create(conv.ConvParams(**pd)))
        seed = 52000 + 100 * block + i
        check_full(pd, seed=seed, bias=bool(pd["bias_term"]))
        op = OracleParams(**pd)
        x, w, b, dy = workloads.random_inputs(oracle.x_shape(op), oracle.w_shape(op), oracle.output_shape(op), seed,
                                              bias=bool(pd["bias_term"]))
        check_full64(pd, x.double(), w.double(), b.double() if b is not None else None, dy.double())
    assert direct >= 6, direct  # most of these shapes take the direct kernels


def check_both_types(pd, seed):
    check_full(pd, seed=seed, bias=bool(pd["bias_term"]))
    op = OracleParams(**pd)
    x, w, b, dy = workloads.random_inputs(oracle.x_shape(op), oracle.w_shape(op), oracle.output_shape(op), seed,
                                          bias=bool(pd["bias_term"]))
    check_full64(pd, x.double(), w.double(), b.double() if b is not None else None, dy.double())


def test_random_thin_row_parameters_reach_the_thin_row_kernel_and_its_staged_form():
    """Random stride-1 layers with at most four input channels or outputs per group: GEMMs of at most four rows."""
    plain = staged = 0
    for i, pd in enumerate(draw_block(*THIN_ROW)):
        names = conv.conv_desc_kernel_names(conv.conv_desc_create(conv.ConvParams(**pd)))
        print("random thin-row case", i, pd, names, flush=True)
        plain += re.search(r"corr_thin_r\d\[", names) is not None
        staged += re.search(r"corr_thin_r\d_lds", names) is not None
        check_both_types(pd, 81000 + i)
    assert plain >= 8 and staged >= 16, (plain, staged)


def test_random_multi_tile_parameters_fp32_and_fp64():
    for i, pd in enumerate(draw_block(*MULTI_TILE)):
        print("random multi-tile case", i, pd, flush=True)
        check_both_types(pd, 61000 + i)


def test_random_many_channel_parameters_reach_the_square_filter_gradient_tile():
    """Random layers with about 128 or 256 output channels per group and a reduced dimension of 100-500: the 128x128
    backward-filter tile (loads that write LDS directly) with ragged rows and columns, every bounds mode."""
    square = 0
    for i, pd in enumerate(draw_block(*MANY_CHANNEL)):
        names = conv.conv_desc_kernel_names(conv.conv_desc_create(conv.ConvParams(**pd)))
        print("random many-channel case", i, pd, names, flush=True)
        square += "wgrad_m32_128x128x32" in names
        check_both_types(pd, 71000 + i)
    assert square >= 8, square


@pytest.mark.skipif("MI355CONV_SOAK_SECONDS" not in os.environ,
                    reason="extended sweep: set MI355CONV_SOAK_SECONDS (and MI355CONV_SOAK_SEED) to run it")
def test_extended_random_sweep():
    """The four generators of this file in turn, fresh parameter sets until the time is up."""
    budget = float(os.environ["MI355CONV_SOAK_SECONDS"])
    rng = np.random.default_rng(int(os.environ.get("MI355CONV_SOAK_SEED", "987654")))
    gens = [random_params, random_thin_group_params, random_multi_tile_params, random_thin_row_params]
    t0, i, told = time.time(), 0, 0.0
    while time.time() - t0 < budget:
        pd = gens[i % 4](rng)
        if time.time() - told > 20.0:   # a progress line every 20 s (run with -s: a silent run looks hung)
            told = time.time()
            print("extended sweep case", i, pd, flush=True)
        try:
            check_both_types(pd, 900000 + i)
        except Exception:
            print("failing case", i, pd, flush=True)
            raise
        i += 1
    print("extended sweep:", i, "cases", flush=True)


@pytest.mark.skipif("MI355CONV_SOAK_SECONDS" not in os.environ,
                    reason="extended sweep: set MI355CONV_SOAK_SECONDS (and MI355CONV_SOAK_SEED) to run it")
def test_extended_random_inner_product_sweep(capsys):
    budget = float(os.environ["MI355CONV_SOAK_SECONDS"])
    rng = np.random.default_rng(int(os.environ.get("MI355CONV_SOAK_SEED", "987654")) + 1)
    t0, i, told = time.time(), 0, time.time()
    while time.time() - t0 < budget:
        m, k, o = int(rng.integers(1, 300)), int(rng.integers(1, 1500)), int(rng.integers(1, 600))
        if rng.integers(0, 3) == 0:   # small shapes: single tiles, short reductions
            m, k, o = int(rng.integers(1, 20)), int(rng.integers(1, 40)), int(rng.integers(1, 20))
        relu, bias, beta = int(rng.integers(0, 2)), bool(rng.integers(0, 2)), float(rng.integers(0, 2))
        x, w, b, dy = workloads.ip_random_inputs(m, k, o, seed=910000 + i, bias=bias)
        try:
            run_ip_case(m, k, o, bias, relu, x, w, b, dy, beta=beta, dw0=workloads.draw((o, k), "normal", 920000 + i),
                        db0=workloads.draw((o,), "normal", 930000 + i))
        except Exception:
            with capsys.disabled():
                print("failing inner-product case", i, (m, k, o, relu, bias, beta), flush=True)
            raise
        capsys.readouterr()   # drop the per-case lines of the cases that passed
        i += 1
        if time.time() - told > 20.0:
            told = time.time()
            with capsys.disabled():
                print("extended inner-product sweep: case", i, flush=True)
    with capsys.disabled():
        print("extended inner-product sweep:", i, "cases", flush=True)


@pytest.mark.skipif("MI355CONV_SOAK_SECONDS" not in os.environ,
                    reason="extended sweep: set MI355CONV_SOAK_SECONDS (and MI355CONV_SOAK_SEED) to run it")
def test_extended_random_policy_gradient_sweep(capsys):
    budget = float(os.environ["MI355CONV_SOAK_SECONDS"])
    rng = np.random.default_rng(int(os.environ.get("MI355CONV_SOAK_SEED", "987654")) + 2)
    t0, i, told = time.time(), 0, time.time()
    while time.time() - t0 < budget:
        while True:
            episodes, lo, actions = int(rng.integers(1, 300)), int(rng.integers(0, 40)), int(rng.integers(2, 130))
            hi = lo + int(rng.integers(0, 500))
            if episodes * (lo + hi) / 2 * actions < 2e6:
                break
        gamma = float(rng.choice([0.99, 0.9, 0.5, 1.0, 0.999]))
        try:
            check_pg_batch(workloads.pg_batch(episodes, lo, hi, actions, seed=940000 + i), gamma, perturb_seed=950000 + i)
        except Exception:
            with capsys.disabled():
                print("failing policy-gradient case", i, (episodes, lo, hi, actions, gamma), flush=True)
            raise
        capsys.readouterr()
        i += 1
        if time.time() - told > 20.0:
            told = time.time()
            with capsys.disabled():
                print("extended policy-gradient sweep: case", i, flush=True)
    with capsys.disabled():
        print("extended policy-gradient sweep:", i, "cases", flush=True)


def test_random_inner_product_shapes():
    rng = np.random.default_rng(IP_RANDOM[0])
    for i in range(IP_RANDOM[1]):
        m, k, o, relu, bias = random_ip_case(rng)
        x, w, b, dy = workloads.ip_random_inputs(m, k, o, seed=41000 + i, bias=bias)
        run_ip_case(m, k, o, bias, relu, x, w, b, dy, beta=float(rng.integers(0, 2)),
                    dw0=workloads.draw((o, k), "normal", 42000 + i), db0=workloads.draw((o,), "normal", 43000 + i))
