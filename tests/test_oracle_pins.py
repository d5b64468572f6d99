"""Pins for the CPU oracle (no GPU, no GPU library).

The oracle is the only thing the GPU kernels are compared with, so it is pinned here to
things other than itself:
  * hand-worked fixtures under tests/golden/ (values derived with pencil and paper),
  * the output-size table,
  * a brute-force evaluation of the definition in pure Python on tiny inputs,
  * exact invariants: adjoint identity, bilinear twin, finite differences,
  * special cases that reduce to library routines (matmul, dot, slicing, zero padding),
  * torch's float64 conv2d and its autograd as a third opinion.
"""
import glob
import itertools
import json
import os

import numpy as np
import pytest
import torch

import oracle
from oracle import OracleParams

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
RNG = np.random.default_rng(20181002)


def _rand(shape):
    return RNG.standard_normal(shape)


# ----------------------------------------------------------------------------- hand fixtures
@pytest.mark.parametrize("path", sorted(glob.glob(os.path.join(GOLDEN, "hand_*.json"))))
def test_hand_fixture(path):
    fx = json.load(open(path))
    p = OracleParams(**fx["params"])
    x, w = np.array(fx["x"], float), np.array(fx["w"], float)
    b = np.array(fx["b"], float) if p.bias_term else None
    np.testing.assert_array_equal(oracle.forward(p, x, w, b), np.array(fx["y"], float))
    idx = np.arange(np.array(fx["y"]).size)
    np.testing.assert_array_equal(oracle.forward_at(p, x, w, b, idx), np.array(fx["y"], float).ravel())
    if "dy" in fx:
        dy = np.array(fx["dy"], float)
        np.testing.assert_array_equal(oracle.backward_data(p, w, dy), np.array(fx["dx"], float))
        np.testing.assert_array_equal(oracle.backward_data_at(p, w, dy, np.arange(x.size)),
                                      np.array(fx["dx"], float).ravel())
        np.testing.assert_array_equal(oracle.backward_filter(p, x, dy), np.array(fx["dw"], float))
        np.testing.assert_array_equal(oracle.backward_filter_at(p, x, dy, np.arange(w.size)),
                                      np.array(fx["dw"], float).ravel())
        if p.bias_term:
            np.testing.assert_array_equal(oracle.backward_bias(p, dy), np.array(fx["db"], float))


def test_output_size_table():
    table = json.load(open(os.path.join(GOLDEN, "output_sizes.json")))
    for i, k, s, pad, d, out in table["rows"]:
        assert oracle.out_size(i, k, s, pad, d) == out, (i, k, s, pad, d)


def test_output_shape_rejects_empty_output():
    with pytest.raises(ValueError):
        oracle.output_shape(OracleParams(1, 1, 4, 4, 1, 5, 5))
    with pytest.raises(ValueError):
        oracle.output_shape(OracleParams(1, 3, 8, 8, 4, 3, 3, group=2))  # 3 % 2 != 0


# ----------------------------------------------------------------------------- brute force
def _brute(p, x, w, b, dy):
    """The definition, as written, in pure Python (tiny inputs only)."""
    _, K, OH, OW = oracle.output_shape(p)
    Cg, Kg = p.c // p.group, K // p.group
    y = np.zeros((p.n, K, OH, OW))
    dx = np.zeros_like(x, dtype=float)
    dw = np.zeros_like(w, dtype=float)
    db = np.zeros(K)
    for n, k, oh, ow in itertools.product(range(p.n), range(K), range(OH), range(OW)):
        g = k // Kg
        acc = b[k] if b is not None else 0.0
        db[k] += dy[n, k, oh, ow]
        for cc, i, j in itertools.product(range(Cg), range(p.kernel_h), range(p.kernel_w)):
            ih = oh * p.stride_h - p.pad_h + i * p.dilation_h
            iw = ow * p.stride_w - p.pad_w + j * p.dilation_w
            if 0 <= ih < p.h and 0 <= iw < p.w:
                acc += w[k, cc, i, j] * x[n, g * Cg + cc, ih, iw]
                dx[n, g * Cg + cc, ih, iw] += w[k, cc, i, j] * dy[n, k, oh, ow]
                dw[k, cc, i, j] += dy[n, k, oh, ow] * x[n, g * Cg + cc, ih, iw]
        y[n, k, oh, ow] = acc
    return y, dx, dw, db


SMALL = [
    OracleParams(2, 3, 5, 6, 4, 3, 2),
    OracleParams(1, 4, 7, 5, 6, 3, 3, stride_h=2, stride_w=1, pad_h=1, pad_w=2, group=2),
    OracleParams(2, 2, 6, 7, 2, 2, 3, stride_h=3, stride_w=2, pad_h=2, pad_w=0, dilation_h=2, dilation_w=1, group=2),
    OracleParams(1, 1, 4, 4, 3, 3, 3, pad_h=3, pad_w=3),                      # pad >= kernel extent
    OracleParams(3, 6, 3, 3, 9, 1, 1, group=3, bias_term=0),
    OracleParams(1, 2, 9, 8, 2, 3, 2, stride_h=2, stride_w=3, dilation_h=3, dilation_w=2, pad_h=3, pad_w=1),
]


def _draw(p):
    x = _rand(oracle.x_shape(p))
    w = _rand(oracle.w_shape(p))
    b = _rand((p.num_output,)) if p.bias_term else None
    dy = _rand(oracle.output_shape(p))
    return x, w, b, dy


@pytest.mark.parametrize("p", SMALL)
def test_matches_brute_force_definition(p):
    x, w, b, dy = _draw(p)
    y, dx, dw, db = _brute(p, x, w, b, dy)
    np.testing.assert_allclose(oracle.forward(p, x, w, b), y, rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.backward_data(p, w, dy), dx, rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.backward_filter(p, x, dy), dw, rtol=0, atol=1e-12)
    if p.bias_term:
        np.testing.assert_allclose(oracle.backward_bias(p, dy), db, rtol=0, atol=1e-12)
    # element-by-element forms agree with the whole-tensor forms
    np.testing.assert_allclose(oracle.forward_at(p, x, w, b, np.arange(y.size)), y.ravel(), atol=1e-12)
    np.testing.assert_allclose(oracle.backward_data_at(p, w, dy, np.arange(dx.size)), dx.ravel(), atol=1e-12)
    np.testing.assert_allclose(oracle.backward_filter_at(p, x, dy, np.arange(dw.size)), dw.ravel(), atol=1e-12)


# ----------------------------------------------------------------------------- invariants
MEDIUM = SMALL + [
    OracleParams(3, 8, 13, 11, 12, 5, 3, stride_h=2, stride_w=2, pad_h=2, pad_w=1, group=4),
    OracleParams(2, 3, 23, 23, 8, 11, 11, stride_h=4, stride_w=4, bias_term=0),
    OracleParams(2, 6, 9, 9, 10, 5, 5, pad_h=2, pad_w=2, group=2),
]


@pytest.mark.parametrize("p", MEDIUM)
def test_adjoint_and_bilinear_identities(p):
    x, w, _, dy = _draw(p)
    q = OracleParams(**{**p.__dict__, "bias_term": 0})
    y = oracle.forward(q, x, w, None)
    lhs = float(np.sum(y * dy))
    assert abs(lhs - float(np.sum(x * oracle.backward_data(q, w, dy)))) <= 1e-11 * max(1.0, abs(lhs))
    assert abs(lhs - float(np.sum(w * oracle.backward_filter(q, x, dy)))) <= 1e-11 * max(1.0, abs(lhs))


@pytest.mark.parametrize("p", MEDIUM[:8])
def test_finite_differences_filter_and_bias(p):
    """L = <y, dy> is linear in w and b, so a central difference is exact up to rounding."""
    x, w, b, dy = _draw(p)
    dw = oracle.backward_filter(p, x, dy)
    flat = RNG.choice(w.size, size=min(w.size, 12), replace=False)
    for f in flat:
        e = np.zeros(w.size)
        e[f] = 0.5
        e = e.reshape(w.shape)
        num = np.sum((oracle.forward(p, x, w + e, b) - oracle.forward(p, x, w - e, b)) * dy)
        assert abs(num - dw.ravel()[f]) <= 1e-9 * max(1.0, abs(num))
    if p.bias_term:
        db = oracle.backward_bias(p, dy)
        for k in range(p.num_output):
            e = np.zeros(p.num_output)
            e[k] = 0.5
            num = np.sum((oracle.forward(p, x, w, b + e) - oracle.forward(p, x, w, b - e)) * dy)
            assert abs(num - db[k]) <= 1e-9 * max(1.0, abs(num))


def test_finite_differences_data():
    p = MEDIUM[1]
    x, w, b, dy = _draw(p)
    dx = oracle.backward_data(p, w, dy)
    for f in RNG.choice(x.size, size=12, replace=False):
        e = np.zeros(x.size)
        e[f] = 0.5
        e = e.reshape(x.shape)
        num = np.sum((oracle.forward(p, x + e, w, b) - oracle.forward(p, x - e, w, b)) * dy)
        assert abs(num - dx.ravel()[f]) <= 1e-9 * max(1.0, abs(num))


# ----------------------------------------------------------------------------- reductions to library routines
def test_1x1_is_per_pixel_matmul():
    p = OracleParams(3, 5, 4, 6, 7, 1, 1)
    x, w, b, dy = _draw(p)
    ref = np.einsum("kc,nchw->nkhw", w[:, :, 0, 0], x) + b[None, :, None, None]
    np.testing.assert_allclose(oracle.forward(p, x, w, b), ref, atol=1e-12)
    np.testing.assert_allclose(oracle.backward_data(p, w, dy), np.einsum("kc,nkhw->nchw", w[:, :, 0, 0], dy), atol=1e-12)
    np.testing.assert_allclose(oracle.backward_filter(p, x, dy)[:, :, 0, 0], np.einsum("nkhw,nchw->kc", dy, x), atol=1e-12)
    np.testing.assert_allclose(oracle.backward_bias(p, dy), dy.sum(axis=(0, 2, 3)), atol=1e-12)


def test_full_size_kernel_is_inner_product():
    p = OracleParams(4, 3, 5, 6, 7, 5, 6)
    x, w, b, dy = _draw(p)
    ref = x.reshape(4, -1) @ w.reshape(7, -1).T + b
    np.testing.assert_allclose(oracle.forward(p, x, w, b).reshape(4, 7), ref, atol=1e-12)
    np.testing.assert_allclose(oracle.backward_data(p, w, dy).reshape(4, -1), dy.reshape(4, 7) @ w.reshape(7, -1), atol=1e-12)
    np.testing.assert_allclose(oracle.backward_filter(p, x, dy).reshape(7, -1), dy.reshape(4, 7).T @ x.reshape(4, -1), atol=1e-12)


def test_single_tap_kernel_is_a_shifted_crop():
    p = OracleParams(2, 1, 6, 7, 1, 3, 4, bias_term=0)
    x = _rand(oracle.x_shape(p))
    for i, j in itertools.product(range(3), range(4)):
        w = np.zeros(oracle.w_shape(p))
        w[0, 0, i, j] = 1.0
        np.testing.assert_array_equal(oracle.forward(p, x, w, None)[:, 0], x[:, 0, i:i + 4, j:j + 4])


def test_pad_equals_explicit_zero_padding():
    p = OracleParams(2, 3, 6, 5, 4, 3, 3, stride_h=2, pad_h=2, pad_w=1)
    x, w, b, dy = _draw(p)
    xp = np.pad(x, ((0, 0), (0, 0), (2, 2), (1, 1)))
    q = OracleParams(2, 3, 10, 7, 4, 3, 3, stride_h=2)
    np.testing.assert_allclose(oracle.forward(p, x, w, b), oracle.forward(q, xp, w, b), atol=1e-13)
    np.testing.assert_allclose(oracle.backward_filter(p, x, dy), oracle.backward_filter(q, xp, dy), atol=1e-12)
    np.testing.assert_allclose(oracle.backward_data(p, w, dy), oracle.backward_data(q, w, dy)[:, :, 2:-2, 1:-1], atol=1e-12)


def test_stride_is_subsampling_of_stride1():
    p1 = OracleParams(2, 2, 9, 10, 3, 3, 2, pad_h=1, pad_w=1)
    ps = OracleParams(2, 2, 9, 10, 3, 3, 2, stride_h=2, stride_w=3, pad_h=1, pad_w=1)
    x, w, b, _ = _draw(p1)
    y1, ys = oracle.forward(p1, x, w, b), oracle.forward(ps, x, w, b)
    np.testing.assert_allclose(ys, y1[:, :, ::2, ::3][:, :, :ys.shape[2], :ys.shape[3]], atol=1e-13)


def test_dilation_is_zero_stuffed_kernel():
    pd = OracleParams(2, 2, 11, 9, 3, 3, 2, dilation_h=3, dilation_w=2, pad_h=1)
    x, w, b, dy = _draw(pd)
    wz = np.zeros((3, 2, 7, 3))
    wz[:, :, ::3, ::2] = w
    pz = OracleParams(2, 2, 11, 9, 3, 7, 3, pad_h=1)
    np.testing.assert_allclose(oracle.forward(pd, x, w, b), oracle.forward(pz, x, wz, b), atol=1e-13)
    np.testing.assert_allclose(oracle.backward_data(pd, w, dy), oracle.backward_data(pz, wz, dy), atol=1e-12)
    np.testing.assert_allclose(oracle.backward_filter(pd, x, dy), oracle.backward_filter(pz, x, dy)[:, :, ::3, ::2], atol=1e-12)


def test_group_is_independent_convs_concatenated():
    p = OracleParams(2, 6, 7, 7, 9, 3, 3, pad_h=1, pad_w=1, group=3)
    x, w, b, dy = _draw(p)
    y = oracle.forward(p, x, w, b)
    dx = oracle.backward_data(p, w, dy)
    dw = oracle.backward_filter(p, x, dy)
    q = OracleParams(2, 2, 7, 7, 3, 3, 3, pad_h=1, pad_w=1)
    for g in range(3):
        cs, ks = slice(2 * g, 2 * g + 2), slice(3 * g, 3 * g + 3)
        np.testing.assert_allclose(y[:, ks], oracle.forward(q, x[:, cs], w[ks], b[ks]), atol=1e-13)
        np.testing.assert_allclose(dx[:, cs], oracle.backward_data(q, w[ks], dy[:, ks]), atol=1e-12)
        np.testing.assert_allclose(dw[ks], oracle.backward_filter(q, x[:, cs], dy[:, ks]), atol=1e-12)


def test_linearity_bias_and_beta():
    p = MEDIUM[6]
    x, w, b, dy = _draw(p)
    x2, w2 = _rand(x.shape), _rand(w.shape)
    q = OracleParams(**{**p.__dict__, "bias_term": 0})
    f = lambda xx, ww: oracle.forward(q, xx, ww, None)
    np.testing.assert_allclose(f(2 * x - 3 * x2, w), 2 * f(x, w) - 3 * f(x2, w), atol=1e-11)
    np.testing.assert_allclose(f(x, 2 * w - 3 * w2), 2 * f(x, w) - 3 * f(x, w2), atol=1e-11)
    np.testing.assert_allclose(oracle.forward(p, x, w, b), f(x, w) + b[None, :, None, None], atol=1e-12)
    # beta = 1 accumulates, beta = 0 overwrites whatever was there (even NaN)
    g = oracle.backward_filter(p, x, dy)
    np.testing.assert_allclose(oracle.backward_filter(p, x, dy, dw=g, beta=1.0), 2 * g, atol=1e-11)
    np.testing.assert_array_equal(oracle.backward_filter(p, x, dy, dw=np.full(w.shape, np.nan), beta=0.0), g)
    gb = oracle.backward_bias(p, dy)
    np.testing.assert_allclose(oracle.backward_bias(p, dy, db=gb, beta=1.0), 2 * gb, atol=1e-11)
    np.testing.assert_array_equal(oracle.backward_bias(p, dy, db=np.full(gb.shape, np.nan), beta=0.0), gb)


def test_argument_checks():
    p = OracleParams(1, 1, 3, 3, 1, 2, 2, bias_term=0)
    x, w = np.zeros((1, 1, 3, 3)), np.zeros((1, 1, 2, 2))
    with pytest.raises(ValueError):
        oracle.forward(p, x, w, np.zeros(1))          # bias given although bias_term = 0
    with pytest.raises(ValueError):
        oracle.backward_bias(p, np.zeros((1, 1, 2, 2)))
    with pytest.raises(ValueError):
        oracle.forward_at(p, x, w, None, [4])           # index out of range


def test_empty_batch():
    p = OracleParams(0, 2, 4, 4, 3, 3, 3)
    assert oracle.forward(p, np.zeros((0, 2, 4, 4)), np.zeros((3, 2, 3, 3)), np.zeros(3)).shape == (0, 3, 2, 2)
    np.testing.assert_array_equal(oracle.backward_filter(p, np.zeros((0, 2, 4, 4)), np.zeros((0, 3, 2, 2))), 0)


# ----------------------------------------------------------------------------- third opinion: torch float64
@pytest.mark.parametrize("p", MEDIUM)
def test_against_torch_float64(p):
    x, w, b, dy = _draw(p)
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    tw = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    tb = torch.tensor(b, dtype=torch.float64, requires_grad=True) if b is not None else None
    ty = torch.nn.functional.conv2d(tx, tw, tb, stride=(p.stride_h, p.stride_w), padding=(p.pad_h, p.pad_w),
                                    dilation=(p.dilation_h, p.dilation_w), groups=p.group)
    ty.backward(torch.tensor(dy))
    np.testing.assert_allclose(oracle.forward(p, x, w, b), ty.detach().numpy(), atol=1e-11)
    np.testing.assert_allclose(oracle.backward_data(p, w, dy), tx.grad.numpy(), atol=1e-11)
    np.testing.assert_allclose(oracle.backward_filter(p, x, dy), tw.grad.numpy(), atol=1e-10)
    if b is not None:
        np.testing.assert_allclose(oracle.backward_bias(p, dy), tb.grad.numpy(), atol=1e-10)


def _im2col_reference(p, x, w, b):
    """The lowering route: unfold x into a (c'*kh*kw) x (oh*ow) matrix per image and group, multiply by
    the group's weight matrix with numpy -- none of the oracle's loop structure."""
    OH = (p.h + 2 * p.pad_h - p.dilation_h * (p.kernel_h - 1) - 1) // p.stride_h + 1
    OW = (p.w + 2 * p.pad_w - p.dilation_w * (p.kernel_w - 1) - 1) // p.stride_w + 1
    Cg, Kg = p.c // p.group, p.num_output // p.group
    xp = np.zeros((p.n, p.c, p.h + 2 * p.pad_h, p.w + 2 * p.pad_w))
    xp[:, :, p.pad_h:p.pad_h + p.h, p.pad_w:p.pad_w + p.w] = x
    y = np.zeros((p.n, p.num_output, OH, OW))
    for n in range(p.n):
        for g in range(p.group):
            col = np.empty((Cg * p.kernel_h * p.kernel_w, OH * OW))
            r = 0
            for c in range(Cg):
                for i in range(p.kernel_h):
                    for j in range(p.kernel_w):
                        win = xp[n, g * Cg + c, i * p.dilation_h:i * p.dilation_h + (OH - 1) * p.stride_h + 1:p.stride_h,
                                 j * p.dilation_w:j * p.dilation_w + (OW - 1) * p.stride_w + 1:p.stride_w]
                        col[r] = win.reshape(-1)
                        r += 1
            wg = w[g * Kg:(g + 1) * Kg].reshape(Kg, -1)
            y[n, g * Kg:(g + 1) * Kg] = (wg @ col).reshape(Kg, OH, OW)
    if b is not None:
        y += b[None, :, None, None]
    return y


@pytest.mark.parametrize("seed", range(6))
def test_forward_equals_lowering_plus_matmul(seed):
    """Random parameter sets (every field) against im2col + GEMM written with numpy slicing."""
    r = np.random.default_rng(4400 + seed)
    while True:
        g = int(r.choice([1, 2, 3]))
        p = OracleParams(n=int(r.integers(1, 4)), c=g * int(r.integers(1, 5)), h=int(r.integers(3, 15)),
                         w=int(r.integers(3, 15)), num_output=g * int(r.integers(1, 5)),
                         kernel_h=int(r.integers(1, 5)), kernel_w=int(r.integers(1, 5)),
                         stride_h=int(r.integers(1, 4)), stride_w=int(r.integers(1, 4)),
                         pad_h=int(r.integers(0, 4)), pad_w=int(r.integers(0, 4)),
                         dilation_h=int(r.integers(1, 3)), dilation_w=int(r.integers(1, 3)), group=g, bias_term=1)
        if (oracle.out_size(p.h, p.kernel_h, p.stride_h, p.pad_h, p.dilation_h) >= 1
                and oracle.out_size(p.w, p.kernel_w, p.stride_w, p.pad_w, p.dilation_w) >= 1):
            break
    x = r.standard_normal(oracle.x_shape(p))
    w = r.standard_normal(oracle.w_shape(p))
    b = r.standard_normal(p.num_output)
    np.testing.assert_allclose(oracle.forward(p, x, w, b), _im2col_reference(p, x, w, b), rtol=1e-12, atol=1e-12)
