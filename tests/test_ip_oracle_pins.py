"""Pins for the InnerProduct (+ReLU) oracle: everything here runs on the CPU and checks
oracle/ip_oracle.c against things other than itself -- a hand-worked fixture, a pure-Python brute
force, the separately pinned convolution oracle with a full-size kernel, numpy's matmul, adjoint
identities, finite differences through the ReLU, and planted mistakes that the pins must catch."""
import json
import os
import subprocess

import numpy as np
import pytest

import oracle
from oracle import OracleParams
from oracle import inner_product as ipo
from oracle.inner_product import IpOracleLib, IpOracleParams

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(os.path.dirname(HERE), "oracle", "ip_oracle.c")
FIX = json.load(open(os.path.join(HERE, "golden", "ip_hand.json")))


def _rand(p, seed):
    r = np.random.default_rng(seed)
    x = r.standard_normal((p.m, p.k)).astype(np.float32).astype(np.float64)
    w = r.standard_normal((p.num_output, p.k)).astype(np.float32).astype(np.float64)
    b = r.standard_normal(p.num_output).astype(np.float32).astype(np.float64)
    dy = r.standard_normal((p.m, p.num_output)).astype(np.float32).astype(np.float64)
    return x, w, b, dy


def check_fixture(lib):
    for mode, relu in (("plain", 0), ("relu", 1)):
        p = IpOracleParams(FIX["m"], FIX["k"], FIX["num_output"], 1, relu)
        e = FIX[mode]
        y = lib.forward(p, FIX["x"], FIX["w"], FIX["b"])
        np.testing.assert_allclose(y, e["y"], rtol=0, atol=1e-14)
        dz = lib.relu_backward(p, y, FIX["dy"])
        np.testing.assert_allclose(dz, e["dz"], rtol=0, atol=0)
        np.testing.assert_allclose(lib.backward_data(p, FIX["w"], dz), e["dx"], rtol=0, atol=1e-14)
        np.testing.assert_allclose(lib.backward_filter(p, FIX["x"], dz), e["dw"], rtol=0, atol=1e-14)
        np.testing.assert_allclose(lib.backward_bias(p, dz), e["db"], rtol=0, atol=1e-14)


def check_brute(lib):
    for seed, (m, k, o, bias, relu) in enumerate([(3, 5, 4, 1, 0), (4, 7, 3, 1, 1), (2, 6, 5, 0, 1)]):
        p = IpOracleParams(m, k, o, bias, relu)
        x, w, b, dy = _rand(p, seed)
        y = np.zeros((m, o))
        for n in range(m):
            for j in range(o):
                z = b[j] if bias else 0.0
                for i in range(k):
                    z += x[n, i] * w[j, i]
                y[n, j] = max(z, 0.0) if relu else z
        got = lib.forward(p, x, w, b if bias else None)
        np.testing.assert_allclose(got, y, rtol=1e-13, atol=1e-13)
        dz = np.array([[dy[n, j] if (not relu or y[n, j] > 0) else 0.0 for j in range(o)] for n in range(m)])
        np.testing.assert_array_equal(lib.relu_backward(p, got, dy), dz)
        dx, dw, db = np.zeros((m, k)), np.zeros((o, k)), np.zeros(o)
        for n in range(m):
            for j in range(o):
                db[j] += dz[n, j]
                for i in range(k):
                    dx[n, i] += dz[n, j] * w[j, i]
                    dw[j, i] += dz[n, j] * x[n, i]
        np.testing.assert_allclose(lib.backward_data(p, w, dz), dx, rtol=1e-13, atol=1e-13)
        np.testing.assert_allclose(lib.backward_filter(p, x, dz), dw, rtol=1e-13, atol=1e-13)
        dw0 = np.full((o, k), 0.25)
        np.testing.assert_allclose(lib.backward_filter(p, x, dz, dw0, beta=1.0), dw0 + dw, rtol=1e-13, atol=1e-13)
        if bias:
            np.testing.assert_allclose(lib.backward_bias(p, dz), db, rtol=1e-13, atol=1e-13)
            db0 = np.full(o, -0.5)
            np.testing.assert_allclose(lib.backward_bias(p, dz, db0, beta=1.0), db0 + db, rtol=1e-13, atol=1e-13)


def test_hand_fixture():
    check_fixture(ipo._load())


def test_brute_force():
    check_brute(ipo._load())


def test_equals_convolution_with_full_size_kernel():
    """An inner product over a flattened [c][h][w] blob is a convolution whose kernel covers the
    whole image (output 1x1); the convolution oracle is pinned on its own."""
    n, c, h, w_, o = 5, 3, 4, 6, 7
    cp = OracleParams(n=n, c=c, h=h, w=w_, num_output=o, kernel_h=h, kernel_w=w_, bias_term=1)
    p = IpOracleParams(n, c * h * w_, o, 1, 0)
    x, w, b, dy = _rand(p, 11)
    y = ipo.forward(p, x, w, b)
    yc = oracle.forward(cp, x.reshape(n, c, h, w_), w.reshape(o, c, h, w_), b)
    np.testing.assert_allclose(y, yc.reshape(n, o), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(ipo.backward_data(p, w, dy),
                               oracle.backward_data(cp, w.reshape(o, c, h, w_), dy.reshape(n, o, 1, 1)).reshape(n, -1),
                               rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(ipo.backward_filter(p, x, dy),
                               oracle.backward_filter(cp, x.reshape(n, c, h, w_), dy.reshape(n, o, 1, 1)).reshape(o, -1),
                               rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(ipo.backward_bias(p, dy), oracle.backward_bias(cp, dy.reshape(n, o, 1, 1)),
                               rtol=1e-13, atol=1e-13)


def test_matmul():
    p = IpOracleParams(9, 33, 17, 1, 0)
    x, w, b, dy = _rand(p, 5)
    np.testing.assert_allclose(ipo.forward(p, x, w, b), x @ w.T + b, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(ipo.backward_data(p, w, dy), dy @ w, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(ipo.backward_filter(p, x, dy), dy.T @ x, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(ipo.backward_bias(p, dy), dy.sum(0), rtol=1e-12, atol=1e-12)


def test_adjoint_identities():
    p = IpOracleParams(6, 19, 8, 0, 0)
    x, w, _, g = _rand(p, 7)
    y = ipo.forward(p, x, w, None)
    lhs = float((y * g).sum())
    assert abs(lhs - float((x * ipo.backward_data(p, w, g)).sum())) <= 1e-12 * abs(lhs)
    assert abs(lhs - float((w * ipo.backward_filter(p, x, g)).sum())) <= 1e-12 * abs(lhs)


def test_finite_differences_through_relu():
    p = IpOracleParams(4, 6, 5, 1, 1)
    x, w, b, g = _rand(p, 3)
    y = ipo.forward(p, x, w, b)
    assert (y > 0).any() and (y == 0).any()
    dz = ipo.relu_backward(p, y, g)
    dx, dw, db = ipo.backward_data(p, w, dz), ipo.backward_filter(p, x, dz), ipo.backward_bias(p, dz)

    def loss(x_, w_, b_):
        return float((ipo.forward(p, x_, w_, b_) * g).sum())

    eps = 1e-6  # far smaller than the distance of any pre-activation from the kink for this seed
    for arr, grad, which in ((x, dx, 0), (w, dw, 1), (b, db, 2)):
        flat = arr.reshape(-1)
        for i in range(0, flat.size, 3):
            hi, lo = arr.copy(), arr.copy()
            hi.reshape(-1)[i] += eps
            lo.reshape(-1)[i] -= eps
            args_hi = [x, w, b]
            args_lo = [x, w, b]
            args_hi[which], args_lo[which] = hi, lo
            fd = (loss(*args_hi) - loss(*args_lo)) / (2 * eps)
            assert abs(fd - grad.reshape(-1)[i]) <= 1e-6 * max(1.0, abs(fd)), (which, i)


def test_relu_edges():
    p = IpOracleParams(1, 2, 3, 1, 1)
    x = np.array([[1.0, -1.0]])
    w = np.array([[1.0, 1.0], [2.0, 1.0], [1.0, 2.0]])   # pre-activations 0, 1, -1 with zero bias
    b = np.zeros(3)
    y = ipo.forward(p, x, w, b)
    np.testing.assert_array_equal(y, [[0.0, 1.0, 0.0]])
    np.testing.assert_array_equal(ipo.relu_backward(p, y, np.array([[5.0, 6.0, 7.0]])), [[0.0, 6.0, 0.0]])
    p0 = IpOracleParams(1, 2, 3, 1, 0)
    np.testing.assert_array_equal(ipo.forward(p0, x, w, b), [[0.0, 1.0, -1.0]])
    np.testing.assert_array_equal(ipo.relu_backward(p0, None, np.array([[5.0, 6.0, 7.0]])), [[5.0, 6.0, 7.0]])


def test_beta_zero_overwrites_without_reading():
    p = IpOracleParams(3, 4, 2, 1, 0)
    x, w, b, dy = _rand(p, 9)
    nan_w, nan_b = np.full((2, 4), np.nan), np.full(2, np.nan)
    assert np.isfinite(ipo.backward_filter(p, x, dy, nan_w, beta=0.0)).all()
    assert np.isfinite(ipo.backward_bias(p, dy, nan_b, beta=0.0)).all()


def test_argument_checks():
    p = IpOracleParams(2, 3, 2, 1, 0)
    x, w, b, dy = _rand(p, 1)
    with pytest.raises(ValueError):
        ipo.forward(p, x, w, None)              # bias_term set but no bias
    with pytest.raises(ValueError):
        ipo.forward(IpOracleParams(2, 3, 2, 0, 0), x, w, b)   # bias given but bias_term clear
    with pytest.raises(ValueError):
        ipo.backward_bias(IpOracleParams(2, 3, 2, 0, 0), dy)
    with pytest.raises(ValueError):
        ipo.forward(IpOracleParams(2, 0, 2, 0, 0), np.zeros((2, 0)), np.zeros((2, 0)), None)
    assert ipo.forward(IpOracleParams(0, 3, 2, 1, 0), np.zeros((0, 3)), w, b).shape == (0, 2)


MUTANTS = [
    ("weights_transposed", "z += x[n * K + k] * w[o * K + k];", "z += x[n * K + k] * w[k * O + o];"),
    ("drops_bias", "double z = p->bias_term ? b[o] : 0.0;", "double z = 0.0;"),
    ("relu_keeps_negatives", "y[n * O + o] = (p->relu && !(z > 0.0)) ? 0.0 : z;", "y[n * O + o] = z;"),
    ("relu_abs", "y[n * O + o] = (p->relu && !(z > 0.0)) ? 0.0 : z;", "y[n * O + o] = (p->relu && !(z > 0.0)) ? -z : z;"),
    ("mask_inverted", "dz[i] = (!p->relu || y[i] > 0.0) ? dy[i] : 0.0;", "dz[i] = (!p->relu || y[i] > 0.0) ? 0.0 : dy[i];"),
    ("mask_passes_zero", "dz[i] = (!p->relu || y[i] > 0.0) ? dy[i] : 0.0;", "dz[i] = (!p->relu || y[i] >= 0.0) ? dy[i] : 0.0;"),
    ("bwd_data_transposed", "s += dz[n * O + o] * w[o * K + k];", "s += dz[n * O + o] * w[k * O + o];"),
    ("bwd_filter_swaps_operands", "s += dz[n * O + o] * x[n * K + k];", "s += dz[n * O + k % O] * x[n * K + k];"),
    ("bwd_filter_ignores_beta", "dw[o * K + k] = (beta == 0.0) ? s : beta * dw[o * K + k] + s;", "dw[o * K + k] = s;"),
    ("bwd_bias_skips_first_row", "for (int64_t n = 0; n < M; ++n) s += dz[n * O + o];", "for (int64_t n = 1; n < M; ++n) s += dz[n * O + o];"),
    ("bwd_bias_ignores_beta", "db[o] = (beta == 0.0) ? s : beta * db[o] + s;", "db[o] = s;"),
]


def _build(text, out_dir, name):
    c, so = os.path.join(out_dir, name + ".c"), os.path.join(out_dir, name + ".so")
    with open(c, "w") as f:
        f.write(text)
    subprocess.run(["gcc", "-O1", "-std=c99", "-fPIC", "-shared", "-I", os.path.dirname(SRC), "-o", so, c], check=True)
    return IpOracleLib(so)


def _suite(lib):
    check_fixture(lib)
    check_brute(lib)


def test_unmodified_source_passes_the_compact_suite(tmp_path):
    _suite(_build(open(SRC).read(), str(tmp_path), "clean"))


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, name, old, new):
    src = open(SRC).read()
    assert old in src, f"mutation site for {name} not found"
    lib = _build(src.replace(old, new), str(tmp_path), name)
    with pytest.raises((AssertionError, ValueError)):
        _suite(lib)
