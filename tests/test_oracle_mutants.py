"""Do the oracle's pins bite?  Each case plants one plausible mistake in a copy of conv_oracle.c
(a dropped term, a wrong sign or index, a transposed operand, an off-by-one), builds it on the
CPU and runs a compact version of the pin suite against it: the hand-worked fixtures, the
output-size table and a brute force of the definition on small shapes.  Every mutant must be
caught; the unmodified source must pass the same suite.  (No GPU involved.)"""
import glob
import itertools
import json
import os
import subprocess

import numpy as np
import pytest

import oracle
from oracle import OracleLib, OracleParams

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(os.path.dirname(HERE), "oracle", "conv_oracle.c")
GOLDEN = os.path.join(HERE, "golden")

# (name, text to find, replacement) -- the text must occur in conv_oracle.c
MUTANTS = [
    ("out_size_ceil", "return floor_div(in + 2 * pad - extent, stride) + 1;",
     "return floor_div(in + 2 * pad - extent + stride - 1, stride) + 1;"),
    ("out_size_ignores_dilation", "int64_t extent = dilation * (kernel - 1) + 1;", "int64_t extent = kernel;"),
    ("forward_drops_bias", "double acc = (p->bias_term && b) ? b[k] : 0.0;", "double acc = 0.0;"),
    ("forward_flips_kernel", "acc += w[W_AT(p, Cg, k, cc, i, j)] * x[X_AT(p, n, g * Cg + cc, ih, iw)];",
     "acc += w[W_AT(p, Cg, k, cc, p->kernel_h - 1 - i, p->kernel_w - 1 - j)] * x[X_AT(p, n, g * Cg + cc, ih, iw)];"),
    ("forward_ignores_group_offset", "acc += w[W_AT(p, Cg, k, cc, i, j)] * x[X_AT(p, n, g * Cg + cc, ih, iw)];",
     "acc += w[W_AT(p, Cg, k, cc, i, j)] * x[X_AT(p, n, cc, ih, iw)];"),
    ("group_by_modulo", "const int64_t g = k / Kg;\n  double acc", "const int64_t g = k % p->group;\n  double acc"),
    ("forward_pad_sign", "const int64_t ih = oh * p->stride_h - p->pad_h + i * p->dilation_h;\n        const int64_t iw = ow * p->stride_w - p->pad_w + j * p->dilation_w;\n        if (ih < 0 || ih >= p->h || iw < 0 || iw >= p->w) continue; /* zero extension */",
     "const int64_t ih = oh * p->stride_h + p->pad_h + i * p->dilation_h;\n        const int64_t iw = ow * p->stride_w - p->pad_w + j * p->dilation_w;\n        if (ih < 0 || ih >= p->h || iw < 0 || iw >= p->w) continue; /* zero extension */"),
    ("forward_swaps_strides", "const int64_t ih = oh * p->stride_h - p->pad_h + i * p->dilation_h;\n        const int64_t iw = ow * p->stride_w - p->pad_w + j * p->dilation_w;\n        if (ih < 0 || ih >= p->h || iw < 0 || iw >= p->w) continue; /* zero extension */",
     "const int64_t ih = oh * p->stride_w - p->pad_h + i * p->dilation_h;\n        const int64_t iw = ow * p->stride_h - p->pad_w + j * p->dilation_w;\n        if (ih < 0 || ih >= p->h || iw < 0 || iw >= p->w) continue; /* zero extension */"),
    ("weight_index_transposed", "#define W_AT(p, Cg, k_, c_, i_, j_) ((((k_) * (Cg) + (c_)) * (p)->kernel_h + (i_)) * (p)->kernel_w + (j_))",
     "#define W_AT(p, Cg, k_, c_, i_, j_) ((((k_) * (Cg) + (c_)) * (p)->kernel_w + (j_)) * (p)->kernel_h + (i_))"),
    ("bwd_data_wrong_sign", "dx[X_AT(p, n, g * Cg + cc, ih, iw)] += w[W_AT(p, Cg, k, cc, i, j)] * gy;",
     "dx[X_AT(p, n, g * Cg + cc, ih, iw)] -= w[W_AT(p, Cg, k, cc, i, j)] * gy;"),
    ("bwd_data_ignores_dilation", "const int64_t ih = oh * p->stride_h - p->pad_h + i * p->dilation_h;\n                const int64_t iw = ow * p->stride_w - p->pad_w + j * p->dilation_w;",
     "const int64_t ih = oh * p->stride_h - p->pad_h + i;\n                const int64_t iw = ow * p->stride_w - p->pad_w + j * p->dilation_w;"),
    ("bwd_data_no_zeroing", "dx[n * p->c * p->h * p->w + e] = 0.0;", "dx[n * p->c * p->h * p->w + e] *= 1.0;"),
    ("bwd_data_at_no_divisibility", "if (th < 0 || th % p->stride_h != 0) continue;", "if (th < 0) continue;"),
    ("bwd_data_at_off_by_one", "if (ow >= OW) continue;", "if (ow > OW) continue;"),
    ("bwd_data_at_wrong_group", "for (int64_t k = g * Kg; k < (g + 1) * Kg; ++k)", "for (int64_t k = 0; k < Kg; ++k)"),
    ("bwd_filter_ignores_beta", "dw[at] = (beta == 0.0 ? 0.0 : beta * dw[at]) + grad;", "dw[at] = grad;"),
    ("bwd_filter_wrong_tap", "const int64_t iw = ow * p->stride_w - p->pad_w + j * p->dilation_w;\n        if (iw < 0 || iw >= p->w) continue;\n        acc += dy",
     "const int64_t iw = ow * p->stride_w - p->pad_w + i * p->dilation_w;\n        if (iw < 0 || iw >= p->w) continue;\n        acc += dy"),
    ("bwd_filter_skips_first_image", "for (int64_t n = 0; n < p->n; ++n)\n    for (int64_t oh = 0; oh < OH; ++oh) {\n      const int64_t ih",
     "for (int64_t n = 1; n < p->n; ++n)\n    for (int64_t oh = 0; oh < OH; ++oh) {\n      const int64_t ih"),
    ("bwd_bias_skips_last_column", "for (int64_t ow = 0; ow < OW; ++ow) acc += dy[Y_AT(p, OH, OW, n, k, oh, ow)];",
     "for (int64_t ow = 0; ow + 1 < OW; ++ow) acc += dy[Y_AT(p, OH, OW, n, k, oh, ow)];"),
    ("bwd_bias_ignores_beta", "db[k] = (beta == 0.0 ? 0.0 : beta * db[k]) + acc;", "db[k] = acc;"),
    ("output_index_swaps_oh_ow", "#define Y_AT(p, OH, OW, n_, k_, oh_, ow_) ((((n_) * (p)->num_output + (k_)) * (OH) + (oh_)) * (OW) + (ow_))",
     "#define Y_AT(p, OH, OW, n_, k_, oh_, ow_) ((((n_) * (p)->num_output + (k_)) * (OW) + (ow_)) * (OH) + (oh_))"),
]


def _build(src_text: str, out_dir: str, name: str) -> OracleLib:
    c = os.path.join(out_dir, name + ".c")
    so = os.path.join(out_dir, name + ".so")
    with open(c, "w") as f:
        f.write(src_text)
    subprocess.run(["gcc", "-O1", "-std=c99", "-fPIC", "-shared", "-I", os.path.dirname(SRC), "-o", so, c], check=True)
    return OracleLib(so)


def _brute(p, x, w, b, dy, OH, OW):
    K = p.num_output
    Cg, Kg = p.c // p.group, K // p.group
    y = np.zeros((p.n, K, OH, OW))
    dx, dw, db = np.zeros_like(x), np.zeros_like(w), np.zeros(K)
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


def _size(i, k, s, p, d):
    return (i + 2 * p - d * (k - 1) - 1) // s + 1


SHAPES = [
    OracleParams(2, 4, 7, 6, 6, 3, 2, stride_h=2, stride_w=1, pad_h=1, pad_w=2, dilation_h=2, dilation_w=1, group=2),
    OracleParams(2, 3, 6, 7, 2, 2, 3, stride_h=1, stride_w=3, pad_h=0, pad_w=1),
]


def pin_suite(lib: OracleLib) -> None:
    """Raises AssertionError / ValueError if `lib` disagrees with the pins."""
    table = json.load(open(os.path.join(GOLDEN, "output_sizes.json")))
    for i, k, s, pad, d, out in table["rows"]:
        assert lib.out_size(i, k, s, pad, d) == out
    for path in sorted(glob.glob(os.path.join(GOLDEN, "hand_*.json"))):
        fx = json.load(open(path))
        p = OracleParams(**fx["params"])
        x, w = np.array(fx["x"], float), np.array(fx["w"], float)
        b = np.array(fx["b"], float) if p.bias_term else None
        np.testing.assert_array_equal(lib.forward(p, x, w, b), np.array(fx["y"], float))
        if "dy" in fx:
            dy = np.array(fx["dy"], float)
            np.testing.assert_array_equal(lib.backward_data(p, w, dy), np.array(fx["dx"], float))
            np.testing.assert_array_equal(lib.backward_data_at(p, w, dy, np.arange(x.size)),
                                          np.array(fx["dx"], float).ravel())
            np.testing.assert_array_equal(lib.backward_filter(p, x, dy), np.array(fx["dw"], float))
            np.testing.assert_array_equal(lib.backward_filter_at(p, x, dy, np.arange(w.size)),
                                          np.array(fx["dw"], float).ravel())
            if p.bias_term:
                np.testing.assert_array_equal(lib.backward_bias(p, dy), np.array(fx["db"], float))
    rng = np.random.default_rng(5)
    for p in SHAPES:
        OH = _size(p.h, p.kernel_h, p.stride_h, p.pad_h, p.dilation_h)
        OW = _size(p.w, p.kernel_w, p.stride_w, p.pad_w, p.dilation_w)
        assert lib.output_shape(p) == (p.n, p.num_output, OH, OW)
        x = rng.standard_normal(oracle.x_shape(p))
        w = rng.standard_normal(oracle.w_shape(p))
        b = rng.standard_normal(p.num_output)
        dy = rng.standard_normal((p.n, p.num_output, OH, OW))
        y, dx, dw, db = _brute(p, x, w, b, dy, OH, OW)
        np.testing.assert_allclose(lib.forward(p, x, w, b), y, atol=1e-12)
        np.testing.assert_allclose(lib.backward_data(p, w, dy), dx, atol=1e-12)
        np.testing.assert_allclose(lib.backward_data_at(p, w, dy, np.arange(dx.size)), dx.ravel(), atol=1e-12)
        np.testing.assert_allclose(lib.backward_filter(p, x, dy), dw, atol=1e-12)
        np.testing.assert_allclose(lib.backward_filter_at(p, x, dy, np.arange(dw.size)), dw.ravel(), atol=1e-12)
        np.testing.assert_allclose(lib.backward_bias(p, dy), db, atol=1e-12)
        g0 = rng.standard_normal(w.shape)
        np.testing.assert_allclose(lib.backward_filter(p, x, dy, dw=g0, beta=1.0), g0 + dw, atol=1e-12)
        b0 = rng.standard_normal(p.num_output)
        np.testing.assert_allclose(lib.backward_bias(p, dy, db=b0, beta=1.0), b0 + db, atol=1e-12)


def test_unmodified_source_passes(tmp_path):
    pin_suite(_build(open(SRC).read(), str(tmp_path), "clean"))


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(tmp_path, name, old, new):
    src = open(SRC).read()
    assert src.count(old) >= 1, f"mutation site of {name} not found in conv_oracle.c"
    lib = _build(src.replace(old, new), str(tmp_path), name)
    with pytest.raises((AssertionError, ValueError)):
        pin_suite(lib)
