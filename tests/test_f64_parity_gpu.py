"""GPU parity of the double-precision passes (conv_*_f64) against the CPU oracle.

Both sides compute in fp64 on the same inputs (fp32 draws widened to double, plus a small
double-only perturbation so that the low mantissa bits are exercised); only the order of the
sums differs.  Gate: normalised maximum error max|gpu - ref| / max|ref| <= 1e-12 per output tensor
(a sum of up to ~4e5 products of O(1) terms carries about sqrt(n) * 2^-53 ~ 1e-13 of rounding)."""
import numpy as np
import pytest
import torch

import oracle
import paper_1810_02272_amd as conv
from oracle import OracleParams
from paper_1810_02272_amd import workloads
from parity_metric import gated_error
from parity_cases import DIRECT_CASES, SWEEP, VARIANT_CASES, P

pytestmark = pytest.mark.gpu
TOL = 1e-12
DEV = "cuda:0"
NAN = float("nan")


def nerr(gpu, ref):
    g = gpu.detach().cpu().numpy().reshape(ref.shape)
    if ref.size == 0:
        return 0.0
    return float(np.max(np.abs(g - ref))) / max(float(np.max(np.abs(ref))), 1e-300)


def widen(t, seed):
    """fp32 draw -> double with the low mantissa bits filled (a relative perturbation of 1e-9)."""
    if t is None:
        return None
    d = t.double()
    return d * (1.0 + 1e-9 * workloads.draw(tuple(t.shape), "normal", seed).double())


def run_all64(pd, x, w, b, dy):
    p = conv.ConvParams(**pd)
    d = conv.conv_desc_create(p)
    ws = torch.full((max(conv.conv_desc_workspace_bytes_f64(d) // 8, 1),), NAN, device=DEV, dtype=torch.float64)
    xd, wd, dyd = x.to(DEV), w.to(DEV), dy.to(DEV)
    bd = b.to(DEV) if b is not None else None
    y = torch.full(tuple(dy.shape), NAN, device=DEV, dtype=torch.float64)
    dx = torch.full(tuple(x.shape), NAN, device=DEV, dtype=torch.float64)
    dw = torch.full(tuple(w.shape), NAN, device=DEV, dtype=torch.float64)
    conv.conv_forward_f64(d, xd, wd, bd, y, ws)
    ws.fill_(NAN)
    conv.conv_backward_data_f64(d, wd, dyd, dx, ws)
    ws.fill_(NAN)
    conv.conv_backward_filter_f64(d, xd, dyd, dw, 0.0, ws)
    db = None
    if b is not None:
        db = torch.full((p.num_output,), NAN, device=DEV, dtype=torch.float64)
        ws.fill_(NAN)
        conv.conv_backward_bias_f64(d, dyd, db, 0.0, ws)
    torch.cuda.synchronize()
    return d, ws, (xd, wd, bd, dyd), (y, dx, dw, db)


def check_full64(pd, x, w, b, dy):
    op = OracleParams(**pd)
    d, ws, _, (y, dx, dw, db) = run_all64(pd, x, w, b, dy)
    xn, wn, dyn = x.numpy(), w.numpy(), dy.numpy()
    bn = b.numpy() if b is not None else None
    refs = {"y": (y, oracle.forward(op, xn, wn, bn)), "dx": (dx, oracle.backward_data(op, wn, dyn)),
            "dw": (dw, oracle.backward_filter(op, xn, dyn))}
    if b is not None:
        refs["db"] = (db, oracle.backward_bias(op, dyn))
    errs = {k: gated_error(op, k, g, r, TOL, xn, wn, bn, dyn, case=("f64", pd)) for k, (g, r) in refs.items()}
    for k, v in errs.items():
        assert np.isfinite(v) and v <= TOL, (pd, k, v)
    return errs


F64_SWEEP = SWEEP + DIRECT_CASES + [c[0] for c in VARIANT_CASES]


@pytest.mark.parametrize("i", range(len(F64_SWEEP)))
def test_f64_sweep_full_compare(i):
    pd = F64_SWEEP[i]
    print("f64 case", i, pd, flush=True)
    op = OracleParams(**pd)
    x, w, b, dy = workloads.random_inputs(oracle.x_shape(op), oracle.w_shape(op), oracle.output_shape(op),
                                          7000 + 10 * i, bias=bool(pd["bias_term"]))
    check_full64(pd, widen(x, 1), widen(w, 2), widen(b, 3), widen(dy, 4))


@pytest.mark.parametrize("name", [l.name for l in workloads.LAYERS if l.config <= 3])
def test_f64_benchmark_layers_configs_0_to_3_full(name):
    l = workloads.BY_NAME[name]
    print("f64 layer", name, flush=True)
    x, w, b, dy = workloads.layer_inputs(l, bias="random")
    check_full64(l.params_dict(), widen(x, 11), widen(w, 12), widen(b, 13), widen(dy, 14))


@pytest.mark.parametrize("name", ["5.a", "5.b", "5.c"])
def test_f64_benchmark_layers_config_4_sampled(name):
    """Configuration 4 at full size in the launch configuration the benchmark times: sampled
    outputs the oracle computes one by one, the bias gradient in full, finiteness everywhere."""
    l = workloads.BY_NAME[name]
    print("f64 layer", name, flush=True)
    pd = l.params_dict()
    op = OracleParams(**pd)
    x, w, b, dy = (t.double() for t in workloads.layer_inputs(l, bias="random"))
    d, ws, _, (y, dx, dw, db) = run_all64(pd, x, w, b, dy)
    xn, wn, bn, dyn = x.numpy(), w.numpy(), b.numpy(), dy.numpy()
    rng = np.random.default_rng(321)

    def samples(total, count):
        return np.unique(np.concatenate([np.array([0, 1, total - 2, total - 1]), rng.integers(0, total, size=count)]))

    yi, xi, wi = samples(y.numel(), 6000), samples(dx.numel(), 6000), samples(dw.numel(), 300)
    ref_y = oracle.forward_at(op, xn, wn, bn, yi)
    ref_dx = oracle.backward_data_at(op, wn, dyn, xi)
    ref_dw = oracle.backward_filter_at(op, xn, dyn, wi)
    yc, dxc, dwc = y.cpu().numpy().ravel(), dx.cpu().numpy().ravel(), dw.cpu().numpy().ravel()
    assert np.max(np.abs(yc[yi] - ref_y)) / np.max(np.abs(ref_y)) <= TOL
    assert np.max(np.abs(dxc[xi] - ref_dx)) / np.max(np.abs(ref_dx)) <= TOL
    assert np.max(np.abs(dwc[wi] - ref_dw)) / np.max(np.abs(ref_dw)) <= TOL
    assert nerr(db, oracle.backward_bias(op, dyn)) <= TOL
    assert np.all(np.isfinite(yc)) and np.all(np.isfinite(dxc)) and np.all(np.isfinite(dwc))


def test_f64_beta_and_empty_batch():
    pd = P(3, 6, 11, 12, 10, 3, 3, 2, 1, 1, 1, 1, 1, 2)
    op = OracleParams(**pd)
    x, w, b, dy = (t.double() for t in workloads.random_inputs(oracle.x_shape(op), oracle.w_shape(op),
                                                               oracle.output_shape(op), 4242))
    d, ws, (xd, wd, bd, dyd), (y, dx, dw, db) = run_all64(pd, x, w, b, dy)
    dw0, db0 = dw.clone(), db.clone()
    conv.conv_backward_filter_f64(d, xd, dyd, dw, 1.0, ws)
    conv.conv_backward_bias_f64(d, dyd, db, 1.0, ws)
    torch.cuda.synchronize()
    assert torch.equal(dw, dw0 + dw0) and torch.equal(db, db0 + db0)
    assert nerr(dw, oracle.backward_filter(op, x.numpy(), dy.numpy(), dw=dw0.cpu().numpy(), beta=1.0)) <= TOL
    # empty batch: gradients become beta times themselves, nothing else is touched
    pe = P(0, 3, 8, 8, 4, 3, 3)
    de = conv.conv_desc_create(conv.ConvParams(**pe))
    wse = torch.zeros(max(conv.conv_desc_workspace_bytes_f64(de) // 8, 1), device=DEV, dtype=torch.float64)
    e_x = torch.zeros(0, 3, 8, 8, device=DEV, dtype=torch.float64)
    e_y = torch.zeros(0, 4, 6, 6, device=DEV, dtype=torch.float64)
    ew = torch.ones(4, 3, 3, 3, device=DEV, dtype=torch.float64)
    edw = torch.full((4, 3, 3, 3), 5.0, device=DEV, dtype=torch.float64)
    edb = torch.full((4,), 5.0, device=DEV, dtype=torch.float64)
    conv.conv_forward_f64(de, e_x, ew, edb, e_y, wse)
    conv.conv_backward_data_f64(de, ew, e_y, e_x, wse)
    conv.conv_backward_filter_f64(de, e_x, e_y, edw, 1.0, wse)
    conv.conv_backward_bias_f64(de, e_y, edb, 1.0, wse)
    torch.cuda.synchronize()
    assert torch.all(edw == 5.0) and torch.all(edb == 5.0)
    conv.conv_backward_filter_f64(de, e_x, e_y, edw, 0.0, wse)
    conv.conv_backward_bias_f64(de, e_y, edb, 0.0, wse)
    torch.cuda.synchronize()
    assert torch.all(edw == 0.0) and torch.all(edb == 0.0)


@pytest.mark.parametrize("group", [1, 2], ids=["gemm", "direct"])
def test_f64_blobs_between_2_and_4_gib(group):
    """Maximum sizes of the double path: blobs of 3.0e8 doubles (2.3 GiB; the limit is 2^29 elements),
    where byte offsets no longer fit 31 bits; on the MFMA kernels (one group) and on the direct kernels
    (two groups of two channels).  Sampled outputs, all of dw, the bias gradient in full."""
    pd = P(19, 4, 2000, 2000, 4, 3, 3, 1, 1, 1, 1, 1, 1, group)
    op = OracleParams(**pd)
    x, w, b, dy = (t.double() for t in workloads.random_inputs(oracle.x_shape(op), oracle.w_shape(op),
                                                               oracle.output_shape(op), 5160))
    assert x.numel() * 8 > (1 << 31)
    d, ws, _, (y, dx, dw, db) = run_all64(pd, x, w, b, dy)
    xn, wn, bn, dyn = x.numpy(), w.numpy(), b.numpy(), dy.numpy()
    rng = np.random.default_rng(8)

    def samples(total, count):
        edge = np.array([0, 1, total // 2 - 1, total // 2, total - 2, total - 1])
        return np.unique(np.concatenate([edge, rng.integers(0, total, size=count)]))

    yi, xi = samples(y.numel(), 4000), samples(dx.numel(), 4000)
    ref_y = oracle.forward_at(op, xn, wn, bn, yi)
    ref_dx = oracle.backward_data_at(op, wn, dyn, xi)
    ref_dw = oracle.backward_filter_at(op, xn, dyn, np.arange(dw.numel()))
    yc, dxc = y.cpu().numpy().ravel(), dx.cpu().numpy().ravel()
    assert np.max(np.abs(yc[yi] - ref_y)) / np.max(np.abs(ref_y)) <= TOL
    assert np.max(np.abs(dxc[xi] - ref_dx)) / np.max(np.abs(ref_dx)) <= TOL
    assert nerr(dw, ref_dw.reshape(tuple(w.shape))) <= TOL
    assert nerr(db, oracle.backward_bias(op, dyn)) <= TOL
    assert np.isfinite(yc).all() and np.isfinite(dxc).all()


@pytest.mark.parametrize("name", ["5.a", "5.b", "5.c"])
def test_f64_benchmark_layers_config_4_full(name):
    """Configuration 4 at full size in doubles, every output element of every pass against the oracle."""
    l = workloads.BY_NAME[name]
    print("f64 layer", name, "full compare", flush=True)
    x, w, b, dy = (t.double() for t in workloads.layer_inputs(l, bias="random"))
    check_full64(l.params_dict(), x, w, b, dy)
