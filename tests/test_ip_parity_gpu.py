"""GPU parity of the InnerProduct (+ReLU) entry points against the CPU oracle, same seeded inputs.

Gate: normalised maximum error max|gpu - ref| / max|ref| <= 1e-4 per output tensor (fp32 products,
fp32 accumulation against the exact double result).  The ReLU's mask is a yes/no decision taken
on a floating-point value, so both sides take it on the same fp32 number: ip_relu_backward is fed
the oracle's y rounded to fp32 and must then match the oracle bit for bit, and the gradient passes
take that dz.  The chained GPU result (mask from the GPU's own y) is checked too: it may differ
from the oracle's only where the pre-activation lies within the forward tolerance of zero.
"""
import numpy as np
import pytest
import torch

import paper_1810_02272_amd as conv
from oracle import inner_product as ipo
from oracle.inner_product import IpOracleParams
from paper_1810_02272_amd import workloads
from parity_cases import IP_BETA_SHAPES, IP_SHAPES
from parity_metric import small_tensor_error

pytestmark = pytest.mark.gpu
TOL = 1e-4
DEV = "cuda:0"
NAN = float("nan")


def nerr(gpu, ref):
    g = gpu.detach().cpu().double().numpy().reshape(ref.shape)
    if ref.size == 0:
        return 0.0
    return float(np.max(np.abs(g - ref))) / max(float(np.max(np.abs(ref))), 1e-30)


def run_case(m, k, o, bias, relu, x, w, b, dy, beta=0.0, dw0=None, db0=None):
    pd = dict(m=m, k=k, num_output=o, bias_term=int(bias), relu=int(relu))
    d = conv.ip_desc_create(conv.IpParams(**pd))
    op = IpOracleParams(**pd)
    ws = torch.full((max(conv.ip_desc_workspace_bytes(d) // 4, 1),), NAN, device=DEV)
    xd, wd, dyd = x.to(DEV), w.to(DEV), dy.to(DEV)
    bd = b.to(DEV) if bias else None
    y = torch.full((m, o), NAN, device=DEV)
    dz = torch.full((m, o), NAN, device=DEV)
    dx = torch.full((m, k), NAN, device=DEV)
    dw = torch.full((o, k), NAN, device=DEV) if dw0 is None else dw0.to(DEV)
    print(f"ip case m={m} k={k} o={o} bias={bias} relu={relu} beta={beta} {conv.ip_desc_kernel_names(d)}", flush=True)
    xn, wn, dyn = x.numpy(), w.numpy(), dy.numpy()
    bn = b.numpy() if bias else None
    yr = ipo.forward(op, xn, wn, bn)
    y32 = torch.from_numpy(yr.astype(np.float32))
    dzr = ipo.relu_backward(op, y32.numpy(), dyn)
    conv.ip_forward(d, xd, wd, bd, y, ws)
    dz_chain = torch.full((m, o), NAN, device=DEV)
    conv.ip_relu_backward(d, y if relu else None, dyd, dz_chain)
    conv.ip_relu_backward(d, y32.to(DEV) if relu else None, dyd, dz)
    ws.fill_(NAN)
    conv.ip_backward_data(d, wd, dz, dx, ws)
    ws.fill_(NAN)
    conv.ip_backward_filter(d, xd, dz, dw, beta, ws)
    db = None
    if bias:
        db = torch.full((o,), NAN, device=DEV) if db0 is None else db0.to(DEV)
        ws.fill_(NAN)
        conv.ip_backward_bias(d, dz, db, beta, ws)
    torch.cuda.synchronize()

    assert np.array_equal(dz.cpu().numpy().astype(np.float64), dzr), "ReLU mask differs on identical fp32 y"
    if m * o:
        zr = ipo.forward(IpOracleParams(m, k, o, int(bias), 0), xn, wn, bn)
        differs = dz_chain.cpu().numpy().astype(np.float64) != dzr
        assert not (differs & (np.abs(zr) > TOL * np.max(np.abs(zr)))).any(), "chained mask differs away from the kink"
    pairs = {"y": (y, yr), "dx": (dx, ipo.backward_data(op, wn, dzr)),
             "dw": (dw, ipo.backward_filter(op, xn, dzr, None if dw0 is None else dw0.numpy(), beta))}
    if bias:
        pairs["db"] = (db, ipo.backward_bias(op, dzr, None if db0 is None else db0.numpy(), beta))

    def term_scale(which):
        """Largest root-sum-square of the terms of an output (the contraction of the squared operands):
        the denominator for a tensor of a few elements that cancelled to far below its terms."""
        sq = lambda a: None if a is None else np.square(np.asarray(a, dtype=np.float64))
        lin = IpOracleParams(m, k, o, int(bias), 0)
        r = {"y": lambda: ipo.forward(lin, sq(xn), sq(wn), sq(bn)),
             "dx": lambda: ipo.backward_data(op, sq(wn), sq(dzr)),
             "dw": lambda: ipo.backward_filter(op, sq(xn), sq(dzr), None if dw0 is None else sq(dw0.numpy()), beta),
             "db": lambda: ipo.backward_bias(op, sq(dzr), None if db0 is None else sq(db0.numpy()), beta)}[which]()
        return float(np.sqrt(np.max(r))) if r.size else 0.0

    errs = {}
    for name, (got, ref) in pairs.items():
        v = small_tensor_error(nerr(got, ref), ref, TOL, lambda: term_scale(name), ("ip", pd, beta), name)
        errs[name] = v
        assert np.isfinite(v) and v <= TOL, (pd, name, v, conv.ip_desc_kernel_names(d))
    if relu and m * o:
        assert float(y.min()) >= 0.0
    return errs


SHAPES = IP_SHAPES


@pytest.mark.parametrize("shape", SHAPES, ids=[f"{m}x{k}x{o}" for m, k, o in SHAPES])
@pytest.mark.parametrize("relu", [0, 1])
def test_ip_sweep(shape, relu):
    m, k, o = shape
    x, w, b, dy = workloads.ip_random_inputs(m, k, o, seed=7000 + 13 * m + k + o)
    run_case(m, k, o, True, relu, x, w, b, dy)


def test_ip_without_bias():
    x, w, _, dy = workloads.ip_random_inputs(33, 300, 70, seed=7100, bias=False)
    run_case(33, 300, 70, False, 1, x, w, None, dy)


@pytest.mark.parametrize("shape", IP_BETA_SHAPES, ids=[f"{m}x{k}x{o}" for m, k, o in IP_BETA_SHAPES])
def test_ip_beta_one_accumulates(shape):
    m, k, o = shape
    x, w, b, dy = workloads.ip_random_inputs(m, k, o, seed=7200 + m)
    dw0 = workloads.draw((o, k), "normal", 7300 + m)
    db0 = workloads.draw((o,), "normal", 7301 + m)
    run_case(m, k, o, True, 1, x, w, b, dy, beta=1.0, dw0=dw0, db0=db0)


@pytest.mark.parametrize("name", [l.name for l in workloads.IP_LAYERS])
def test_ip_benchmark_layers_full_size(name):
    """The benchmark's layers at full size, in the launch configuration bench.py times."""
    l = workloads.IP_BY_NAME[name]
    x, w, b, dy = workloads.ip_inputs(l, bias="random")
    run_case(l.m, l.k, l.num_output, True, l.relu, x, w, b, dy)


def test_ip_relu_backward_in_place_and_copy():
    m, o = 50, 77
    d1 = conv.ip_desc_create(conv.IpParams(m, 8, o, 1, 1))
    d0 = conv.ip_desc_create(conv.IpParams(m, 8, o, 1, 0))
    y = workloads.draw((m, o), "normal", 7400).clamp_min(0.0)
    dy = workloads.draw((m, o), "normal", 7401)
    ref = torch.where(y > 0, dy, torch.zeros_like(dy))
    g = dy.to(DEV).clone()
    conv.ip_relu_backward(d1, y.to(DEV), g, g)           # in place
    assert torch.equal(g.cpu(), ref)
    out = torch.full((m, o), NAN, device=DEV)
    conv.ip_relu_backward(d0, None, dy.to(DEV), out)      # no ReLU: plain copy
    assert torch.equal(out.cpu(), dy)


def test_ip_empty_batch():
    d = conv.ip_desc_create(conv.IpParams(0, 6, 4, 1, 1))
    ws = torch.zeros(max(conv.ip_desc_workspace_bytes(d) // 4, 1), device=DEV)
    e = torch.empty((0, 6), device=DEV)
    eo = torch.empty((0, 4), device=DEV)
    w = torch.ones((4, 6), device=DEV)
    b = torch.ones(4, device=DEV)
    conv.ip_forward(d, e, w, b, eo, ws)
    conv.ip_relu_backward(d, eo, eo, eo)
    conv.ip_backward_data(d, w, eo, e, ws)
    dw = torch.full((4, 6), 2.0, device=DEV)
    db = torch.full((4,), 3.0, device=DEV)
    conv.ip_backward_filter(d, e, eo, dw, 1.0, ws)
    conv.ip_backward_bias(d, eo, db, 1.0, ws)
    assert torch.equal(dw.cpu(), torch.full((4, 6), 2.0)) and torch.equal(db.cpu(), torch.full((4,), 3.0))
    dw.fill_(NAN)
    db.fill_(NAN)
    conv.ip_backward_filter(d, e, eo, dw, 0.0, ws)
    conv.ip_backward_bias(d, eo, db, 0.0, ws)
    assert torch.equal(dw.cpu(), torch.zeros(4, 6)) and torch.equal(db.cpu(), torch.zeros(4))


def test_ip_repeat_runs_are_bit_identical():
    l = workloads.IP_BY_NAME["ip1.1"]
    x, w, b, dy = workloads.ip_inputs(l, bias="random")
    d = conv.ip_desc_create(conv.IpParams(**l.params_dict()))
    ws = torch.zeros(max(conv.ip_desc_workspace_bytes(d) // 4, 1), device=DEV)
    xd, wd, bd, dyd = x.to(DEV), w.to(DEV), b.to(DEV), dy.to(DEV)
    outs = []
    for _ in range(2):
        y, dx, dw = torch.empty((l.m, l.num_output), device=DEV), torch.empty_like(xd), torch.empty_like(wd)
        conv.ip_forward(d, xd, wd, bd, y, ws)
        conv.ip_backward_data(d, wd, dyd, dx, ws)
        conv.ip_backward_filter(d, xd, dyd, dw, 0.0, ws)
        torch.cuda.synchronize()
        outs.append((y.cpu(), dx.cpu(), dw.cpu()))
    for a, b_ in zip(*outs):
        assert torch.equal(a, b_)


def test_ip_forward_output_above_1_gib():
    """Maximum sizes: an output blob of more than 2^30 bytes (16400 x 16400 floats), where the store of
    the contraction kernel no longer fits range-checked 32-bit offsets and takes plain pointers."""
    m, k, o = 16400, 2, 16400
    pd = dict(m=m, k=k, num_output=o, bias_term=1, relu=0)
    d = conv.ip_desc_create(conv.IpParams(**pd))
    names = conv.ip_desc_kernel_names(d)
    print("large InnerProduct output:", names, flush=True)
    assert ",ep]" in names.split(";")[0]
    x, w, b, _ = workloads.ip_random_inputs(m, k, o, seed=7500)
    ws = torch.full((max(conv.ip_desc_workspace_bytes(d) // 4, 1),), NAN, device=DEV)
    y = torch.full((m, o), NAN, device=DEV)
    conv.ip_forward(d, x.to(DEV), w.to(DEV), b.to(DEV), y, ws)
    torch.cuda.synchronize()
    ref = ipo.forward(IpOracleParams(**pd), x.numpy(), w.numpy(), b.numpy())
    got = y.cpu().numpy()
    del y, ws
    worst, top = 0.0, float(np.max(np.abs(ref)))
    for r0 in range(0, m, 1024):   # by row blocks: no second full-size double array on the host
        worst = max(worst, float(np.max(np.abs(got[r0:r0 + 1024].astype(np.float64) - ref[r0:r0 + 1024]))))
    assert np.isfinite(got).all() and worst / top <= TOL
