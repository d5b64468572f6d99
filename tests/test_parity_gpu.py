"""GPU parity: the HIP path behind the C boundary against the CPU oracle, same seeded inputs.

Tolerance.  The kernels multiply in fp32 and accumulate in fp32 (MFMA); the oracle is the exact
double-precision result for the same fp32 inputs.  The gate is the normalised maximum error
max|gpu - ref| / max|ref| <= 1e-4 per output tensor (the bar the benchmark definition states); a
tensor that cancels to far below the scale of its terms is measured against that scale
(parity_metric.py).
"""
import numpy as np
import pytest
import torch

import oracle
import paper_1810_02272_amd as conv
from oracle import OracleParams
from paper_1810_02272_amd import workloads
from parity_cases import DIRECT_CASES, PATCH_CASES, SWEEP, VARIANT_CASES, P
from parity_metric import gated_error, nerr

pytestmark = pytest.mark.gpu
TOL = 1e-4
DEV = "cuda:0"


def run_all(pd: dict, x, w, b, dy, beta_check=True, poison=True):
    """Run the four passes on the GPU; returns (y, dx, dw, db) device tensors."""
    p = conv.ConvParams(**pd)
    d = conv.conv_desc_create(p)
    ws_bytes = conv.conv_desc_workspace_bytes(d)
    fill = float("nan") if poison else 0.0
    ws = torch.full((max(ws_bytes // 4, 1),), fill, device=DEV)
    xd, wd, dyd = x.to(DEV), w.to(DEV), dy.to(DEV)
    bd = b.to(DEV) if b is not None else None
    y = torch.full(tuple(dy.shape), fill, device=DEV)
    dx = torch.full(tuple(x.shape), fill, device=DEV)
    dw = torch.full(tuple(w.shape), fill, device=DEV)
    conv.conv_forward(d, xd, wd, bd, y, ws)
    ws.fill_(fill)
    conv.conv_backward_data(d, wd, dyd, dx, ws)
    ws.fill_(fill)
    conv.conv_backward_filter(d, xd, dyd, dw, 0.0, ws)
    db = None
    if b is not None:
        db = torch.full((p.num_output,), fill, device=DEV)
        ws.fill_(fill)
        conv.conv_backward_bias(d, dyd, db, 0.0, ws)
    torch.cuda.synchronize()
    return d, ws, (xd, wd, bd, dyd), (y, dx, dw, db)


def check_full(pd: dict, seed: int, bias=True):
    op = OracleParams(**pd)
    xs, wsh, ys = oracle.x_shape(op), oracle.w_shape(op), oracle.output_shape(op)
    x, w, b, dy = workloads.random_inputs(xs, wsh, ys, seed, bias=bias)
    d, ws, dev_in, (y, dx, dw, db) = run_all(pd, x, w, b, dy)
    assert conv.conv_desc_output_shape(d) == ys
    xn, wn, dyn = x.numpy(), w.numpy(), dy.numpy()
    bn = b.numpy() if b is not None else None
    refs = {"y": (y, oracle.forward(op, xn, wn, bn)), "dx": (dx, oracle.backward_data(op, wn, dyn)),
            "dw": (dw, oracle.backward_filter(op, xn, dyn))}
    if b is not None:
        refs["db"] = (db, oracle.backward_bias(op, dyn))
    errs = {k: gated_error(op, k, g, r, TOL, xn, wn, bn, dyn, case=pd) for k, (g, r) in refs.items()}
    for k, v in errs.items():
        assert np.isfinite(v) and v <= TOL, (pd, k, v, conv.conv_desc_kernel_names(d))
    if b is not None:
        check_filter_and_bias_in_one_pass(pd, op, d, ws, dev_in, dw, refs["db"][1], (xn, wn, bn, dyn))
    return errs


def check_filter_and_bias_in_one_pass(pd, op, d, ws, dev_in, dw, db_ref, host, beta=0.0, dw0=None, db0=None):
    """conv_backward_filter_bias: dw bit-identical to conv_backward_filter's, db against the oracle."""
    xd, _, _, dyd = dev_in
    dw2 = torch.full_like(dw, float("nan")) if dw0 is None else dw0.clone()
    db2 = torch.full((pd["num_output"],), float("nan"), device=DEV) if db0 is None else db0.clone()
    ws.fill_(float("nan"))
    conv.conv_backward_filter_bias(d, xd, dyd, dw2, db2, beta, ws)
    torch.cuda.synchronize()
    assert torch.equal(dw2, dw), (pd, conv.conv_desc_kernel_names(d))
    v = gated_error(op, "db", db2, db_ref, TOL, *host, case=("filter+bias", pd))
    assert np.isfinite(v) and v <= TOL, (pd, "db from the filter-gradient pass", v, conv.conv_desc_kernel_names(d))
    return db2


@pytest.mark.parametrize("i", range(len(SWEEP)))
def test_sweep_full_compare(i):
    pd = SWEEP[i]
    print("case", i, pd, flush=True)
    check_full(pd, seed=7000 + 10 * i, bias=bool(pd["bias_term"]))


@pytest.mark.parametrize("i", range(len(DIRECT_CASES)))
def test_thin_groups_direct_kernels(i):
    pd = DIRECT_CASES[i]
    d = conv.conv_desc_create(conv.ConvParams(**pd))
    assert "direct" in conv.conv_desc_kernel_names(d), conv.conv_desc_kernel_names(d)
    check_full(pd, 4400 + i, bias=bool(pd["bias_term"]))


def test_thin_groups_blobs_not_16_byte_aligned():
    """The four-columns-per-thread kernels need 16-byte aligned blobs; blobs that start 4 bytes off
    such a boundary take the one-column kernels (the C boundary only asks for the base type's alignment)."""
    pd = P(3, 8, 14, 16, 8, 3, 3, 1, 1, 1, 1, 1, 1, 8)
    op = OracleParams(**pd)
    x, w, b, dy = workloads.random_inputs(oracle.x_shape(op), oracle.w_shape(op), oracle.output_shape(op), 4711)
    d = conv.conv_desc_create(conv.ConvParams(**pd))
    assert "direct" in conv.conv_desc_kernel_names(d)
    ws = torch.zeros(max(conv.conv_desc_workspace_bytes(d) // 4, 1), device=DEV)

    def off_by_one(t):
        buf = torch.full((t.numel() + 1,), float("nan"), device=DEV)
        v = buf[1:].view(t.shape)
        v.copy_(t)
        assert v.data_ptr() % 16 == 4 and v.is_contiguous()
        return v

    xd, dyd, wd, bd = off_by_one(x), off_by_one(dy), w.to(DEV), b.to(DEV)
    y, dx, dw = off_by_one(torch.zeros_like(dy)), off_by_one(torch.zeros_like(x)), torch.zeros_like(wd)
    conv.conv_forward(d, xd, wd, bd, y, ws)
    conv.conv_backward_data(d, wd, dyd, dx, ws)
    conv.conv_backward_filter(d, xd, dyd, dw, 0.0, ws)
    db = torch.zeros_like(bd)
    conv.conv_backward_bias(d, dyd, db, 0.0, ws)  # planes of a multiple of four elements, 4 bytes off a boundary
    torch.cuda.synchronize()
    assert nerr(y, oracle.forward(op, x.numpy(), w.numpy(), b.numpy())) <= TOL
    assert nerr(dx, oracle.backward_data(op, w.numpy(), dy.numpy())) <= TOL
    assert nerr(dw, oracle.backward_filter(op, x.numpy(), dy.numpy())) <= TOL
    assert nerr(db, oracle.backward_bias(op, dy.numpy())) <= TOL


def selected(pd):
    d = conv.conv_desc_create(conv.ConvParams(**pd))
    return dict(kv.split("=", 1) for kv in conv.conv_desc_kernel_names(d).split(";"))


@pytest.mark.parametrize("i", range(len(PATCH_CASES)))
def test_patch_kernel_full_compare(i):
    pd, which, variant = PATCH_CASES[i]
    print("patch case", i, pd, flush=True)
    assert selected(pd)[which].startswith(variant), selected(pd)
    check_full(pd, seed=9000 + 10 * i)


@pytest.mark.parametrize("i", range(len(VARIANT_CASES)))
def test_every_tile_and_bounds_mode_full_compare(i):
    """One shape per (pass, tile, bounds mode) that the other lists do not select (the CPU test
    test_variant_coverage.py checks that together they select every variant)."""
    pd, which, variant = VARIANT_CASES[i]
    print("variant case", i, which, variant, pd, flush=True)
    assert selected(pd)[which].startswith(variant), selected(pd)
    check_full(pd, seed=9500 + 10 * i)


@pytest.mark.parametrize("name", [l.name for l in workloads.LAYERS if l.config <= 3])
def test_benchmark_layers_configs_0_to_3_full(name):
    """Configurations 0-3 at full size, every output element against the oracle."""
    l = workloads.BY_NAME[name]
    print("layer", name, flush=True)
    pd = l.params_dict()
    op = OracleParams(**pd)
    x, w, b, dy = workloads.layer_inputs(l, bias="random")
    d, ws, _, (y, dx, dw, db) = run_all(pd, x, w, b, dy)
    xn, wn, bn, dyn = x.numpy(), w.numpy(), b.numpy(), dy.numpy()
    assert nerr(y, oracle.forward(op, xn, wn, bn)) <= TOL
    assert nerr(dx, oracle.backward_data(op, wn, dyn)) <= TOL
    assert nerr(dw, oracle.backward_filter(op, xn, dyn)) <= TOL
    assert nerr(db, oracle.backward_bias(op, dyn)) <= TOL


@pytest.mark.parametrize("name", [l.name for l in workloads.DW_LAYERS])
def test_depthwise_layers_full(name):
    """The depthwise layers `bench.py --workload dw` times, at full size, element by element."""
    l = workloads.BY_NAME[name]
    pd = l.params_dict()
    assert "direct" in conv.conv_desc_kernel_names(conv.conv_desc_create(conv.ConvParams(**pd)))
    op = OracleParams(**pd)
    x, w, b, dy = workloads.layer_inputs(l, bias="random")
    d, ws, _, (y, dx, dw, db) = run_all(pd, x, w, b, dy)
    xn, wn, bn, dyn = x.numpy(), w.numpy(), b.numpy(), dy.numpy()
    assert nerr(y, oracle.forward(op, xn, wn, bn)) <= TOL
    assert nerr(dx, oracle.backward_data(op, wn, dyn)) <= TOL
    assert nerr(dw, oracle.backward_filter(op, xn, dyn)) <= TOL
    assert nerr(db, oracle.backward_bias(op, dyn)) <= TOL


@pytest.mark.parametrize("name", ["5.a", "5.b", "5.c"])
def test_benchmark_layers_config_4_sampled(name):
    """The large grouped-conv configuration at full size, in the launch configuration the benchmark
    times: outputs the oracle computes one by one (random samples plus corners), the bias gradient
    in full, and exact invariants that hold at any size."""
    l = workloads.BY_NAME[name]
    print("layer", name, flush=True)
    pd = l.params_dict()
    op = OracleParams(**pd)
    x, w, b, dy = workloads.layer_inputs(l, bias="random")
    d, ws, (xd, wd, bd, dyd), (y, dx, dw, db) = run_all(pd, x, w, b, dy)
    xn, wn, bn, dyn = x.numpy(), w.numpy(), b.numpy(), dy.numpy()
    rng = np.random.default_rng(123)

    def samples(total, count):
        edge = np.array([0, 1, total - 2, total - 1])
        return np.unique(np.concatenate([edge, rng.integers(0, total, size=count)]))

    yi, xi, wi = samples(y.numel(), 6000), samples(dx.numel(), 6000), samples(dw.numel(), 300)
    ref_y = oracle.forward_at(op, xn, wn, bn, yi)
    ref_dx = oracle.backward_data_at(op, wn, dyn, xi)
    ref_dw = oracle.backward_filter_at(op, xn, dyn, wi)
    ref_db = oracle.backward_bias(op, dyn)
    yc, dxc, dwc = y.cpu().double().numpy().ravel(), dx.cpu().double().numpy().ravel(), dw.cpu().double().numpy().ravel()
    # normalise by the largest magnitude of the whole GPU tensor's sampled reference
    assert np.max(np.abs(yc[yi] - ref_y)) / np.max(np.abs(ref_y)) <= TOL
    assert np.max(np.abs(dxc[xi] - ref_dx)) / np.max(np.abs(ref_dx)) <= TOL
    assert np.max(np.abs(dwc[wi] - ref_dw)) / np.max(np.abs(ref_dw)) <= TOL
    assert nerr(db, ref_db) <= TOL
    assert np.all(np.isfinite(yc)) and np.all(np.isfinite(dxc)) and np.all(np.isfinite(dwc))
    # invariants over the whole tensors: <y - b, dy> = <x, dx> = <w, dw> (double sums of fp32 results)
    lin = float(np.sum((yc.reshape(y.shape) - bn[None, :, None, None]) * dyn.astype(np.float64)))
    via_dx = float(np.sum(dxc * xn.astype(np.float64).ravel()))
    via_dw = float(np.sum(dwc * wn.astype(np.float64).ravel()))
    scale = float(np.sqrt(y.numel())) * float(np.max(np.abs(ref_y))) * l.dy_std
    assert abs(lin - via_dx) <= 1e-3 * scale and abs(lin - via_dw) <= 1e-3 * scale, (lin, via_dx, via_dw, scale)
    # both parameter gradients from one read of dy, at full size
    check_filter_and_bias_in_one_pass(pd, op, d, ws, (xd, wd, bd, dyd), dw, ref_db, (xn, wn, bn, dyn))
    # beta = 1 at full size (the wide form of the split reduction): dw + dw and db + db are exact in fp32
    dw0, db0 = dw.clone(), db.clone()
    conv.conv_backward_filter(d, xd, dyd, dw, 1.0, ws)
    conv.conv_backward_bias(d, dyd, db, 1.0, ws)
    torch.cuda.synchronize()
    assert torch.equal(dw, dw0 + dw0) and torch.equal(db, db0 + db0)


@pytest.mark.parametrize("pd", [P(3, 6, 11, 12, 10, 3, 3, 2, 1, 1, 1, 1, 1, 2),
                                P(3, 6, 11, 12, 6, 3, 3, 2, 1, 1, 1, 1, 1, 6)], ids=["gemm", "direct"])
def test_beta_accumulates_and_overwrites(pd):
    op = OracleParams(**pd)
    x, w, b, dy = workloads.random_inputs(oracle.x_shape(op), oracle.w_shape(op), oracle.output_shape(op), 4242)
    d, ws, (xd, wd, bd, dyd), (y, dx, dw, db) = run_all(pd, x, w, b, dy)
    dw0, db0 = dw.clone(), db.clone()
    conv.conv_backward_filter(d, xd, dyd, dw, 1.0, ws)
    conv.conv_backward_bias(d, dyd, db, 1.0, ws)
    torch.cuda.synchronize()
    assert torch.equal(dw, dw0 + dw0) and torch.equal(db, db0 + db0)   # x + x is exact in fp32
    ref = oracle.backward_filter(op, x.numpy(), dy.numpy(), dw=dw0.cpu().numpy(), beta=1.0)
    assert nerr(dw, ref) <= TOL
    # both gradients in one pass: beta = 0 overwrites NaNs, beta = 1 adds to what is there
    host = (x.numpy(), w.numpy(), b.numpy(), dy.numpy())
    db1 = check_filter_and_bias_in_one_pass(pd, op, d, ws, (xd, wd, bd, dyd), dw0, oracle.backward_bias(op, dy.numpy()),
                                            host)
    db_ref2 = oracle.backward_bias(op, dy.numpy(), db=db1.cpu().numpy(), beta=1.0)
    db2 = check_filter_and_bias_in_one_pass(pd, op, d, ws, (xd, wd, bd, dyd), dw, db_ref2, host, beta=1.0, dw0=dw0,
                                            db0=db1)
    assert torch.equal(db2, db1 + db1)


def test_runs_are_bitwise_repeatable():
    pd = P(4, 8, 19, 19, 24, 5, 5, 2, 2, 2, 2, 1, 1, 2)
    op = OracleParams(**pd)
    x, w, b, dy = workloads.random_inputs(oracle.x_shape(op), oracle.w_shape(op), oracle.output_shape(op), 99)
    _, _, _, first = run_all(pd, x, w, b, dy)
    _, _, _, second = run_all(pd, x, w, b, dy, poison=False)
    for a, c in zip(first, second):
        assert torch.equal(a, c)


def test_filter_and_bias_in_one_pass_on_configs_0_to_3_and_depthwise():
    for l in [l for l in workloads.LAYERS if l.config <= 3] + [workloads.BY_NAME["dw.e"]]:
        pd = l.params_dict()
        op = OracleParams(**pd)
        x, w, b, dy = workloads.layer_inputs(l, bias="random")
        d, ws, dev_in, (y, dx, dw, db) = run_all(pd, x, w, b, dy)
        check_filter_and_bias_in_one_pass(pd, op, d, ws, dev_in, dw, oracle.backward_bias(op, dy.numpy()),
                                          (x.numpy(), w.numpy(), b.numpy(), dy.numpy()))


def test_empty_batch_is_a_noop():
    pd = P(0, 3, 8, 8, 4, 3, 3)
    p = conv.ConvParams(**pd)
    d = conv.conv_desc_create(p)
    ws = torch.zeros(max(conv.conv_desc_workspace_bytes(d) // 4, 1), device=DEV)
    x = torch.zeros(0, 3, 8, 8, device=DEV)
    w = torch.ones(4, 3, 3, 3, device=DEV)
    b = torch.ones(4, device=DEV)
    y = torch.zeros(0, 4, 6, 6, device=DEV)
    dw = torch.full((4, 3, 3, 3), 5.0, device=DEV)
    db = torch.full((4,), 5.0, device=DEV)
    conv.conv_forward(d, x, w, b, y, ws)
    conv.conv_backward_data(d, w, y, x, ws)
    conv.conv_backward_filter(d, x, y, dw, 1.0, ws)
    conv.conv_backward_bias(d, y, db, 1.0, ws)
    torch.cuda.synchronize()
    assert torch.all(dw == 5.0) and torch.all(db == 5.0)
    conv.conv_backward_filter(d, x, y, dw, 0.0, ws)
    conv.conv_backward_bias(d, y, db, 0.0, ws)
    torch.cuda.synchronize()
    assert torch.all(dw == 0.0) and torch.all(db == 0.0)
    dw.fill_(5.0)
    db.fill_(7.0)
    conv.conv_backward_filter_bias(d, x, y, dw, db, 1.0, ws)
    torch.cuda.synchronize()
    assert torch.all(dw == 5.0) and torch.all(db == 7.0)
    conv.conv_backward_filter_bias(d, x, y, dw, db, 0.0, ws)
    torch.cuda.synchronize()
    assert torch.all(dw == 0.0) and torch.all(db == 0.0)


def test_runs_on_a_side_stream():
    pd = P(2, 4, 10, 10, 6, 3, 3, 1, 1, 1, 1)
    op = OracleParams(**pd)
    x, w, b, dy = workloads.random_inputs(oracle.x_shape(op), oracle.w_shape(op), oracle.output_shape(op), 5)
    p = conv.ConvParams(**pd)
    d = conv.conv_desc_create(p)
    ws = torch.zeros(max(conv.conv_desc_workspace_bytes(d) // 4, 1), device=DEV)
    xd, wd, bd = x.to(DEV), w.to(DEV), b.to(DEV)
    y = torch.zeros(tuple(dy.shape), device=DEV)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        conv.conv_forward(d, xd, wd, bd, y, ws)
    s.synchronize()
    assert nerr(y, oracle.forward(op, x.numpy(), w.numpy(), b.numpy())) <= TOL


@pytest.mark.parametrize("n,group", [(37, 1), (37, 2), (19, 1)], ids=["gemm", "direct", "gemm-1.1GiB"])
def test_blobs_between_1_and_4_gib(n, group):
    """Maximum sizes: x, y, dx and dy of 2.2 GiB each (5.9e8 elements; the limit is 2^30), where byte
    offsets no longer fit 31 bits and the GEMM kernels fall back to compare-based bounds checks and
    64-bit store addresses (one group), the same sizes on the direct kernels (two groups of two
    channels), and blobs of 1.1 GiB, which take the range-checked stores with one select per element.
    Sampled outputs the oracle computes one by one, all of dw, the bias gradient in full, finiteness
    everywhere."""
    pd = P(n, 4, 2000, 2000, 4, 3, 3, 1, 1, 1, 1, 1, 1, group)
    op = OracleParams(**pd)
    x, w, b, dy = workloads.random_inputs(oracle.x_shape(op), oracle.w_shape(op), oracle.output_shape(op), 5150)
    assert x.numel() * 4 > (1 << 30) and dy.numel() * 4 > (1 << 30)
    assert (x.numel() * 4 > (1 << 31)) == (n == 37)
    d, ws, _, (y, dx, dw, db) = run_all(pd, x, w, b, dy)
    print("large blobs:", conv.conv_desc_kernel_names(d), flush=True)
    assert ("direct" in conv.conv_desc_kernel_names(d)) == (group == 2)
    xn, wn, bn, dyn = x.numpy(), w.numpy(), b.numpy(), dy.numpy()
    rng = np.random.default_rng(7)

    def samples(total, count):
        edge = np.array([0, 1, total // 2 - 1, total // 2, total - 2, total - 1])
        return np.unique(np.concatenate([edge, rng.integers(0, total, size=count)]))

    yi, xi = samples(y.numel(), 4000), samples(dx.numel(), 4000)
    wi = np.arange(dw.numel())
    ref_y = oracle.forward_at(op, xn, wn, bn, yi)
    ref_dx = oracle.backward_data_at(op, wn, dyn, xi)
    ref_dw = oracle.backward_filter_at(op, xn, dyn, wi)
    yc, dxc = y.cpu().numpy().ravel(), dx.cpu().numpy().ravel()
    assert np.max(np.abs(yc[yi].astype(np.float64) - ref_y)) / np.max(np.abs(ref_y)) <= TOL
    assert np.max(np.abs(dxc[xi].astype(np.float64) - ref_dx)) / np.max(np.abs(ref_dx)) <= TOL
    assert nerr(dw, ref_dw.reshape(tuple(w.shape))) <= TOL
    assert nerr(db, oracle.backward_bias(op, dyn)) <= TOL
    assert np.isfinite(yc).all() and np.isfinite(dxc).all()


def test_one_descriptor_two_threads_two_streams():
    """A descriptor is immutable and may be shared between threads; passes on different streams need
    their own workspace."""
    import threading

    pd = P(6, 8, 21, 19, 12, 3, 3, 1, 1, 1, 1, 1, 1, 2)
    op = OracleParams(**pd)
    d = conv.conv_desc_create(conv.ConvParams(**pd))
    ws_elems = max(conv.conv_desc_workspace_bytes(d) // 4, 1)
    results, errors = {}, []

    def worker(idx):
        try:
            torch.cuda.set_device(0)
            x, w, b, dy = workloads.random_inputs(oracle.x_shape(op), oracle.w_shape(op), oracle.output_shape(op),
                                                  6000 + idx)
            s = torch.cuda.Stream()
            with torch.cuda.stream(s):
                ws = torch.zeros(ws_elems, device=DEV)
                xd, wd, bd, dyd = x.to(DEV), w.to(DEV), b.to(DEV), dy.to(DEV)
                y, dx, dw = torch.empty_like(dyd), torch.empty_like(xd), torch.empty_like(wd)
                for _ in range(20):
                    conv.conv_forward(d, xd, wd, bd, y, ws, s)
                    conv.conv_backward_data(d, wd, dyd, dx, ws, s)
                    conv.conv_backward_filter(d, xd, dyd, dw, 0.0, ws, s)
            s.synchronize()
            results[idx] = (nerr(y, oracle.forward(op, x.numpy(), w.numpy(), b.numpy())),
                            nerr(dx, oracle.backward_data(op, w.numpy(), dy.numpy())),
                            nerr(dw, oracle.backward_filter(op, x.numpy(), dy.numpy())))
        except Exception as e:  # surfaced by the assertion below
            errors.append(repr(e))

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    assert len(results) == 2 and all(v <= TOL for r in results.values() for v in r), results


def test_gradients_on_a_second_stream_overlapping_backward_data():
    """The schedule of a training loop (and of bench.py --overlap): forward passes, then backward data on
    the launch stream while the filter and bias gradients of the same layer run on a second stream with
    a workspace of their own.  Every result against the oracle, and bit-identical to the serial run."""
    layers = [l for l in workloads.LAYERS if l.config == 3]
    main, side = torch.cuda.current_stream(), torch.cuda.Stream()
    state, ws_elems = [], 1
    for l in layers:
        pd = l.params_dict()
        x, w, b, dy = workloads.layer_inputs(l)
        d = conv.conv_desc_create(conv.ConvParams(**pd))
        ws_elems = max(ws_elems, conv.conv_desc_workspace_bytes(d) // 4)
        state.append(dict(op=OracleParams(**pd), d=d, host=(x, w, b, dy), x=x.to(DEV), w=w.to(DEV), b=b.to(DEV),
                          dy=dy.to(DEV)))
    ws = [torch.full((ws_elems,), float("nan"), device=DEV) for _ in range(2)]

    def outputs(t):
        t["out"] = [torch.full(tuple(v.shape), float("nan"), device=DEV)
                    for v in (t["dy"], t["x"], t["w"], t["b"])]
        return t["out"]

    for t in state:  # serial
        y, dx, dw, db = outputs(t)
        conv.conv_forward(t["d"], t["x"], t["w"], t["b"], y, ws[0])
        conv.conv_backward_data(t["d"], t["w"], t["dy"], dx, ws[0])
        conv.conv_backward_filter(t["d"], t["x"], t["dy"], dw, 0.0, ws[0])
        conv.conv_backward_bias(t["d"], t["dy"], db, 0.0, ws[0])
    torch.cuda.synchronize()
    serial = [[v.clone() for v in t["out"]] for t in state]

    for _ in range(3):
        for t in state:
            y = outputs(t)[0]
            conv.conv_forward(t["d"], t["x"], t["w"], t["b"], y, ws[0], main)
        fork = torch.cuda.Event()
        fork.record(main)
        side.wait_event(fork)
        for t in reversed(state):
            _, dx, dw, db = t["out"]
            conv.conv_backward_data(t["d"], t["w"], t["dy"], dx, ws[0], main)
            conv.conv_backward_filter(t["d"], t["x"], t["dy"], dw, 0.0, ws[1], side)
            conv.conv_backward_bias(t["d"], t["dy"], db, 0.0, ws[1], side)
        join = torch.cuda.Event()
        join.record(side)
        main.wait_event(join)
        torch.cuda.synchronize()
        for t, ref in zip(state, serial):
            assert all(torch.equal(a, r) for a, r in zip(t["out"], ref))
    for t in state:
        x, w, b, dy = (v.numpy() for v in t["host"])
        y, dx, dw, db = t["out"]
        assert nerr(y, oracle.forward(t["op"], x, w, b)) <= TOL
        assert nerr(dx, oracle.backward_data(t["op"], w, dy)) <= TOL
        assert nerr(dw, oracle.backward_filter(t["op"], x, dy)) <= TOL
        assert nerr(db, oracle.backward_bias(t["op"], dy)) <= TOL


def test_passes_can_be_captured_in_a_hip_graph():
    """Every pass only enqueues kernels on the caller's stream (no allocation, no memset, no
    synchronisation), so a step can be captured once and replayed: replays after changes to the
    input buffers must match eager runs of the same inputs bit for bit."""
    pd = P(5, 6, 18, 17, 8, 3, 3, 2, 1, 1, 1, 1, 1, 2)
    op = OracleParams(**pd)
    d = conv.conv_desc_create(conv.ConvParams(**pd))
    ws = torch.zeros(max(conv.conv_desc_workspace_bytes(d) // 4, 1), device=DEV)
    x0, w0, b0, dy0 = workloads.random_inputs(oracle.x_shape(op), oracle.w_shape(op), oracle.output_shape(op), 808)
    xd, wd, bd, dyd = x0.to(DEV), w0.to(DEV), b0.to(DEV), dy0.to(DEV)
    y, dx, dw, db = torch.empty_like(dyd), torch.empty_like(xd), torch.empty_like(wd), torch.empty_like(bd)

    def step():
        conv.conv_forward(d, xd, wd, bd, y, ws)
        conv.conv_backward_data(d, wd, dyd, dx, ws)
        conv.conv_backward_filter(d, xd, dyd, dw, 0.0, ws)
        conv.conv_backward_bias(d, dyd, db, 0.0, ws)

    step()  # warm-up outside the capture (one-time kernel attribute set-up)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        x1, w1, b1, dy1 = workloads.random_inputs(oracle.x_shape(op), oracle.w_shape(op), oracle.output_shape(op),
                                                  900 + rep)
        xd.copy_(x1.to(DEV)); wd.copy_(w1.to(DEV)); bd.copy_(b1.to(DEV)); dyd.copy_(dy1.to(DEV))
        for t in (y, dx, dw, db):
            t.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (y, dx, dw, db)]
        step()  # eager, same inputs
        torch.cuda.synchronize()
        for a, e in zip(got, (y, dx, dw, db)):
            assert torch.equal(a, e)
        assert nerr(y, oracle.forward(op, x1.numpy(), w1.numpy(), b1.numpy())) <= TOL
        assert nerr(dw, oracle.backward_filter(op, x1.numpy(), dy1.numpy())) <= TOL


@pytest.mark.parametrize("name", ["5.a", "5.b", "5.c"])
def test_benchmark_layers_config_4_full(name):
    """The large configuration at full size, every output element of every pass against the oracle
    (the 16 host cores of the GPU machine finish one layer in a few seconds)."""
    l = workloads.BY_NAME[name]
    print("layer", name, "full compare", flush=True)
    pd = l.params_dict()
    op = OracleParams(**pd)
    x, w, b, dy = workloads.layer_inputs(l, bias="random")
    d, ws, _, (y, dx, dw, db) = run_all(pd, x, w, b, dy)
    xn, wn, bn, dyn = x.numpy(), w.numpy(), b.numpy(), dy.numpy()
    assert nerr(y, oracle.forward(op, xn, wn, bn)) <= TOL
    print("  forward ok", flush=True)
    assert nerr(dx, oracle.backward_data(op, wn, dyn)) <= TOL
    print("  backward data ok", flush=True)
    assert nerr(dw, oracle.backward_filter(op, xn, dyn)) <= TOL
    assert nerr(db, oracle.backward_bias(op, dyn)) <= TOL


@pytest.mark.parametrize("f64", [False, True], ids=["fp32", "fp64"])
def test_bench_probe_reports_clock_and_rate(f64):
    """The benchmark's register-loop helper (bench_probe.py): a plausible core clock and a rate below
    the published peak."""
    import bench_probe
    r = bench_probe.register_loop_rate(f64=f64, workgroups=512, iters=2048)
    print("mfma probe:", r, flush=True)
    assert 0.5 < r["core_clock_ghz"] < 3.0
    assert (20.0 < r["tflops"] < 80.0) if f64 else (40.0 < r["tflops"] < 160.0)
