"""Host-only checks of the C boundary (no GPU): the library loads, exports every symbol the header
declares, validates parameters, computes output shapes and sizes its workspace."""
import ctypes
import json
import os
import re

import pytest

import paper_1810_02272_amd as conv
from paper_1810_02272_amd import binding, workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(ROOT, "tests", "golden")


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "mi355conv.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(conv_[a-z0-9_]+)\s*\(", header))
    assert {"conv_desc_create", "conv_forward", "conv_backward_data", "conv_backward_filter",
            "conv_backward_bias", "conv_desc_workspace_bytes_f64", "conv_forward_f64", "conv_backward_data_f64",
            "conv_backward_filter_f64", "conv_backward_bias_f64"} <= declared
    lib = ctypes.CDLL(conv.library_path())
    for name in declared:
        assert hasattr(lib, name), name


def test_output_shape_matches_size_table():
    table = json.load(open(os.path.join(GOLDEN, "output_sizes.json")))
    for i, k, s, pad, d, out in table["rows"]:
        p = conv.ConvParams(1, 1, i, i, 1, k, k, s, s, pad, pad, d, d)
        if out < 1:
            with pytest.raises(conv.ConvError) as e:
                conv.conv_desc_create(p)
            assert e.value.status == binding.CONV_ESHAPE
        else:
            assert conv.conv_desc_output_shape(conv.conv_desc_create(p)) == (1, 1, out, out)


def test_benchmark_layers_shapes_and_workspace():
    for l in workloads.LAYERS:
        d = conv.conv_desc_create(conv.ConvParams(**l.params_dict()))
        assert conv.conv_desc_output_shape(d) == l.y_shape
        assert 0 < conv.conv_desc_workspace_bytes(d) < (1 << 30)
        names = conv.conv_desc_kernel_names(d)
        assert "fwd=" in names and "bwd_data=" in names and "bwd_filter=" in names


def test_thin_groups_select_the_direct_kernels():
    """Depthwise and near-depthwise descriptors take the direct kernels (forward and backward data then
    need no workspace); wide groups and ungrouped layers stay on the matrix-unit tiles."""
    for l in workloads.DW_LAYERS:
        d = conv.conv_desc_create(conv.ConvParams(**l.params_dict()))
        assert conv.conv_desc_output_shape(d) == l.y_shape
        names = dict(kv.split("=", 1) for kv in conv.conv_desc_kernel_names(d).split(";"))
        assert all(names[k].startswith("direct[") for k in ("fwd", "bwd_data", "bwd_filter")), names
        assert conv.conv_desc_kernel_names_f64(d).startswith("fwd=direct64[")
        assert 0 < conv.conv_desc_workspace_bytes(d) <= 32 << 20
    for l in workloads.LAYERS:
        assert "direct" not in conv.conv_desc_kernel_names(conv.conv_desc_create(conv.ConvParams(**l.params_dict())))
    base = dict(n=4, h=20, w=20, kernel_h=3, kernel_w=3, pad_h=1, pad_w=1)
    for c, k, g, direct in [(32, 32, 32, True), (32, 128, 32, True), (32, 32, 8, True), (64, 64, 8, False),
                            (32, 512, 32, False), (32, 32, 1, False)]:
        names = conv.conv_desc_kernel_names(conv.conv_desc_create(conv.ConvParams(c=c, num_output=k, group=g, **base)))
        assert ("direct" in names) == direct, (c, k, g, names)
    # more than 64 taps: the filter gradient's lane layout does not apply
    big = conv.conv_desc_create(conv.ConvParams(n=1, c=8, h=20, w=20, num_output=8, kernel_h=9, kernel_w=9, group=8))
    assert "direct" not in conv.conv_desc_kernel_names(big)


@pytest.mark.parametrize("bad", [
    dict(c=0), dict(h=0), dict(num_output=0), dict(kernel_h=0), dict(stride_w=0), dict(pad_h=-1),
    dict(dilation_w=0), dict(group=0), dict(group=2, c=3), dict(group=2, c=4, num_output=3), dict(bias_term=2),
    dict(n=-1),
])
def test_invalid_parameters_are_rejected(bad):
    base = dict(n=2, c=4, h=8, w=8, num_output=4, kernel_h=3, kernel_w=3)
    base.update(bad)
    with pytest.raises(conv.ConvError) as e:
        conv.conv_desc_create(conv.ConvParams(**base))
    assert e.value.status == binding.CONV_EINVAL


def test_too_large_tensors_are_rejected():
    big = 2 ** 31 - 1
    for prm in [(4096, 64, 128, 128, 64, 3, 3),
                (big, big, 2 ** 24, 2 ** 24, big, 1, 1),   # products far beyond 64 bits
                (1, big, 1, 1, big, 1, 1),                 # weight blob alone too large
                (big, 1, 1, 1, 1, 1, 1)]:                  # 2^31 - 1 images of one element
        with pytest.raises(conv.ConvError) as e:
            conv.conv_desc_create(conv.ConvParams(*prm))
        assert e.value.status == binding.CONV_ESHAPE, prm


def test_null_arguments_and_status_strings():
    lib = binding._load()
    assert lib.conv_desc_create(None, None) == binding.CONV_EINVAL
    assert lib.conv_desc_destroy(None) == binding.CONV_EINVAL
    assert lib.conv_desc_workspace_bytes(None, None) == binding.CONV_EINVAL
    d = conv.conv_desc_create(conv.ConvParams(1, 1, 4, 4, 1, 3, 3, bias_term=0))
    # null tensors, bias given for bias_term = 0, bias gradient on a bias-free layer, beta not 0/1
    assert lib.conv_forward(d.handle, None, None, None, None, None, 0, None) == binding.CONV_EINVAL
    assert lib.conv_forward(d.handle, 16, 16, 16, 16, None, 0, None) == binding.CONV_EINVAL
    assert lib.conv_backward_bias(d.handle, 16, 16, 0.0, 16, 1 << 20, None) == binding.CONV_EINVAL
    assert lib.conv_backward_filter(d.handle, 16, 16, 16, 0.5, 16, 1 << 20, None) == binding.CONV_EINVAL
    assert lib.conv_backward_filter_bias(d.handle, 16, 16, 16, 16, 0.0, 16, 1 << 20, None) == binding.CONV_EINVAL
    db_ok = conv.conv_desc_create(conv.ConvParams(1, 1, 4, 4, 1, 3, 3, bias_term=1))
    assert lib.conv_backward_filter_bias(db_ok.handle, 16, 16, 16, None, 0.0, 16, 1 << 20, None) == binding.CONV_EINVAL
    assert lib.conv_backward_filter_bias(db_ok.handle, 16, 16, 16, 16, 2.0, 16, 1 << 20, None) == binding.CONV_EINVAL
    assert lib.conv_backward_filter_bias(db_ok.handle, 16, 16, 16, 16, 0.0, None, 0, None) == binding.CONV_EWORKSPACE
    # workspace missing / too small is detected before anything is enqueued
    # (a layer large enough to pack its weights into the workspace first; small ones read them directly)
    big = conv.conv_desc_create(conv.ConvParams(64, 256, 16, 16, 256, 3, 3, bias_term=0))
    assert lib.conv_forward(big.handle, 16, 16, None, 16, None, 0, None) == binding.CONV_EWORKSPACE
    assert lib.conv_backward_data(big.handle, 16, 16, 16, 16, 4, None) == binding.CONV_EWORKSPACE
    assert lib.conv_backward_filter(d.handle, 16, 16, 16, 1.0, None, 0, None) == binding.CONV_EWORKSPACE
    for s in (0, -1, -2, -3, -4, -99):
        assert conv.conv_status_string(s)
    assert conv.conv_status_string(0) == "success"


def test_bench_probe_library_checks_arguments_and_the_layer_library_has_no_probe():
    """The register-loop probe is a benchmark helper in a library of its own (bench_probe.hip beside
    bench.py); the layer library exports no such symbol."""
    import bench_probe
    lib = bench_probe.load()
    assert lib.bench_mfma_probe(0, 4, 10, None, None, None) == -1
    for wg, it in ((0, 10), (65537, 10), (4, 0), (4, (1 << 20) + 1)):
        assert lib.bench_mfma_probe(0, wg, it, 16, None, None) == -1
        assert lib.bench_mfma_probe(1, wg, it, 16, None, None) == -1
    import torch
    with pytest.raises(ValueError):
        bench_probe.mfma_probe(4, 10, torch.zeros(32, dtype=torch.int64))
    assert not hasattr(ctypes.CDLL(conv.library_path()), "conv_mfma_probe")


def test_static_workspace_refuses_layers_beyond_its_limit_and_bad_arguments():
    """conv_backward_filter_static: argument and size errors are found before any runtime call."""
    lib = binding._load()
    # a weight blob of 36 MiB: even one slice of partials exceeds the 32 MiB array
    d = conv.conv_desc_create(conv.ConvParams(**dict(n=1, c=1024, h=8, w=8, num_output=1024, kernel_h=3, kernel_w=3, pad_h=1, pad_w=1)))
    assert lib.conv_backward_filter_static(d.handle, 16, 16, 16, ctypes.c_float(0.0), None) == binding.CONV_EWORKSPACE
    ok = conv.conv_desc_create(conv.ConvParams(**dict(n=1, c=2, h=5, w=5, num_output=2, kernel_h=3, kernel_w=3)))
    assert lib.conv_backward_filter_static(None, 16, 16, 16, ctypes.c_float(0.0), None) == binding.CONV_EINVAL
    assert lib.conv_backward_filter_static(ok.handle, 16, 16, None, ctypes.c_float(0.0), None) == binding.CONV_EINVAL
    assert lib.conv_backward_filter_static(ok.handle, 16, 16, 16, ctypes.c_float(0.5), None) == binding.CONV_EINVAL
    assert lib.conv_backward_filter_static(ok.handle, None, 16, 16, ctypes.c_float(0.0), None) == binding.CONV_EINVAL


def test_binding_refuses_cpu_tensors():
    import torch
    p = conv.ConvParams(1, 1, 4, 4, 1, 3, 3)
    d = conv.conv_desc_create(p)
    x = torch.zeros(1, 1, 4, 4)
    with pytest.raises(TypeError):
        conv.conv_forward(d, x, torch.zeros(1, 1, 3, 3), torch.zeros(1), torch.zeros(1, 1, 2, 2))


# ---- InnerProduct boundary (include/mi355ip.h) ----

def test_library_exports_every_declared_ip_symbol():
    header = open(os.path.join(ROOT, "include", "mi355ip.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(ip_[a-z_]+)\s*\(", header))
    assert {"ip_desc_create", "ip_desc_destroy", "ip_desc_workspace_bytes", "ip_desc_kernel_names", "ip_forward",
            "ip_relu_backward", "ip_backward_data", "ip_backward_filter", "ip_backward_bias"} <= declared
    lib = ctypes.CDLL(conv.library_path())
    for name in declared:
        assert hasattr(lib, name), name


def test_ip_descriptors_and_workspace():
    for m, k, o in [(128, 9216, 4096), (64, 800, 500), (64, 500, 10), (1, 4, 1), (0, 5, 3), (7, 33, 129)]:
        d = conv.ip_desc_create(conv.IpParams(m, k, o, 1, 1))
        assert 0 < conv.ip_desc_workspace_bytes(d) < (1 << 30)
        names = conv.ip_desc_kernel_names(d)
        assert all(key in names for key in ("fwd=", "bwd_data=", "bwd_filter=", "bwd_bias="))
        conv.ip_desc_destroy(d)
        conv.ip_desc_destroy(d)  # idempotent through the binding


@pytest.mark.parametrize("bad", [dict(m=-1), dict(k=0), dict(num_output=0), dict(bias_term=2), dict(relu=-1)])
def test_ip_invalid_parameters_are_rejected(bad):
    base = dict(m=4, k=8, num_output=3, bias_term=1, relu=0)
    base.update(bad)
    with pytest.raises(conv.ConvError) as e:
        conv.ip_desc_create(conv.IpParams(**base))
    assert e.value.status == binding.CONV_EINVAL


def test_ip_too_large_is_a_shape_error():
    with pytest.raises(conv.ConvError) as e:
        conv.ip_desc_create(conv.IpParams(m=1 << 16, k=1 << 15, num_output=8))
    assert e.value.status == binding.CONV_ESHAPE


def test_ip_null_arguments_and_flags():
    lib = binding._load()
    conv.ip_desc_create(conv.IpParams(1, 1, 1))  # sets the argtypes
    d = conv.ip_desc_create(conv.IpParams(4, 8, 3, 1, 1))
    dn = conv.ip_desc_create(conv.IpParams(4, 8, 3, 0, 0))
    fake = ctypes.c_void_p(256)  # never dereferenced: every call below must fail before any launch
    assert lib.ip_desc_create(None, None) == binding.CONV_EINVAL
    assert lib.ip_forward(None, fake, fake, fake, fake, None, 0, None) == binding.CONV_EINVAL
    assert lib.ip_forward(d.handle, fake, fake, None, fake, None, 0, None) == binding.CONV_EINVAL      # bias missing
    assert lib.ip_forward(dn.handle, fake, fake, fake, fake, None, 0, None) == binding.CONV_EINVAL     # bias unexpected
    assert lib.ip_forward(d.handle, fake, fake, fake, fake, None, 0, None) == binding.CONV_EWORKSPACE
    assert lib.ip_relu_backward(d.handle, None, fake, fake, None) == binding.CONV_EINVAL               # relu needs y
    assert lib.ip_backward_data(d.handle, fake, None, fake, None, 0, None) == binding.CONV_EINVAL
    # (a layer large enough for its gather passes to pack their weights into the workspace first)
    big = conv.ip_desc_create(conv.IpParams(128, 4096, 4096, 1, 1))
    assert lib.ip_backward_data(big.handle, fake, fake, fake, None, 0, None) == binding.CONV_EWORKSPACE
    assert lib.ip_backward_filter(d.handle, fake, fake, fake, 0.5, fake, 1 << 20, None) == binding.CONV_EINVAL
    assert lib.ip_backward_filter(big.handle, fake, fake, fake, 1.0, None, 0, None) == binding.CONV_EWORKSPACE
    assert lib.ip_backward_bias(dn.handle, fake, fake, 0.0, fake, 1 << 20, None) == binding.CONV_EINVAL
    assert lib.ip_backward_bias(d.handle, fake, fake, 0.0, None, 0, None) == binding.CONV_EWORKSPACE
    assert lib.ip_desc_workspace_bytes(None, None) == binding.CONV_EINVAL


# ---- policy-gradient boundary (include/mi355pg.h) ----

def test_library_exports_every_declared_pg_symbol_and_checks_arguments():
    header = open(os.path.join(ROOT, "include", "mi355pg.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(pg_[a-z_]+)\s*\(", header))
    assert {"pg_sigmoid_sample_action", "pg_discount_rewards", "pg_sigmoid_bottom_diff",
            "pg_softmax_bottom_diff"} == declared
    from paper_1810_02272_amd import pg_binding
    lib = pg_binding._load()
    for name in declared:
        assert hasattr(lib, name), name
    fake = ctypes.c_void_p(256)  # never dereferenced: every call below returns before any launch
    assert lib.pg_sigmoid_sample_action(fake, fake, fake, -1, None) == binding.CONV_EINVAL
    assert lib.pg_sigmoid_sample_action(None, fake, fake, 4, None) == binding.CONV_EINVAL
    assert lib.pg_sigmoid_sample_action(None, None, None, 0, None) == binding.CONV_OK
    assert lib.pg_discount_rewards(fake, None, 2, 8, 0.9, fake, None) == binding.CONV_EINVAL
    assert lib.pg_discount_rewards(None, None, 0, 0, 0.9, None, None) == binding.CONV_OK
    assert lib.pg_sigmoid_bottom_diff(fake, fake, None, None, None, 4, None) == binding.CONV_EINVAL
    assert lib.pg_softmax_bottom_diff(fake, fake, None, None, fake, 4, 0, None) == binding.CONV_EINVAL
    assert lib.pg_softmax_bottom_diff(fake, fake, None, None, fake, 1 << 30, 2, None) == binding.CONV_ESHAPE
    assert lib.pg_softmax_bottom_diff(None, None, None, None, None, 0, 3, None) == binding.CONV_OK
    big = 0x7FFFFFFF  # beyond what the kernels' 32-bit index arithmetic covers
    assert lib.pg_sigmoid_sample_action(fake, fake, fake, big, None) == binding.CONV_ESHAPE
    assert lib.pg_sigmoid_bottom_diff(fake, fake, None, None, fake, big, None) == binding.CONV_ESHAPE
    assert lib.pg_discount_rewards(fake, fake, 4, big, 0.9, fake, None) == binding.CONV_ESHAPE


def test_f64_entry_points_check_arguments():
    lib = binding._load()
    d = conv.conv_desc_create(conv.ConvParams(2, 4, 8, 8, 4, 3, 3))
    dn = conv.conv_desc_create(conv.ConvParams(2, 4, 8, 8, 4, 3, 3, bias_term=0))
    assert conv.conv_desc_workspace_bytes_f64(d) > 0
    assert "fwd=corr64_" in conv.conv_desc_kernel_names_f64(d)
    fake = ctypes.c_void_p(256)  # never dereferenced: every call below fails before any launch
    assert lib.conv_forward_f64(None, fake, fake, fake, fake, None, 0, None) == binding.CONV_EINVAL
    assert lib.conv_forward_f64(d.handle, fake, fake, None, fake, None, 0, None) == binding.CONV_EINVAL
    assert lib.conv_forward_f64(dn.handle, fake, fake, fake, fake, None, 0, None) == binding.CONV_EINVAL
    assert lib.conv_forward_f64(d.handle, fake, fake, fake, fake, None, 0, None) == binding.CONV_EWORKSPACE
    assert lib.conv_backward_data_f64(d.handle, fake, None, fake, None, 0, None) == binding.CONV_EINVAL
    assert lib.conv_backward_data_f64(d.handle, fake, fake, fake, fake, 8, None) == binding.CONV_EWORKSPACE
    assert lib.conv_backward_filter_f64(d.handle, fake, fake, fake, 0.5, fake, 1 << 20, None) == binding.CONV_EINVAL
    assert lib.conv_backward_filter_f64(d.handle, fake, fake, fake, 1.0, None, 0, None) == binding.CONV_EWORKSPACE
    assert lib.conv_backward_bias_f64(dn.handle, fake, fake, 0.0, fake, 1 << 20, None) == binding.CONV_EINVAL
    assert lib.conv_backward_bias_f64(d.handle, fake, fake, 0.0, None, 0, None) == binding.CONV_EWORKSPACE
    # a blob of 2^29 elements or more has no double path
    big = conv.conv_desc_create(conv.ConvParams(1 << 10, 1 << 9, 32, 32, 1, 1, 1))
    with pytest.raises(conv.ConvError) as e:
        conv.conv_desc_workspace_bytes_f64(big)
    assert e.value.status == binding.CONV_ESHAPE
    assert lib.conv_forward_f64(big.handle, fake, fake, fake, fake, fake, 1 << 40, None) == binding.CONV_ESHAPE
    assert conv.conv_desc_kernel_names_f64(big) == ""
