"""Which kernel variant does every case of the GPU parity suite select?  Runs on the CPU: creating a
descriptor touches no device, and conv_desc_kernel_names spells out every template parameter and
run-time branch that selects different kernel code (tile, bounds mode, patch staging, epilogue form,
LDS-direct or register staging, direct-kernel form).  The assertions below say that each variant the
library can select is selected by at least one case the default `-m gpu` run compares with the oracle --
so a variant without a parity test fails here, on the CPU, before any GPU run."""
import re

import numpy as np
import pytest

import paper_1810_02272_amd as conv
import parity_cases as pc

CORR_TILES = ["corr_m32_128x128x16", "corr_m32_128x64x16", "corr_m32_96x128x16", "corr_m32_64x128x16",
              "corr_m32_64x64x16", "corr_m32_32x256x16", "corr_m32_32x128x16", "corr_m16_48x256x16",
              "corr_m16_48x128x16", "corr_m16_16x256x16", "corr_m16_16x64x16"]
PATCH_TILES = ["corr_m32_128x128x16", "corr_m32_32x128x16", "corr_m32_32x256x16", "corr_m16_48x256x16",
               "corr_m16_16x256x16"]
WGRAD_TILES = ["wgrad_m32_128x128x32", "wgrad_m32_96x128x32", "wgrad_m32_64x128x32", "wgrad_m32_32x128x32",
               "wgrad_m32_128x64x32"]
F64_ROWS = [96, 64, 48, 32, 16]
DIRECT_FWD = ["elem", "rows_k3", "rows_k3_unit", "rows_k5", "rows_k5_unit", "rows_vec_k3", "rows_vec_k5", "s2_k3", "s2_k5"]
DIRECT_BWD = ["elem", "elem_k3", "rows_k3", "rows_k3_unit", "rows_k5", "rows_k5_unit", "rows_vec_k3", "rows_vec_k5",
              "bwd_s2_vec_k3", "bwd_s2_vec_k5", "bwd_blocks_k3", "bwd_blocks_k5"]
DIRECT_WGRAD = ["wgrad_taps", "rows_k3", "rows_k3_unit", "rows_k5", "rows_k5_unit", "rows_vec_k3", "rows_vec_k5", "s2_k3",
                "s2_k5"]


def fields(names):
    return dict(kv.split("=", 1) for kv in names.split(";"))


def split_variant(v):
    """'tile[m2,es](S=4,L=3)' -> ('tile[m2,es]', 4)"""
    m = re.fullmatch(r"(.*)\(S=(\d+),L=\d+\)", v)
    return (m.group(1), int(m.group(2))) if m else (v, 1)


@pytest.fixture(scope="module")
def selected():
    """pass -> {variant: number of splits seen}, over every fp32 case; the same for fp64."""
    out = {"fp32": {}, "fp64": {}}
    for key, cases, names in (("fp32", pc.fp32_conv_cases(), conv.conv_desc_kernel_names),
                              ("fp64", pc.fp64_conv_cases(), conv.conv_desc_kernel_names_f64)):
        for pd in cases:
            d = conv.conv_desc_create(conv.ConvParams(**pd))
            for which, v in fields(names(d)).items():
                variant, splits = split_variant(v)
                out[key].setdefault(which, {}).setdefault(variant, set()).add(splits > 1)
    return out


def missing(have, want):
    return sorted(w for w in want if not any(h.startswith(w) for h in have))


def test_every_gather_tile_and_bounds_mode_has_a_gpu_parity_case(selected):
    fwd, bwd = selected["fp32"]["fwd"], selected["fp32"]["bwd_data"]
    # forward takes every bounds mode; a backward-data gather always has padding (modes 1 and 2)
    assert missing(fwd, [f"{t}[m{m}," for t in CORR_TILES for m in (0, 1, 2)]) == []
    assert missing(bwd, [f"{t}[m{m}," for t in CORR_TILES for m in (1, 2)]) == []
    assert not any("[m0" in v for v in bwd)


def test_every_thin_row_count_and_bounds_mode_has_a_gpu_parity_case(selected):
    """corr_thin_kernel (at most four GEMM rows per group): ROWS x MODE instances, always the offset-only epilogue."""
    fwd, bwd = selected["fp32"]["fwd"], selected["fp32"]["bwd_data"]
    assert missing(fwd, [f"corr_thin_r{r}[m{m},es]" for r in (1, 2, 3, 4) for m in (0, 1, 2)]) == []
    assert missing(bwd, [f"corr_thin_r{r}[m{m},es]" for r in (1, 2, 3, 4) for m in (1, 2)]) == []
    # the LDS-staged form (stride-1, dilation-1 gathers with 3x3 or 5x5 taps whose rows fit LDS)
    staged = [f"corr_thin_r{r}_lds{tw}[es]" for r in (1, 2, 3, 4) for tw in (3, 5)]
    assert missing(fwd, staged) == []
    assert missing(bwd, staged) == []
    for v, seen in list(fwd.items()) + list(bwd.items()):
        if v.startswith("corr_thin"):
            assert seen == {False}, v   # never split


def test_every_patch_tile_has_a_gpu_parity_case(selected):
    fwd, bwd = selected["fp32"]["fwd"], selected["fp32"]["bwd_data"]
    assert missing(fwd, [f"{t}_patch[es]" for t in PATCH_TILES]) == []      # forward: one phase per channel
    assert missing(bwd, [f"{t}_patch[e{e}]" for t in PATCH_TILES for e in "sr"]) == []
    # no other tile may take the patch kernel: it is built for these five only
    for v in list(fwd) + list(bwd):
        if "_patch" in v:
            assert v.split("_patch")[0] in PATCH_TILES, v


def test_every_epilogue_form_and_split_launches_have_gpu_parity_cases(selected):
    fwd, bwd = selected["fp32"]["fwd"], selected["fp32"]["bwd_data"]
    forms = lambda have: {re.search(r",e(.)\]", v).group(1) for v in have if re.search(r",e(.)\]", v)}
    assert forms(fwd) >= {"s"} and forms(bwd) >= {"s", "r"}
    # split reductions (partial outputs + reduce kernel) with both range-checked epilogue forms
    assert any(True in s for v, s in fwd.items() if ",es]" in v)
    assert any(True in s for v, s in bwd.items() if ",es]" in v)
    assert any(True in s for v, s in bwd.items() if ",er]" in v)
    # The plain-pointer form (a blob of 2^31 bytes or more) is run by test_blobs_between_1_and_4_gib:
    big = pc.P(37, 4, 2000, 2000, 4, 3, 3, 1, 1, 1, 1)
    names = fields(conv.conv_desc_kernel_names(conv.conv_desc_create(conv.ConvParams(**big))))
    assert ",ep]" in names["fwd"] and ",ep]" in names["bwd_data"] and "[m1" in names["fwd"], names


def test_every_filter_gradient_tile_and_bounds_mode_has_a_gpu_parity_case(selected):
    wg = selected["fp32"]["bwd_filter"]
    assert missing(wg, [f"{t}[m{m}," for t in WGRAD_TILES for m in (0, 1, 2)]) == []
    for v in wg:   # staging is a property of the tile
        if v.startswith("wgrad"):
            assert ("lds" in v) == v.startswith("wgrad_m32_128x128x32"), v
    assert {"one", "two"} <= {re.search(r"\[(\w+)\]", v).group(1) for v in selected["fp32"]["bwd_bias"]}


def test_every_direct_form_has_a_gpu_parity_case(selected):
    for key, prefix in (("fp32", "direct"), ("fp64", "direct64")):
        s = selected[key]
        assert missing(s["fwd"], [f"{prefix}[{f}]" for f in DIRECT_FWD]) == [], key
        assert missing(s["bwd_data"], [f"{prefix}[{f}]" for f in DIRECT_BWD]) == [], key
        assert missing(s["bwd_filter"], [f"{prefix}[{f}]" for f in DIRECT_WGRAD]) == [], key
        known = {f"{prefix}[{f}]" for f in DIRECT_FWD + DIRECT_BWD + DIRECT_WGRAD}
        for which in ("fwd", "bwd_data", "bwd_filter"):
            for v in s[which]:
                if v.startswith(prefix + "["):
                    assert v in known, v   # a form this test does not know about


def test_every_fp64_tile_has_a_gpu_parity_case(selected):
    s = selected["fp64"]
    assert missing(s["fwd"], [f"corr64_{r}x64x16[es]" for r in F64_ROWS]) == []
    assert missing(s["bwd_data"], [f"corr64_{r}x64x16[e{e}]" for r in F64_ROWS for e in "sp"]) == []
    assert missing(s["bwd_filter"], [f"wgrad64_{r}x64x16" for r in F64_ROWS]) == []
    # split reductions (partial outputs + reduce64_kernel): forward, backward data with both epilogue forms
    assert any(True in seen for v, seen in s["fwd"].items() if v.startswith("corr64") and "[es]" in v)
    assert any(True in seen for v, seen in s["bwd_data"].items() if v.startswith("corr64") and "[es]" in v)
    assert any(True in seen for v, seen in s["bwd_data"].items() if v.startswith("corr64") and "[ep]" in v)


def test_no_variant_outside_the_lists_above(selected):
    """A new tile or flag must be added to the lists of this file (and so get a parity case)."""
    for v in list(selected["fp32"]["fwd"]) + list(selected["fp32"]["bwd_data"]):
        if v.startswith("corr_thin"):
            assert re.fullmatch(r"corr_thin_r[1234](\[m[012],es\]|_lds[35]\[es\])", v), v
        elif v.startswith("corr_"):
            assert re.fullmatch(r"(%s)(\[m[012],e[srp]\]|_patch\[e[sr]\])" % "|".join(CORR_TILES), v), v
    for v in selected["fp32"]["bwd_filter"]:
        if v.startswith("wgrad"):
            assert re.fullmatch(r"(%s)\[m[012],(lds|reg),e[rp]\]" % "|".join(WGRAD_TILES), v), v
    for which in ("fwd", "bwd_data"):
        for v in selected["fp64"][which]:
            if v.startswith("corr64"):
                assert re.fullmatch(r"corr64_(%s)x64x16\[e[sp]\]" % "|".join(map(str, F64_ROWS)), v), v


def test_inner_product_shapes_cover_the_three_contractions():
    """The InnerProduct passes run on the convolution kernels; its GPU cases add variants of their own
    (the filter-gradient kernel with a bias / ReLU reduce, accumulation in the gather epilogue)."""
    from paper_1810_02272_amd import workloads

    shapes = list(pc.IP_SHAPES) + [(l.m, l.k, l.num_output) for l in workloads.IP_LAYERS]
    rng = np.random.default_rng(pc.IP_RANDOM[0])
    shapes += [pc.random_ip_case(rng)[:3] for _ in range(pc.IP_RANDOM[1])]
    seen = {"fwd": set(), "bwd_data": set(), "bwd_filter": set()}
    for m, k, o in shapes:
        d = conv.ip_desc_create(conv.IpParams(m, k, o, 1, 1))
        for which, v in fields(conv.ip_desc_kernel_names(d)).items():
            if which in seen:
                seen[which].add(split_variant(v)[0])
    assert all(v.startswith("wgrad") for v in seen["fwd"]) and len(seen["fwd"]) >= 3, seen["fwd"]
    assert all(v.startswith("corr") for v in seen["bwd_data"] | seen["bwd_filter"])
    # beta = 1: the filter gradient is added in the epilogue of the gather kernels and of the kernel for GEMMs of at
    # most four rows (test_ip_beta_one_accumulates)
    beta_kernels = set()
    for m, k, o in pc.IP_BETA_SHAPES:
        d = conv.ip_desc_create(conv.IpParams(m, k, o, 1, 1))
        beta_kernels.add(split_variant(fields(conv.ip_desc_kernel_names(d))["bwd_filter"])[0].split("[")[0])
    assert any(v.startswith("corr_thin_r") for v in beta_kernels), beta_kernels
    assert any(v.startswith("corr_m") for v in beta_kernels), beta_kernels
    # a forward output of more than 2^30 bytes takes the plain-pointer store of the filter-gradient kernel
    # (test_ip_forward_output_above_1_gib)
    d = conv.ip_desc_create(conv.IpParams(16400, 2, 16400, 1, 0))
    assert ",ep]" in fields(conv.ip_desc_kernel_names(d))["fwd"]
