"""Turns rocprofv3 CSV output of a ``bench.py`` run into the short text summaries kept under profiles/.

    python profile_summary.py trace  <dir with *_kernel_trace.csv>  > profiles/<name>.txt
    python profile_summary.py traffic <fetch dir> <write dir> [--workload config4|f64|ip5|dw|pg]
    python profile_summary.py sq <dir with *_counter_collection.csv of an SQ_* --pmc run>

``trace`` prints calls / average / min / max duration per (kernel, grid).  ``traffic`` reads two
``--pmc`` runs (FETCH_SIZE, then WRITE_SIZE, both KiB per dispatch) of
``bench.py --copy-calibration``, scales each counter by what it reads for the plain 256 MiB device
copy in the same run, prints HBM bytes per (layer, pass) and merges them into
profiles/hbm_traffic.json (which bench.py reports as ``roofline.traffic``).  Dispatches are
matched to (layer, pass) by their order inside a step (the main kernel of each pass, per layer);
``--workload`` names the bench.py workload the two runs were made with.
``sq`` condenses a run with SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_VALU_MFMA_BUSY_CYCLES
SQ_INSTS_VALU_MFMA_MOPS_F32 (or _F64 for the double path) SQ_WAIT_INST_ANY SQ_LDS_BANK_CONFLICT SQ_INSTS_MFMA SQ_INSTS_VALU into MFMA
utilisation per kernel (counters are summed over 32 shader engines / 1024 SIMDs of the chip).
"""
from __future__ import annotations

import csv
import glob
import json
import os
import sys
from collections import OrderedDict

MAIN = ("corr_kernel", "corr_patch_kernel", "wgrad_kernel", "bias_grad_kernel")
PASSES = ("fwd", "bwd_data", "bwd_filter", "bwd_bias")
# workload -> (main kernels in pass order, pass names, layers, key prefix in hbm_traffic.json)
WORKLOADS = {
    # the default step takes both parameter gradients from one pass (conv_backward_filter_bias)
    "config4": (MAIN[:3], ("fwd", "bwd_data", "bwd_filter_bias"), ["5.a", "5.b", "5.c"], ""),
    "f64": (("corr64_kernel", "wgrad64_kernel", "bias_grad64_kernel"), PASSES, ["5.a", "5.b", "5.c"], "f64/"),
    "ip5": (("wgrad_kernel", "relu_bwd_kernel", "corr_kernel", "colsum_kernel", "colsum_direct_kernel"),
            ("fwd", "relu_bwd", "bwd_data", "bwd_filter", "bwd_bias"), ["ip5.6", "ip5.7", "ip5.8"], ""),
    "dw": (("direct_rows_kernel", "direct_rows_vec_kernel", "direct_rows_s2_kernel", "direct_bwd_blocks_kernel",
            "direct_bwd_s2_vec_kernel", "direct_wgrad_rows_kernel", "direct_wgrad_rows_vec_kernel",
            "direct_wgrad_rows_s2_kernel"), ("fwd", "bwd_data", "bwd_filter_bias"),
           ["dw.a", "dw.b", "dw.c", "dw.d", "dw.e"], ""),
    "pg": (("pg_sample_kernel", "pg_discount_kernel", "pg_sigmoid_kernel", "pg_softmax_rows_kernel"),
           ("sample_action", "discount_rewards", "sigmoid_bottom_diff", "softmax_bottom_diff"), ["pg"], ""),
}
COPY_BYTES = 256 * 1024 * 1024


def _short(name: str) -> str:
    return (name.replace("mi355conv::(anonymous namespace)::", "").replace("(mi355conv::", "(")
            .replace("void ", ""))


def _one(pattern: str) -> str:
    files = sorted(glob.glob(pattern, recursive=True))
    if not files:
        raise SystemExit(f"no file matches {pattern}")
    return files[0]


def trace(directory: str) -> None:
    rows = list(csv.DictReader(open(_one(os.path.join(directory, "**", "*kernel_trace.csv")))))
    agg: "OrderedDict[tuple, list]" = OrderedDict()
    for r in rows:
        blocks = int(r["Grid_Size_X"]) // max(int(r["Workgroup_Size_X"]), 1)
        key = (_short(r["Kernel_Name"])[:58], blocks, r["LDS_Block_Size"])
        agg.setdefault(key, []).append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
    print(f"{'kernel':58s} {'blocks':>7s} {'LDS B':>6s} {'calls':>5s} {'avg us':>9s} {'min us':>9s} {'max us':>9s}")
    for (name, blocks, lds), v in agg.items():
        print(f"{name:58s} {blocks:7d} {lds:>6s} {len(v):5d} {sum(v) / len(v) / 1e3:9.1f} {min(v) / 1e3:9.1f} "
              f"{max(v) / 1e3:9.1f}")


def _counter(directory: str):
    rows = list(csv.DictReader(open(_one(os.path.join(directory, "**", "*counter_collection.csv")))))
    return [(_short(r["Kernel_Name"]), int(r["Grid_Size"]) // max(int(r["Workgroup_Size"]), 1),
             float(r["Counter_Value"])) for r in rows]


def _per_pass(rows, main_kernels, passes, layers, prefix):
    copies = [v for n, b, v in rows if "copyBuffer" in n and b >= 256]  # the 256 MiB calibration copies only
    if not copies:
        raise SystemExit("no calibration copy found: run bench.py with --copy-calibration")
    kib_per_copy = sum(copies) / len(copies)
    factor = (COPY_BYTES / 1024.0) / kib_per_copy  # true KiB per counted KiB
    main = [(n, v) for n, b, v in rows if any(m + "<" in n or m + "(" in n for m in main_kernels)]
    per_step = len(layers) * len(passes)
    out: "OrderedDict[str, list]" = OrderedDict()
    for i, (n, v) in enumerate(main):
        layer, p = layers[(i % per_step) // len(passes)], passes[i % len(passes)]
        out.setdefault(f"{prefix}{layer}:{p}", []).append(v * factor * 1024.0)
    return factor, {k: sum(v) / len(v) for k, v in out.items()}


def traffic(fetch_dir: str, write_dir: str, workload: str) -> None:
    spec = WORKLOADS[workload]
    ff, fetch = _per_pass(_counter(fetch_dir), *spec)
    wf, write = _per_pass(_counter(write_dir), *spec)
    print(f"calibration: FETCH_SIZE x {ff:.3f}, WRITE_SIZE x {wf:.3f} (from the 256 MiB device copy)")
    print(f"{'layer:pass':22s} {'read MB':>10s} {'written MB':>11s} {'total MB':>10s}   (main kernel of the pass)")
    total = {}
    for k in fetch:
        total[k] = int(fetch[k] + write[k])
        print(f"{k:22s} {fetch[k] / 1e6:10.1f} {write[k] / 1e6:11.1f} {total[k] / 1e6:10.1f}")
    root = os.path.dirname(os.path.abspath(__file__))
    path = os.path.join(root, "profiles", "hbm_traffic.json")
    merged = json.load(open(path)) if os.path.exists(path) else {}
    merged.update(total)
    with open(path, "w") as f:
        json.dump(merged, f, indent=1)


def sq(directory: str) -> None:
    rows = list(csv.DictReader(open(_one(os.path.join(directory, "**", "*counter_collection.csv")))))
    agg: "OrderedDict[tuple, dict]" = OrderedDict()
    for r in rows:
        name = _short(r["Kernel_Name"])
        if not any(m in name for m in MAIN[:3] + ("corr64_kernel", "wgrad64_kernel")):
            continue
        key = (name[:50], int(r["Grid_Size"]) // max(int(r["Workgroup_Size"]), 1))
        agg.setdefault(key, {}).setdefault(r["Counter_Name"], []).append(float(r["Counter_Value"]))
    print(f"{'kernel':50s} {'blocks':>6s} {'kcycles':>8s} {'MFMA busy':>9s} {'GFLOP(mfma)':>11s} {'waves/SIMD':>10s} "
          f"{'wait':>5s} {'VALU/MFMA':>9s} {'LDS confl':>9s}")
    for (name, blocks), c in agg.items():
        v = {k: sum(x) / len(x) for k, x in c.items()}
        cyc = v["SQ_BUSY_CYCLES"] / 32.0
        print(f"{name:50s} {blocks:6d} {cyc / 1e3:8.0f} {100 * v['SQ_VALU_MFMA_BUSY_CYCLES'] / 1024 / cyc:8.1f}% "
              f"{v.get('SQ_INSTS_VALU_MFMA_MOPS_F32', v.get('SQ_INSTS_VALU_MFMA_MOPS_F64', 0.0)) * 512 / 1e9:11.2f} "
              f"{v['SQ_WAVE_CYCLES'] * 4 / 1024 / cyc:10.2f} "
              f"{100 * v['SQ_WAIT_INST_ANY'] / v['SQ_WAVE_CYCLES']:4.0f}% "
              f"{(v['SQ_INSTS_VALU'] - v['SQ_INSTS_MFMA']) / v['SQ_INSTS_MFMA']:9.2f} {v['SQ_LDS_BANK_CONFLICT']:9.0f}")


def main(argv) -> None:
    if len(argv) >= 3 and argv[1] == "trace":
        trace(argv[2])
    elif len(argv) >= 3 and argv[1] == "sq":
        sq(argv[2])
    elif len(argv) >= 4 and argv[1] == "traffic":
        workload = argv[argv.index("--workload") + 1] if "--workload" in argv else "config4"
        traffic(argv[2], argv[3], workload)
    else:
        raise SystemExit(__doc__)


if __name__ == "__main__":
    main(sys.argv)
