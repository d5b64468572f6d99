import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


def pytest_collection_modifyitems(config, items):
    """Skip gpu-marked tests when no GPU is visible (they are deselected with -m "not gpu" anyway)."""
    try:
        import torch
        have_gpu = torch.cuda.is_available()
    except Exception:  # pragma: no cover
        have_gpu = False
    if have_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


def pytest_terminal_summary(terminalreporter):
    """How often the small-tensor rule of parity_metric.py replaced the plain error metric, and where."""
    try:
        import parity_metric
    except Exception:  # pragma: no cover
        return
    rec = parity_metric.FALLBACKS
    terminalreporter.write_line(f"parity metric: term-scale denominator used {len(rec)} time(s) "
                                f"(tensors of at most {parity_metric.SMALL_TENSOR} elements that miss the plain bar)")
    for r in rec:
        terminalreporter.write_line(f"  {r['tensor']} ({r['elements']} elements) plain {r['plain']:.3e} -> "
                                    f"scaled {r['scaled']:.3e}: {r['case']}")
