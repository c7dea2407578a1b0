import os
import sys
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _has_gpu():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _has_gpu():
        return
    skip = pytest.mark.skip(reason="no GPU in this environment")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


def pytest_sessionfinish(session, exitstatus):
    """AXONN_TEST_REPORT=1: the element-wise error factors the GPU parity checks measured, next to their bounds."""
    if os.environ.get("AXONN_TEST_REPORT") != "1":
        return
    try:
        import helpers
    except Exception:
        return
    worst = {}
    for label, f, c, e in helpers._elem_report:
        w = worst.setdefault(label, [0.0, c, 0.0, 0])
        w[0] = max(w[0], f); w[2] = max(w[2], e); w[3] += 1
    print("\nelement-wise factors (worst per label: factor / bound, rel_fro, checks)")
    for label, (f, c, e, n) in sorted(worst.items()):
        print("  %-40s %8.3f / %-8g  %.2e  %d" % (label, f, c, e, n))
