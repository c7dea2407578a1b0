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


# The parity tests of these modules run once with each of the two 16-bit element types (the library's bfloat16 and
# half-precision builds, both loaded into this process): inputs are rounded to the type, device buffers are of the
# type, and the oracle rounds the 16-bit parameter copy to it.  Of the full-size cases only the 12B-shape stage
# runs in half precision as well.
BOTH_ELEMENT_TYPES = {"test_gpu_ops", "test_gpu_stage", "test_gpu_lm_ends", "test_gpu_loss_scaling",
                      "test_gpu_checkpointing", "test_gpu_pipeline"}
FULL_SIZE_IN_HALF = ("test_gpu_fullsize", "test_full_size_stage_parity", {"name": "12b", "ac": 0})


def pytest_generate_tests(metafunc):
    if "axonn_elem" not in metafunc.fixturenames:
        return
    mod = metafunc.module.__name__.rsplit(".", 1)[-1]
    if mod in BOTH_ELEMENT_TYPES or (mod, metafunc.function.__name__) == FULL_SIZE_IN_HALF[:2]:
        metafunc.parametrize("axonn_elem", ["bf16", "fp16"], indirect=True)


@pytest.fixture(autouse=True)
def axonn_elem(request):
    """Selects the element type of a test (parametrized above; otherwise the process's own, AXONN_ELEM)."""
    elem = getattr(request, "param", None)
    if elem is None:
        yield None
        return
    from paper_2110_13005_amd import binding as B
    if elem == "fp16":
        name = request.node.name
        if "copy_kernel" in name:
            pytest.skip("the launcher's knobs are exercised with the bfloat16 build")
        mod = request.module.__name__.rsplit(".", 1)[-1]
        if mod == FULL_SIZE_IN_HALF[0]:
            params = request.node.callspec.params
            if any(params.get(k) != v for k, v in FULL_SIZE_IN_HALF[2].items()):
                pytest.skip("full size in half precision: the 12B-shape stage only")
    before = B.ELEM
    B.select_elem(elem)
    try:
        yield elem
    finally:
        B.select_elem(before)


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
