"""The half-precision build of the library (libaxonn_stage_fp16.so: the paper's arithmetic, Sec. 2 "Mixed
precision") against the same fp64 oracle, to the same bounds as the bfloat16 build.

A process works with one of the two builds (AXONN_ELEM, read when the binding is imported), so the parity tests of the
single operations, of the stage, of the pipeline's ends and of loss scaling run again in a child process with
AXONN_ELEM=fp16: inputs are then rounded to half precision, device buffers are torch.float16, and the oracle rounds the
16-bit parameter copy to half precision."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

FP16_FILES = ["test_gpu_ops.py", "test_gpu_stage.py", "test_gpu_lm_ends.py", "test_gpu_loss_scaling.py",
              "test_gpu_checkpointing.py", "test_gpu_pipeline.py"]


@pytest.mark.skipif(os.environ.get("AXONN_ELEM", "bf16") != "bf16", reason="already the child process")
@pytest.mark.timeout(1500)
def test_half_precision_build_parity_suite():
    here = os.path.dirname(os.path.abspath(__file__))
    env = dict(os.environ, AXONN_ELEM="fp16")
    r = subprocess.run([sys.executable, "-m", "pytest", *[os.path.join(here, f) for f in FP16_FILES], "-x", "-q",
                        "-p", "no:cacheprovider", "-m", "gpu", "-k", "not copy_kernel"],
                       env=env, capture_output=True, text=True, timeout=1400, cwd=os.path.dirname(here))
    tail = r.stdout[-4000:] + r.stderr[-2000:]
    assert r.returncode == 0, tail
    assert " passed" in r.stdout and " failed" not in r.stdout, tail


@pytest.mark.skipif(os.environ.get("AXONN_ELEM", "bf16") != "bf16", reason="already the child process")
@pytest.mark.timeout(900)
def test_half_precision_build_full_size_stage():
    """The 12B-shape stage at full size, in the benchmark's launch configuration, with the half-precision build."""
    here = os.path.dirname(os.path.abspath(__file__))
    env = dict(os.environ, AXONN_ELEM="fp16")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(here, "test_gpu_fullsize.py"), "-x", "-q",
                        "-p", "no:cacheprovider", "-m", "gpu", "-k", "test_full_size_stage_parity and 12b-0 and not table1"],
                       env=env, capture_output=True, text=True, timeout=800, cwd=os.path.dirname(here))
    tail = r.stdout[-4000:] + r.stderr[-2000:]
    assert r.returncode == 0, tail
    assert "1 passed" in r.stdout, tail
