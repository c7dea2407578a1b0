"""CPU-side checks of the C-ABI library: it loads without a GPU and exports every symbol the
header declares; argument validation that needs no device returns the documented codes."""
import ctypes
import os
import re

import pytest

from paper_2110_13005_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _header_symbols():
    text = open(os.path.join(ROOT, "include", "axonn_stage.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(axonn_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = B.load()
    syms = _header_symbols()
    assert len(syms) >= 30
    for s in syms:
        assert hasattr(lib, s), "missing export: " + s
    assert sorted(B.EXPORTED_SYMBOLS) == syms, "binding and header disagree"


def test_half_precision_build_exports_the_same_symbols():
    """libaxonn_stage_fp16.so is the same C ABI over the other 16-bit element type."""
    from paper_2110_13005_amd import build as BLD
    lib = ctypes.CDLL(BLD.LIB_PATH_FP16)
    for s in _header_symbols():
        assert hasattr(lib, s), "missing export: " + s
    lib.axonn_element_type.restype = ctypes.c_int32
    assert lib.axonn_element_type() == 1 and B.load().axonn_element_type() == 0


def test_binding_holds_both_builds_and_routes_by_selection():
    """select_elem() switches the library that handle-free calls go to, the torch dtype and the rounding of the
    synthetic inputs; both libraries stay loaded, and each keeps an error message of its own."""
    import numpy as np
    import torch
    from paper_2110_13005_amd import inputs
    before = B.ELEM
    try:
        B.select_elem("bf16")
        lib_b = B.load()
        assert B.axonn_element_type() == 0 and B.torch_elem_dtype() == torch.bfloat16
        x = np.float32(1.0 + 2.0 ** -10)
        assert inputs.snap_elem(np.array([x]))[0] == np.float32(1.0)            # bfloat16 keeps 8 bits
        B.select_elem("fp16")
        lib_h = B.load()
        assert lib_h is not lib_b and B.load("bf16") is lib_b
        assert B.axonn_element_type() == 1 and B.torch_elem_dtype() == torch.float16
        assert inputs.snap_elem(np.array([x]))[0] == x                          # half precision keeps 11
        with pytest.raises(B.AxonnError) as e:
            B.axonn_tuning(99, 0)
        assert e.value.status == B.AXONN_EINVAL and b"99" in lib_h.axonn_last_error()
        assert b"99" not in lib_b.axonn_last_error()
        with pytest.raises(ValueError):
            B.select_elem("fp8")
    finally:
        B.select_elem(before)


def test_argument_validation_without_device():
    lib = B.load()
    assert lib.axonn_stage_create(None, None) == B.AXONN_EINVAL
    assert b"null" in lib.axonn_last_error()
    out = ctypes.c_void_p()
    cfg = B.axonn_stage_config(2, 256, 3, 1024, 128, 2, 4, 4, 1e-5, 0, 1, 0, 0)   # 256 % 3 != 0
    assert lib.axonn_stage_create(ctypes.byref(cfg), ctypes.byref(out)) == B.AXONN_EINVAL
    cfg = B.axonn_stage_config(2, 2048, 8, 8192, 128, 2, 4, 4, 1e-5, 0, 1, 0, 0)  # head dim 256
    assert lib.axonn_stage_create(ctypes.byref(cfg), ctypes.byref(out)) == B.AXONN_EUNSUPPORTED
    assert b"head dim" in lib.axonn_last_error()
    cfg = B.axonn_stage_config(2, 256, 4, 1024, 128, 2, 4, 5, 1e-5, 0, 1, 0, 0)   # pipeline_limit > M
    assert lib.axonn_stage_create(ctypes.byref(cfg), ctypes.byref(out)) == B.AXONN_EINVAL
    cfg = B.axonn_stage_config(2, 256, 4, 1024, 3, 1, 4, 4, 1e-5, 0, 1, 0, 0)     # 3 tokens
    assert lib.axonn_stage_create(ctypes.byref(cfg), ctypes.byref(out)) == B.AXONN_EUNSUPPORTED
    cfg = B.axonn_stage_config(4, 256, 4, 1024, 128, 2, 4, 4, 1e-5, 0, 1, 0, 0, 3)  # stride 3, 4 layers
    assert lib.axonn_stage_create(ctypes.byref(cfg), ctypes.byref(out)) == B.AXONN_EINVAL
    assert b"ckpt_stride" in lib.axonn_last_error()
    with pytest.raises(B.AxonnError) as e:
        B.axonn_gemm_bf16(1, 0, 0, 64, 64, 60, 1, 64, 1, 64, 1, 64)          # K % 8 != 0
    assert e.value.status == B.AXONN_EUNSUPPORTED
    with pytest.raises(B.AxonnError) as e:
        B.axonn_gemm_bf16(0, 1, 0, 64, 64, 64, 1, 64, 1, 64, 1, 64)          # layout not built
    assert e.value.status == B.AXONN_EUNSUPPORTED
    with pytest.raises(B.AxonnError) as e:
        B.axonn_gemm_wgrad_colsum(3, 64, 64, 64, 1, 64, 1, 64, 1, 64, 1, 1)     # not an accumulating epilogue
    assert e.value.status == B.AXONN_EINVAL
    with pytest.raises(B.AxonnError) as e:
        B.axonn_gemm_wgrad_colsum(5, 64, 64, 64, 1, 64, 1, 64, 1, 64, None, 1)  # no place for the column sums
    assert e.value.status == B.AXONN_EINVAL
    with pytest.raises(B.AxonnError) as e:
        B.axonn_gemm_wgrad_colsum(5, 64, 64, 64, 1, 64, 1, 56, 1, 64, 1, 1)     # ldb < N
    assert e.value.status == B.AXONN_EINVAL
    with pytest.raises(B.AxonnError) as e:
        B.axonn_adam_bucket(8, 1, 1, 1, 1, 1, 1e-3, 0.9, 0.95, 1e-8, 0.0, 0, 1.0)  # step 0
    assert e.value.status == B.AXONN_EINVAL
    with pytest.raises(B.AxonnError) as e:
        B.axonn_attention_fwd(1, 128, 4, 200, 1, 1, 1)
    assert e.value.status == B.AXONN_EUNSUPPORTED
