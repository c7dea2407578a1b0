"""Builds the shared library in-tree with hipcc for gfx950 (cross-compiles without a GPU), twice from the same
sources: libaxonn_stage.so with bfloat16 as the 16-bit element type, libaxonn_stage_fp16.so with IEEE half.

    python -m paper_2110_13005_amd.build
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB_PATH = os.path.join(HERE, "libaxonn_stage.so")
LIB_PATH_FP16 = os.path.join(HERE, "libaxonn_stage_fp16.so")
VARIANTS = {"bf16": (LIB_PATH, []), "fp16": (LIB_PATH_FP16, ["-DAXONN_ELEM_FP16"])}
SOURCES = ["gemm.hip", "attention.hip", "elementwise.hip", "lm_ends.hip", "stage.cpp"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function",
         # the GEMM main loops are written as fully unrolled loops over compile-time schedules (`#pragma unroll`):
         # left partly rolled, their fragment arrays would live in scratch memory instead of registers
         "-mllvm", "-pragma-unroll-threshold=100000"]


def _compile(job):
    variant, src = job
    obj = os.path.join(OBJ_DIR, variant, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC, *FLAGS, *VARIANTS[variant][1], "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s (%s):\n%s" % (src, variant, err))
    if err.strip():
        sys.stderr.write(err + "\n")
    return variant, obj


def build(verbose=True, variants=("bf16", "fp16")):
    """Compiles every source (always: no staleness check) and links the shared libraries."""
    for v in variants:
        os.makedirs(os.path.join(OBJ_DIR, v), exist_ok=True)
    jobs = [(v, s) for s in SOURCES for v in variants]       # the long compilations (gemm.hip) first
    with ThreadPoolExecutor(max_workers=6) as ex:
        done = list(ex.map(_compile, jobs))
    for v in variants:
        lib = VARIANTS[v][0]
        objs = [o for (vv, o) in done if vv == v]
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stderr)
        if verbose:
            print("built", lib)
    return LIB_PATH


if __name__ == "__main__":
    build(variants=tuple(sys.argv[1:]) or ("bf16", "fp16"))
