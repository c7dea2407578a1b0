"""The two builds of the library (bfloat16 and half precision, the paper's arithmetic: Sec. 2 "Mixed precision") in one
process.

The parity tests of the single operations, of the stage, of the pipeline's ends, of checkpointing and of loss scaling
run once per element type (the `axonn_elem` parametrization in conftest.py).  What is left for this file: stages of
both element types alive at the same time, their calls interleaved, each still giving its own library's result."""
import numpy as np
import pytest

import oracle
from paper_2110_13005_amd import binding as B
from paper_2110_13005_amd.inputs import StageShape, make_stage_inputs
from paper_2110_13005_amd.stage import Stage
from helpers import dev_bf16, host, check_batch, EPS

pytestmark = pytest.mark.gpu


def test_stages_of_both_element_types_side_by_side():
    import torch
    sh = StageShape(2, 256, 4, 128, 2, 2)
    M = sh.n_microbatches
    before = B.ELEM
    made = {}
    try:
        for elem in ("bf16", "fp16"):
            B.select_elem(elem)
            layers, xs, dys = make_stage_inputs(sh, seed=11, perturb=True)          # rounded to `elem`
            st = Stage(sh)
            st.load_params(layers)
            X = [dev_bf16(x) for x in xs]
            DY = [dev_bf16(d) for d in dys]
            Y = [torch.zeros_like(X[0]) for _ in range(M)]
            DX = [torch.zeros_like(X[0]) for _ in range(M)]
            ref = oracle.stage_batch(xs, dys, layers, sh.n_heads, EPS)
            made[elem] = (st, X, DY, Y, DX, ref)
            assert B.axonn_element_type() == (1 if elem == "fp16" else 0)
        assert made["bf16"][0].params.dtype == torch.bfloat16 and made["fp16"][0].params.dtype == torch.float16
        # both batches with their calls interleaved, whichever type is selected: a handle goes to the library
        # that created it
        for pick, (st, *_rest) in zip(("fp16", "bf16"), made.values()):
            B.select_elem(pick)
            st.zero_grad()
        for i in range(M):
            for elem in ("bf16", "fp16"):
                B.select_elem("fp16" if (i + (elem == "fp16")) % 2 else "bf16")
                st, X, DY, Y, DX, _ = made[elem]
                st.forward(i, X[i], Y[i])
        for i in range(M):
            for elem in ("fp16", "bf16"):
                B.select_elem("bf16" if (i + (elem == "fp16")) % 2 else "fp16")
                st, X, DY, Y, DX, _ = made[elem]
                st.backward(i, DY[i], DX[i])
        torch.cuda.synchronize()
        for elem in ("bf16", "fp16"):
            st, X, DY, Y, DX, ref = made[elem]
            check_batch([host(y) for y in Y], [host(d) for d in DX], st.grads_numpy(), ref)
    finally:
        for st, *_ in made.values():
            st.close()
        B.select_elem(before)
