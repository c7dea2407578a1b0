"""The optimizer step that starts during the tail of the batch's backward work (one-GPU counterpart of
Sec. 5.3): identical results to the plain step and to the oracle, for every chunk size and gradient mode."""
import ctypes

import numpy as np
import pytest

import oracle
from paper_2110_13005_amd import binding as B
from paper_2110_13005_amd.inputs import StageShape, make_stage_inputs
from paper_2110_13005_amd.stage import Stage
from helpers import rel_fro, dev_bf16, host

pytestmark = pytest.mark.gpu
HYPER = (1e-3, 0.9, 0.95, 1e-8, 0.01)


def _pinned(n):
    p = B.axonn_pinned_alloc(4 * n)
    return p, np.ctypeslib.as_array((ctypes.c_float * n).from_address(p))


def _two_batches(sh, layers, xs, dys, opts, chunk, bucket, n_streams=2):
    """Two batches with an optimizer step after each; chunk None: plain step after a join, else the
    overlapped step right after run().  Returns per batch (theta, m, v, params16, grads16)."""
    import torch
    M = sh.n_microbatches
    out = []
    with Stage(sh, **opts) as st:
        st.load_params(layers)
        n = st.n_params
        ptrs, arrs = zip(*[_pinned(n) for _ in range(3)])
        arrs[0][:] = st.params.float().cpu().numpy(); arrs[1][:] = 0; arrs[2][:] = 0
        B.axonn_stage_optimizer_attach(st.handle, ptrs[0], ptrs[1], ptrs[2], n, bucket)
        X = [dev_bf16(x) for x in xs]; DY = [dev_bf16(d) for d in dys]
        Y = [torch.zeros_like(X[0]) for _ in range(M)]; DX = [torch.zeros_like(X[0]) for _ in range(M)]
        for step in (1, 2):
            st.zero_grad()
            for i in range(M):
                st.post(0, i, X[i], Y[i])
            if chunk is not None:
                with pytest.raises(B.AxonnError) as e:     # nothing of the batch has run yet
                    B.axonn_stage_optimizer_step_overlapped(st.handle, *HYPER, step, 1.0 / M, chunk)
                assert e.value.status == B.AXONN_ESTATE
            for i in range(M):
                st.post(1, i, DY[i], DX[i])
            st.run(n_streams)
            if chunk is None:
                st.join()
                B.axonn_stage_optimizer_step(st.handle, *HYPER, step, 1.0 / M)
            else:
                B.axonn_stage_optimizer_step_overlapped(st.handle, *HYPER, step, 1.0 / M, chunk)
                st.join()
            torch.cuda.synchronize()
            out.append(tuple(a.copy() for a in arrs) + (host(st.params), host(st.grads)))
    for p in ptrs:
        B.axonn_pinned_free(p)
    return out


@pytest.mark.parametrize("opts", [dict(grad_accum_fp32=1, wgrad_group=0), dict(grad_accum_fp32=0, wgrad_group=2),
                                  dict(grad_accum_fp32=1, ckpt_stride=2), dict(grad_accum_fp32=0, ckpt_stride=1)],
                         ids=["fp32acc", "bf16acc-group2", "ckpt2-fp32acc", "ckpt1-bf16acc"])
def test_overlapped_step_equals_plain_step_and_oracle(opts):
    sh = StageShape(4, 256, 4, 128, 1, 5)
    layers, xs, dys = make_stage_inputs(sh, seed=7, perturb=True)
    bucket = 1 << 18          # 13 buckets, the last one ragged; layer boundaries fall inside buckets
    plain = _two_batches(sh, layers, xs, dys, opts, None, bucket)
    # oracle: Adam on the gradients the plain run produced, from the state before each step
    theta = np.concatenate([np.asarray(p[k], np.float32).ravel() for p in layers for k in oracle.PARAM_NAMES])
    m = np.zeros_like(theta); v = np.zeros_like(theta)
    for step, got in zip((1, 2), plain):
        theta, m, v, _ = oracle.adam_step(theta, m, v, got[4], *HYPER, step, 1.0 / sh.n_microbatches, half=B.ELEM)
        assert rel_fro(got[0], theta) <= 1e-6 and rel_fro(got[1], m) <= 1e-6 and rel_fro(got[2], v) <= 1e-6
        theta, m, v = (np.asarray(a, np.float32) for a in got[:3])      # continue from the GPU state
    for chunk, n_streams in ((1, 2), (3, 3), (1000, 2), (2, 1)):
        over = _two_batches(sh, layers, xs, dys, opts, chunk, bucket, n_streams=n_streams)
        for a, b in zip(plain, over):
            for x, y in zip(a[:4], b[:4]):
                assert np.array_equal(x, y), (opts, chunk, n_streams)


def test_overlapped_step_single_stream_and_direct_calls():
    """One library stream, and direct Forward/Backward calls on the null stream: every wait the step makes is
    then on work queued earlier in the same stream."""
    import torch
    sh = StageShape(2, 128, 2, 64, 2, 3)
    layers, xs, dys = make_stage_inputs(sh, seed=8, perturb=True)
    opts = dict(grad_accum_fp32=0, wgrad_group=0)
    a = _two_batches(sh, layers, xs, dys, opts, None, 1 << 16, n_streams=1)
    b = _two_batches(sh, layers, xs, dys, opts, 2, 1 << 16, n_streams=1)
    for p, q in zip(a, b):
        for x, y in zip(p, q):
            assert np.array_equal(x, y)
    M = sh.n_microbatches
    with Stage(sh, **opts) as st:
        st.load_params(layers)
        n = st.n_params
        ptrs, arrs = zip(*[_pinned(n) for _ in range(3)])
        arrs[0][:] = st.params.float().cpu().numpy(); arrs[1][:] = 0; arrs[2][:] = 0
        B.axonn_stage_optimizer_attach(st.handle, ptrs[0], ptrs[1], ptrs[2], n, 1 << 16)
        X = [dev_bf16(x) for x in xs]; DY = [dev_bf16(d) for d in dys]
        Y = [torch.zeros_like(X[0]) for _ in range(M)]; DX = [torch.zeros_like(X[0]) for _ in range(M)]
        st.zero_grad()
        for i in range(M):
            st.forward(i, X[i], Y[i])
        for i in range(M):
            if i == M - 1:
                with pytest.raises(B.AxonnError):
                    B.axonn_stage_optimizer_step_overlapped(st.handle, *HYPER, 1, 1.0 / M, 1)
            st.backward(i, DY[i], DX[i])
        B.axonn_stage_optimizer_step_overlapped(st.handle, *HYPER, 1, 1.0 / M, 1)
        torch.cuda.synchronize()
        for x, y in zip(a[0][:3], arrs):
            assert rel_fro(y, x) <= 1e-6          # same gradients up to the accumulation order of the schedule
    for p in ptrs:
        B.axonn_pinned_free(p)
