"""Parity at the full benchmark sizes (12B-, 24B- and 100B-class stage shapes, and the
1.6e9-parameter offloaded optimizer step), in the launch configuration bench.py times: all
microbatches in flight, message-driven run on two library streams.

The fp64 oracle is too slow for a whole batch at these sizes, so it computes microbatch 0 only:
  * its stage output and input gradient are compared in full (per-microbatch tensors do not depend
    on the other microbatches);
  * the parameter gradients of a batch that holds microbatch 0 alone are compared in full;
  * the full batch is tied to that by linearity, a property that holds at any size: the gradients
    of the M-microbatch run equal the sum of the gradients of single-microbatch runs (checked on
    sampled tensors against two further single-microbatch GPU runs where M allows).
Bounds: the benchmark definition's (2e-2 forward, 3e-2 gradients, 1e-6 Adam master state)."""
import sys
import time

import numpy as np
import pytest

import oracle
from paper_2110_13005_amd import binding as B
from paper_2110_13005_amd.inputs import CONFIGS, OPT_CONFIG, QKV_INPUT_SPLIT, StageShape, make_stage_inputs
from paper_2110_13005_amd.stage import Stage
from helpers import rel_fro, elem_factor, dev_bf16, host

pytestmark = pytest.mark.gpu
EPS = 1e-5


def _say(msg):
    print("[fullsize] " + msg, flush=True)
    sys.stdout.flush()


# Element-wise bound of the full-size stage outputs, in 16-bit roundings (helpers.elem_factor): an output element is
# a sum over the 4 (2) layers of residual-branch terms, each the product of a rounded activation row with a weight
# column plus the roundings of five stored tensors per layer; with the relative Frobenius errors measured (6e-3 to
# 2.8e-2, i.e. 1.5 to 7 roundings of the typical element on average) the worst of 10^7 to 10^8 elements lies 5 to 6
# standard deviations out (measured: 7 to 11 forward, 14 to 28 for dx).
FULL_SIZE_ELEM_C = 48.0


def _message_run(st, X, DY, Y, DX, n_streams=2):
    import torch
    M = len(X)
    st.zero_grad()
    for i in range(M):
        st.post(0, i, X[i], Y[i])
    for i in range(M):
        st.post(1, i, DY[i], DX[i])
    st.run(n_streams)
    st.join()
    torch.cuda.synchronize()


@pytest.mark.parametrize("name,ac", [("12b", 0), ("24b", 0), ("100b", 0), ("12b", 2), ("table1_12b", 0)])
def test_full_size_stage_parity(name, ac):
    """ac > 0: the same with activation checkpointing of that stride (Sec. 5.1), against the oracle's
    regenerating pass."""
    import torch
    sh = CONFIGS[name]
    if name == "table1_12b":
        # the paper's own shape (head dim 188, sequence 512, microbatch 8): 4 of the stage's 8 layers and 6 of the
        # microbatches keep the oracle's share of the test near half a minute
        sh = StageShape(4, sh.hidden, sh.n_heads, sh.seq_len, sh.microbatch_size, 6)
    M = sh.n_microbatches
    t0 = time.time()
    _say("%s: generating inputs (seed 0)" % name)
    # the recipe draws all M microbatches; only microbatch 0's values are needed on the host
    layers, xs, dys = make_stage_inputs(sh, seed=0, n_microbatches=1)
    rng = np.random.default_rng(1)
    # bench.py's launch configuration (bf16 gradient accumulation, weight gradients in groups of 3);
    # the 100B shape additionally takes the split-input QKV projection: with h = 10240 and N(0, 0.02)
    # weights the attention logits have standard deviation 4 and the peaked softmax amplifies the bf16
    # rounding of LayerNorm's output about sixfold (without it the worst gradient error is 3.4e-2)
    opts = dict(grad_accum_fp32=0, wgrad_group=3, qkv_input_split=QKV_INPUT_SPLIT.get(name, 0), ckpt_stride=ac)
    name = name if not ac else "%s/ac=%d" % (name, ac)
    with Stage(sh, **opts) as st:
        st.load_params(layers)
        bsh = (sh.microbatch_size, sh.seq_len, sh.hidden)
        X = [dev_bf16(xs[0])] + [torch.randn(bsh, device="cuda").to(B.torch_elem_dtype()) for _ in range(M - 1)]
        DY = [dev_bf16(dys[0])] + [torch.randn(bsh, device="cuda").to(B.torch_elem_dtype()) for _ in range(M - 1)]
        Y = [torch.zeros_like(X[0]) for _ in range(M)]
        DX = [torch.zeros_like(X[0]) for _ in range(M)]
        _say("%s: GPU batch of %d microbatches, message-driven, 2 streams" % (name, M))
        _message_run(st, X, DY, Y, DX)
        y0, dx0 = host(Y[0]), host(DX[0])
        y_last, dx_last = host(Y[M - 1]), host(DX[M - 1])
        x_last = X[M - 1].float().cpu().numpy().reshape(xs[0].shape)
        dy_last = DY[M - 1].float().cpu().numpy().reshape(dys[0].shape)
        # sampled parameter-gradient tensors of the full batch, for the linearity check
        names = ["layer0.w_qkv", "layer%d.w_fc2" % (sh.n_layers - 1), "layer0.ln1_g", "layer%d.b_fc1" % (sh.n_layers - 1)]
        full = {n: st.tensor(n, grad=True).double().clone() for n in names}
    # single-microbatch batches on a stage with one slot
    one = StageShape(sh.n_layers, sh.hidden, sh.n_heads, sh.seq_len, sh.microbatch_size, 1, sh.ffn_hidden)
    with Stage(one, **opts) as s1:
        s1.load_params(layers)
        acc = {n: 0.0 for n in names}
        g0 = None
        Yt, DXt = torch.zeros_like(X[0]), torch.zeros_like(X[0])
        for i in range(M):
            _message_run(s1, [X[i]], [DY[i]], [Yt], [DXt], n_streams=1)
            for n in names:
                acc[n] = acc[n] + s1.tensor(n, grad=True).double()
            if i == 0:
                g0 = s1.grads_numpy()
                assert torch.equal(Yt, Y[0]) and torch.equal(DXt, DX[0])   # same kernels, same bits
    for n in names:
        e = float((full[n] - acc[n]).norm() / acc[n].norm())
        _say("%s: linearity %s rel err %.2e" % (name, n, e))
        assert e <= 1e-2, (n, e)       # M roundings of bf16 single-batch gradients vs one rounding
    _say("%s: oracle on microbatch 0 (fp64, host) ..." % name)
    t1 = time.time()
    if ac:
        from oracle import transformer as OT
        l64 = [{k: np.asarray(v, np.float64) for k, v in p.items()} for p in layers]
        z, kept = OT.stage_forward_checkpointed(xs[0], l64, sh.n_heads, EPS, ac)
        dx, ref_g = OT.stage_backward_checkpointed(dys[0], kept, l64, sh.n_heads, EPS, ac)
        ref_out, ref_dx = [z], [dx]
    else:
        ref_out, ref_dx, ref_g = oracle.stage_batch(xs, dys, layers, sh.n_heads, EPS)
    _say("%s: oracle took %.0f s" % (name, time.time() - t1))
    e_f = rel_fro(y0.reshape(ref_out[0].shape), ref_out[0])
    e_b = rel_fro(dx0.reshape(ref_dx[0].shape), ref_dx[0])
    worst, worst_name = 0.0, ""
    for li, g in enumerate(g0):
        for k, v in g.items():
            e = rel_fro(v, ref_g[li][k])
            if e > worst:
                worst, worst_name = e, "layer%d.%s" % (li, k)
    # element-wise, in 16-bit roundings of an element's own size plus its row's typical size (helpers.elem_factor)
    f_f = elem_factor(y0.reshape(ref_out[0].shape), ref_out[0])
    f_b = elem_factor(dx0.reshape(ref_dx[0].shape), ref_dx[0])
    _say("%s: forward %.3e  dx %.3e  worst grad %.3e (%s)  element factors %.1f / %.1f  total %.0f s"
         % (name, e_f, e_b, worst, worst_name, f_f, f_b, time.time() - t0))
    assert e_f <= 2e-2 and e_b <= 3e-2 and worst <= 3e-2
    assert f_f <= FULL_SIZE_ELEM_C and f_b <= FULL_SIZE_ELEM_C, (f_f, f_b)
    if not ac:
        # the batch's last microbatch (device-drawn N(0,1) values, read back) against the oracle as well: the first
        # and the last slot, the first and the last message of the run
        t1 = time.time()
        if B.ELEM == "fp16":
            x_last, dy_last = x_last.astype(np.float32), dy_last.astype(np.float32)
        o2, d2, _ = oracle.stage_batch([x_last], [dy_last], layers, sh.n_heads, EPS)
        e_f2 = rel_fro(y_last.reshape(o2[0].shape), o2[0])
        e_b2 = rel_fro(dx_last.reshape(d2[0].shape), d2[0])
        f_f2 = elem_factor(y_last.reshape(o2[0].shape), o2[0])
        f_b2 = elem_factor(dx_last.reshape(d2[0].shape), d2[0])
        _say("%s: last microbatch forward %.3e  dx %.3e  element factors %.1f / %.1f  (oracle %.0f s)"
             % (name, e_f2, e_b2, f_f2, f_b2, time.time() - t1))
        assert e_f2 <= 2e-2 and e_b2 <= 3e-2
        assert f_f2 <= FULL_SIZE_ELEM_C and f_b2 <= FULL_SIZE_ELEM_C, (f_f2, f_b2)


def test_full_size_last_stage_head():
    """The last stage's extras at the 12B shape and the paper's vocabulary (Sec. 6.1): T = 2048 tokens,
    h = 5120, V = 51200, 8 microbatches in the pre-division.  The oracle computes the whole microbatch; the
    5120 x 51200 head gradient is compared on sampled column blocks (first, last, seeded random) and in norm."""
    import torch
    from oracle import lm_ends as OE
    T, h, V, M = 2048, 5120, 51200, 8
    rng = np.random.default_rng(0)
    _say("head: generating inputs")
    from paper_2110_13005_amd.inputs import snap_elem
    from paper_2110_13005_amd.stage import view_bf16
    x = snap_elem(rng.standard_normal((1, T, h), dtype=np.float32))
    W = snap_elem(rng.standard_normal((h, V), dtype=np.float32) * np.float32(0.02))
    g = snap_elem((1 + 0.02 * rng.standard_normal(h)).astype(np.float32))
    bt = snap_elem((0.02 * rng.standard_normal(h)).astype(np.float32))
    tg = rng.integers(0, V, (1, T))
    hd = B.axonn_head_create(0, V, h, T, M, EPS)
    try:
        p, gr, n = B.axonn_head_buffers(hd)
        params, grads = view_bf16(p, n), view_bf16(gr, n)
        params[:h] = dev_bf16(g); params[h:2 * h] = dev_bf16(bt); params[2 * h:] = dev_bf16(W).reshape(-1)
        loss = torch.zeros(1, device="cuda"); dx = torch.zeros(T, h, dtype=B.torch_elem_dtype(), device="cuda")
        X = dev_bf16(x); TG = torch.from_numpy(tg.astype(np.int32)).cuda()
        _say("head: GPU forward + loss + backward")
        B.axonn_head_forward_backward(hd, X, TG, loss, dx)
        torch.cuda.synchronize()
        _say("head: oracle (fp64, host) ...")
        t1 = time.time()
        rl, c = OE.head_loss_forward(x, g, bt, W, tg, EPS, M)
        rdx, rg = OE.head_loss_backward(c, g, W, tg, M)
        _say("head: oracle took %.0f s" % (time.time() - t1))
        e_l = abs(loss.item() - rl) / abs(rl)
        e_dx = rel_fro(host(dx).reshape(rdx.shape), rdx)
        gW = grads[2 * h:].view(h, V)
        cols = [0, V - 512] + [int(c0) for c0 in rng.integers(0, V // 512 - 1, 6) * 512]
        e_w = max(rel_fro(host(gW[:, c0:c0 + 512]), rg["w_head"][:, c0:c0 + 512]) for c0 in cols)
        e_norm = abs(float(gW.float().norm()) - np.linalg.norm(rg["w_head"])) / np.linalg.norm(rg["w_head"])
        e_g = max(rel_fro(host(grads[:h]), rg["lnf_g"]), rel_fro(host(grads[h:2 * h]), rg["lnf_b"]))
        _say("head: loss %.5f (oracle %.5f, rel %.1e)  dx %.2e  dW blocks %.2e  |dW| %.1e  LN grads %.2e"
             % (loss.item(), rl, e_l, e_dx, e_w, e_norm, e_g))
        assert e_l <= 2e-3 and e_dx <= 3e-2 and e_w <= 3e-2 and e_norm <= 1e-2 and e_g <= 3e-2
    finally:
        params = grads = None
        B.axonn_head_destroy(hd)


def test_full_size_offloaded_adam():
    """Config 5: 1.6e9 parameters, 2^26-element buckets (24, last one ragged), mid-training
    state, lr 1e-4, betas (0.9, 0.95), eps 1e-8, step 100.  The oracle is evaluated on sampled
    index ranges: the first and last elements, every bucket boundary and seeded random blocks."""
    import ctypes
    import torch
    oc = OPT_CONFIG
    n, bucket = oc["n"], oc["bucket_elems"]
    _say("adam: allocating 3 x %.1f GB pinned" % (4 * n / 1e9))
    ptrs = [B.axonn_pinned_alloc(4 * n) for _ in range(3)]
    arrs = [np.ctypeslib.as_array((ctypes.c_float * n).from_address(p)) for p in ptrs]
    g = torch.Generator(device="cuda"); g.manual_seed(0)
    G16 = torch.empty(n, dtype=B.torch_elem_dtype(), device="cuda")
    P16 = torch.zeros(n, dtype=B.torch_elem_dtype(), device="cuda")
    step = 1 << 26
    for o in range(0, n, step):
        c = min(step, n - o)
        torch.from_numpy(arrs[0][o:o + c]).copy_(torch.randn(c, generator=g, device="cuda") * 0.02)
        torch.from_numpy(arrs[1][o:o + c]).copy_(torch.randn(c, generator=g, device="cuda") * 1e-4)
        torch.from_numpy(arrs[2][o:o + c]).copy_((torch.randn(c, generator=g, device="cuda") * 1e-6).abs())
        G16[o:o + c] = (torch.randn(c, generator=g, device="cuda") * 1e-3).to(B.torch_elem_dtype())
    torch.cuda.synchronize()
    # sampled ranges, inputs copied out before the step overwrites them
    rng = np.random.default_rng(0)
    starts = [0, n - 4096] + [b * bucket - 2048 for b in range(1, (n + bucket - 1) // bucket)]
    starts += [int(s) for s in rng.integers(0, n - 4096, size=40)]
    sample = [(s, s + 4096) for s in starts]
    before = [(arrs[0][a:b].copy(), arrs[1][a:b].copy(), arrs[2][a:b].copy(), G16[a:b].float().cpu().numpy()) for a, b in sample]
    opt = B.axonn_offload_adam_create(0, n, bucket, P16, G16, ptrs[0], ptrs[1], ptrs[2])
    try:
        assert B.axonn_offload_adam_device_bytes(opt) == 3 * 12 * bucket     # footprint independent of n
        _say("adam: step over %d buckets" % ((n + bucket - 1) // bucket))
        t0 = time.time()
        B.axonn_offload_adam_step(opt, oc["lr"], oc["beta1"], oc["beta2"], oc["eps"], oc["weight_decay"], oc["step"], oc["grad_scale"])
        torch.cuda.synchronize()
        _say("adam: step took %.3f s" % (time.time() - t0))
        worst = 0.0
        for (a, b), (th, m, v, g16) in zip(sample, before):
            rt, rm, rv, r16 = oracle.adam_step(th, m, v, g16, oc["lr"], oc["beta1"], oc["beta2"], oc["eps"], oc["weight_decay"], oc["step"], oc["grad_scale"], half=B.ELEM)
            worst = max(worst, rel_fro(arrs[0][a:b], rt), rel_fro(arrs[1][a:b], rm), rel_fro(arrs[2][a:b], rv))
            got16 = P16[a:b].float().cpu().numpy()
            assert np.array_equal(got16, oracle.half_round(arrs[0][a:b], B.ELEM))
            assert np.abs(got16 - r16).max() <= np.abs(r16).max() * 2.0 ** -7
        _say("adam: worst relative error %.2e" % worst)
        assert worst <= 1e-6
        # everything was touched exactly once: bf16 parameters are the rounding of the master copy
        for o in range(0, n, step):
            c = min(step, n - o)
            assert torch.equal(P16[o:o + c].cpu(), torch.from_numpy(arrs[0][o:o + c]).to(B.torch_elem_dtype()))
    finally:
        B.axonn_offload_adam_destroy(opt)
        for p in ptrs:
            B.axonn_pinned_free(p)
