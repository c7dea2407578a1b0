"""GPU parity of the pipeline's two ends (Alg. 2's special cases: token + position embedding in front; final
LayerNorm, LM head and the pre-divided cross-entropy behind, Sec. 4.2) against the fp64 oracle, through the
C ABI: the single operations, and stages that are the first, the last, or both."""
import numpy as np
import pytest

from oracle import lm_ends as OE
from oracle import transformer as OT
from paper_2110_13005_amd import binding as B
from paper_2110_13005_amd.inputs import StageShape, make_stage_inputs, make_lm_inputs, snap_elem
from paper_2110_13005_amd.stage import Stage, view_bf16
from helpers import rel_fro, dev_bf16, host, dev_i32, EmbedHandle, HeadHandle, oracle_model, FWD_TOL, GRAD_TOL, EPS

pytestmark = pytest.mark.gpu


def test_embedding_forward_backward_with_repeated_and_out_of_range_ids():
    import torch
    rng = np.random.default_rng(0)
    V, h, s, b = 40, 136, 24, 3                    # few rows: many repeats; 136 columns: a ragged vector tail
    wte, wpe = snap_elem(rng.standard_normal((V, h), dtype=np.float32)), snap_elem(rng.standard_normal((s, h), dtype=np.float32))
    e = EmbedHandle(V, h, s, b, wte, wpe)
    try:
        tot_te, tot_pe = 0.0, 0.0
        for it in range(3):
            tokens = rng.integers(0, V, (b, s))
            if it == 1:
                tokens[0, 0], tokens[1, 3], tokens[2, 5] = -7, V, V + 1000      # clamped to 0, V-1, V-1
            clamped = np.clip(tokens, 0, V - 1)
            x = torch.zeros(b, s, h, dtype=B.torch_elem_dtype(), device="cuda")
            B.axonn_embed_forward(e.h, dev_i32(tokens), x)
            ref = OE.embedding_forward(clamped, wte, wpe)
            assert rel_fro(host(x), ref) <= 4e-3                               # one bf16 rounding of the sum
            dx = snap_elem(rng.standard_normal((b, s, h), dtype=np.float32))
            B.axonn_embed_backward(e.h, dev_i32(tokens), dev_bf16(dx))
            torch.cuda.synchronize()
            dte, dpe = OE.embedding_backward(dx, clamped, V, s)
            tot_te, tot_pe = tot_te + dte, tot_pe + dpe
            gte, gpe = e.grads_numpy()
            assert rel_fro(gte, tot_te) <= 6e-3 and rel_fro(gpe, tot_pe) <= 6e-3
            unused = np.setdiff1d(np.arange(V), clamped.ravel())
            if it == 0 and len(unused):
                assert not gte[unused].any()                                   # rows nobody used stay exactly zero
        B.axonn_embed_zero_grad(e.h)                                           # the next pass overwrites
        tokens = rng.integers(0, V, (b, s)); dx = snap_elem(rng.standard_normal((b, s, h), dtype=np.float32))
        B.axonn_embed_backward(e.h, dev_i32(tokens), dev_bf16(dx))
        torch.cuda.synchronize()
        dte, dpe = OE.embedding_backward(dx, tokens, V, s)
        gte, gpe = e.grads_numpy()
        assert rel_fro(gte, dte) <= 4e-3 and rel_fro(gpe, dpe) <= 4e-3
    finally:
        e.close()


@pytest.mark.parametrize("T,h,V,M", [(256, 192, 1000, 2), (72, 64, 264, 3), (2056, 256, 4104, 1)])
def test_head_loss_and_backward(T, h, V, M):
    """Several row tiles and ragged tails in every dimension; gradients accumulate over M microbatches."""
    import torch
    rng = np.random.default_rng(T)
    g = snap_elem((1 + 0.1 * rng.standard_normal(h)).astype(np.float32)); bt = snap_elem((0.1 * rng.standard_normal(h)).astype(np.float32))
    W = snap_elem((0.05 * rng.standard_normal((h, V))).astype(np.float32))
    hd = HeadHandle(V, h, T, M, g, bt, W)
    try:
        tot = None
        for it in range(M):
            x = snap_elem(rng.standard_normal((1, T, h), dtype=np.float32)); tg = rng.integers(0, V, (1, T))
            loss = torch.zeros(1, device="cuda"); dx = torch.zeros(T, h, dtype=B.torch_elem_dtype(), device="cuda")
            B.axonn_head_forward_backward(hd.h, dev_bf16(x), dev_i32(tg), loss, dx)
            torch.cuda.synchronize()
            rl, c = OE.head_loss_forward(x, g, bt, W, tg, EPS, M)
            rdx, rg = OE.head_loss_backward(c, g, W, tg, M)
            assert abs(loss.item() - rl) <= 2e-3 * abs(rl), (loss.item(), rl)
            assert rel_fro(host(dx).reshape(rdx.shape), rdx) <= GRAD_TOL
            tot = rg if tot is None else {k: tot[k] + rg[k] for k in rg}
            got = hd.grads_numpy()
            for k in tot:
                assert rel_fro(got[k], tot[k]) <= GRAD_TOL, (k, it)
    finally:
        hd.close()


@pytest.mark.parametrize("n_streams,ckpt", [(1, 0), (2, 0), (3, 2)])
def test_whole_model_on_one_stage_message_driven(n_streams, ckpt):
    """A stage that is both the first and the last one: token messages in, losses out, every gradient against the
    oracle's plain embedding -> layers -> head -> loss chain."""
    import torch
    sh = StageShape(2, 128, 2, 64, 2, 4)
    V = 520
    layers, _, _ = make_stage_inputs(sh, seed=11, perturb=True)
    tokens, targets, wte, wpe, g, bt, W = make_lm_inputs(sh, V, seed=12)
    ref_losses, ref = oracle_model(tokens, targets, wte, wpe, layers, g, bt, W, sh.n_heads, sh.n_microbatches)
    M = sh.n_microbatches
    e = EmbedHandle(V, sh.hidden, sh.seq_len, sh.microbatch_size, wte, wpe)
    hd = HeadHandle(V, sh.hidden, sh.tokens, M, g, bt, W)
    try:
        with Stage(sh, pipeline_limit=2, ckpt_stride=ckpt) as st:
            st.load_params(layers)
            B.axonn_stage_attach_ends(st.handle, e.h, hd.h)
            TK = [dev_i32(t) for t in tokens]; TG = [dev_i32(t) for t in targets]
            losses = torch.zeros(M, device="cuda")
            for rep in range(2):        # the second batch must start from cleared accumulators at both ends
                st.zero_grad()
                with pytest.raises(B.AxonnError):
                    st.post(1, 0, TK[0], None)                       # a last stage takes no backward messages
                for i in range(M):
                    st.post(0, i, TK[i], None, targets=TG[i], loss=losses[i:i + 1])
                st.run(n_streams)
                st.join()
                torch.cuda.synchronize()
                for i in range(M):
                    assert abs(losses[i].item() - ref_losses[i]) <= 2e-3 * abs(ref_losses[i])
                for li, gl in enumerate(st.grads_numpy()):
                    for k, v in gl.items():
                        assert rel_fro(v, ref["layers"][li][k]) <= GRAD_TOL, (li, k)
                got = hd.grads_numpy()
                for k in got:
                    assert rel_fro(got[k], ref["head"][k]) <= GRAD_TOL, k
                gte, gpe = e.grads_numpy()
                assert rel_fro(gte, ref["wte"]) <= GRAD_TOL and rel_fro(gpe, ref["wpe"]) <= GRAD_TOL
            with pytest.raises(B.AxonnError):
                st.forward(0, TK[0], TK[0])                          # direct calls are refused with ends attached
    finally:
        e.close(); hd.close()


def test_first_stage_and_last_stage_separately():
    """The two special cases of Alg. 2 one at a time: a first stage (tokens in, activations out; gradients in,
    nothing out) and a last stage (activations in, loss and input gradient out at once)."""
    import torch
    sh = StageShape(2, 128, 2, 64, 1, 3)
    V, M = 264, 3
    layers, xs, dys = make_stage_inputs(sh, seed=13, perturb=True)
    tokens, targets, wte, wpe, g, bt, W = make_lm_inputs(sh, V, seed=14)
    l64 = [{k: np.asarray(v, np.float64) for k, v in p.items()} for p in layers]
    # first stage
    e = EmbedHandle(V, sh.hidden, sh.seq_len, sh.microbatch_size, wte, wpe)
    try:
        with Stage(sh) as st:
            st.load_params(layers)
            B.axonn_stage_attach_ends(st.handle, e.h, None)
            Y = [torch.zeros(sh.microbatch_size, sh.seq_len, sh.hidden, dtype=B.torch_elem_dtype(), device="cuda") for _ in range(M)]
            TK = [dev_i32(t) for t in tokens]; DY = [dev_bf16(d) for d in dys]
            st.zero_grad()
            for i in range(M):
                st.post(0, i, TK[i], Y[i])
            for i in range(M):
                st.post(1, i, DY[i], None)
            st.run(2); st.join(); torch.cuda.synchronize()
            tot_te = 0.0
            for i in range(M):
                z, caches = OT.stage_forward(OE.embedding_forward(tokens[i], wte, wpe), l64, sh.n_heads, EPS)
                assert rel_fro(host(Y[i]).reshape(z.shape), z) <= FWD_TOL
                dx, _ = OT.stage_backward(dys[i], caches, l64, sh.n_heads)
                tot_te = tot_te + OE.embedding_backward(dx, tokens[i], V, sh.seq_len)[0]
            assert rel_fro(e.grads_numpy()[0], tot_te) <= GRAD_TOL
    finally:
        e.close()
    # last stage
    hd = HeadHandle(V, sh.hidden, sh.tokens, M, g, bt, W)
    try:
        with Stage(sh) as st:
            st.load_params(layers)
            B.axonn_stage_attach_ends(st.handle, None, hd.h)
            X = [dev_bf16(x) for x in xs]
            DX = [torch.zeros_like(X[0]) for _ in range(M)]
            TG = [dev_i32(t) for t in targets]
            losses = torch.zeros(M, device="cuda")
            st.zero_grad()
            with pytest.raises(B.AxonnError):
                st.post(0, 0, X[0], DX[0])                           # targets and loss are required
            for i in range(M):
                st.post(0, i, X[i], DX[i], targets=TG[i], loss=losses[i:i + 1])
            st.run(2); st.join(); torch.cuda.synchronize()
            log = B.axonn_stage_dispatch_log(st.handle)
            assert log == [(i, k) for i in range(M) for k in (0, 1)]      # Backward follows each Forward at once
            for i in range(M):
                z, caches = OT.stage_forward(xs[i], l64, sh.n_heads, EPS)
                loss, c = OE.head_loss_forward(z, g, bt, W, targets[i], EPS, M)
                dz, _ = OE.head_loss_backward(c, g, W, targets[i], M)
                dx, _ = OT.stage_backward(dz, caches, l64, sh.n_heads)
                assert abs(losses[i].item() - loss) <= 2e-3 * abs(loss)
                assert rel_fro(host(DX[i]).reshape(dx.shape), dx) <= GRAD_TOL
    finally:
        hd.close()
