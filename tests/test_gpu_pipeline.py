"""Alg. 2 end to end on one GPU: a first stage (embedding + the first half of the layers) and a last stage (the
second half + head and loss) as two stage objects that only talk through messages -- device buffers plus
"done" events, as neighbouring GPUs would -- served in turn by one host thread with the non-blocking receive
loop.  Everything is checked against the oracle's plain embedding -> layers -> head -> loss chain."""
import numpy as np
import pytest

from paper_2110_13005_amd import binding as B
from paper_2110_13005_amd.inputs import StageShape, make_stage_inputs, make_lm_inputs
from paper_2110_13005_amd.stage import Stage
from helpers import rel_fro, EmbedHandle, HeadHandle, dev_i32, oracle_model, GRAD_TOL

pytestmark = pytest.mark.gpu


def _event():
    import torch
    e = torch.cuda.Event()
    e.record()            # torch creates the underlying event at the first record; the library records it again
    return e


@pytest.mark.parametrize("n_streams,limit_a", [(2, 2), (1, 1), (3, 4)])
def test_two_stage_pipeline_message_driven(n_streams, limit_a):
    import torch
    whole = StageShape(4, 128, 2, 64, 2, 6)
    half = StageShape(2, whole.hidden, whole.n_heads, whole.seq_len, whole.microbatch_size, whole.n_microbatches)
    V, M = 520, whole.n_microbatches
    layers, _, _ = make_stage_inputs(whole, seed=21, perturb=True)
    tokens, targets, wte, wpe, g, bt, W = make_lm_inputs(whole, V, seed=22)
    ref_losses, ref = oracle_model(tokens, targets, wte, wpe, layers, g, bt, W, whole.n_heads, M)
    e = EmbedHandle(V, whole.hidden, whole.seq_len, whole.microbatch_size, wte, wpe)
    hd = HeadHandle(V, whole.hidden, whole.tokens, M, g, bt, W)
    try:
        with Stage(half, pipeline_limit=limit_a) as A, Stage(half, pipeline_limit=2) as Bst:
            A.load_params(layers[:2]); Bst.load_params(layers[2:])
            B.axonn_stage_attach_ends(A.handle, e.h, None)
            B.axonn_stage_attach_ends(Bst.handle, None, hd.h)
            bsh = (whole.microbatch_size, whole.seq_len, whole.hidden)
            TK = [dev_i32(t) for t in tokens]; TG = [dev_i32(t) for t in targets]
            ACT = [torch.zeros(bsh, dtype=B.torch_elem_dtype(), device="cuda") for _ in range(M)]    # A -> B
            GRD = [torch.zeros(bsh, dtype=B.torch_elem_dtype(), device="cuda") for _ in range(M)]    # B -> A
            sent = [_event() for _ in range(M)]; back = [_event() for _ in range(M)]
            losses = torch.zeros(M, device="cuda")
            torch.cuda.synchronize()
            for rep in range(2):
                A.zero_grad(); Bst.zero_grad()
                for i in range(M):      # the first stage's microbatch queue: admission is limited by pipeline_limit
                    A.post(0, i, TK[i], ACT[i], done_event=sent[i])
                seen_a = seen_b = 0
                rem_a = rem_b = 2 * M
                spins = 0
                while rem_a or rem_b:
                    _, rem_a = A.poll(n_streams)
                    log = B.axonn_stage_dispatch_log(A.handle)
                    for mb, kind in log[seen_a:]:
                        if kind == 0:   # Send(output, next stage)
                            Bst.post(0, mb, ACT[mb], GRD[mb], ready_event=sent[mb], targets=TG[mb],
                                     loss=losses[mb:mb + 1], done_event=back[mb])
                    seen_a = len(log)
                    _, rem_b = Bst.poll(n_streams)
                    log = B.axonn_stage_dispatch_log(Bst.handle)
                    for mb, kind in log[seen_b:]:
                        if kind == 1:   # Send(output, previous stage)
                            A.post(1, mb, GRD[mb], None, ready_event=back[mb])
                    seen_b = len(log)
                    spins += 1
                    assert spins < 2_000_000, "the pipeline made no progress"
                A.join(); Bst.join()
                torch.cuda.synchronize()
                # the first stage never has more than pipeline_limit microbatches in flight, and reaches it
                live, peak = set(), 0
                for mb, kind in B.axonn_stage_dispatch_log(A.handle):
                    live.add(mb) if kind == 0 else live.remove(mb)
                    peak = max(peak, len(live))
                assert peak == min(limit_a, M)
                # the last stage runs Backward right after each Forward
                lb = B.axonn_stage_dispatch_log(Bst.handle)
                assert all(lb[2 * j][0] == lb[2 * j + 1][0] and lb[2 * j][1] == 0 and lb[2 * j + 1][1] == 1 for j in range(M))
                for i in range(M):
                    assert abs(losses[i].item() - ref_losses[i]) <= 2e-3 * abs(ref_losses[i])
                got = A.grads_numpy() + Bst.grads_numpy()
                for li, gl in enumerate(got):
                    for k, v in gl.items():
                        assert rel_fro(v, ref["layers"][li][k]) <= GRAD_TOL, (li, k)
                gh = hd.grads_numpy()
                for k in gh:
                    assert rel_fro(gh[k], ref["head"][k]) <= GRAD_TOL, k
                gte, gpe = e.grads_numpy()
                assert rel_fro(gte, ref["wte"]) <= GRAD_TOL and rel_fro(gpe, ref["wpe"]) <= GRAD_TOL
    finally:
        e.close(); hd.close()
