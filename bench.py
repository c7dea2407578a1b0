#!/usr/bin/env python3
"""Benchmark of the stage hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 12b] [--streams 2]

A step is one batch through the whole hot path: start of batch, M forward and M backward
messages through the message-driven scheduler, then the bucketed host-offloaded Adam step
on the stage's parameters.  Inputs (weights, microbatch activations, upstream gradients,
optimizer state) are resident before the timed region.  The headline `value` is the
forward+backward rate (analytic causal FLOPs / time of the forward+backward region, which
HIP events separate from the optimizer region inside every step); `ms_per_step` is the whole
step including the optimizer.  One JSON line is printed.  After the default workload the
same line carries short forward+backward measurements of the 24b and 100b stage shapes
(`other_workloads`) and the bare pinned-copy rates of the machine's host link (`host_link`).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402


# L2-miss bytes per launch of the weight-gradient GEMM from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# (summaries and the scaling by a plain copy under profiles/); keyed by (config, wgrad_group, grad_accum).
WGRAD_TRAFFIC_BYTES = {("12b", 3, "bf16"): 1.687e9}   # profiles/gemm_wgrad_12b_hbm_traffic.md
VOCAB = 51200


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="12b", choices=["tiny", "12b", "24b", "100b", "table1_12b"])
    ap.add_argument("--streams", type=int, default=2, help="library streams of the message-driven run")
    ap.add_argument("--pipeline-limit", type=int, default=0, help="0 = all microbatches in flight")
    ap.add_argument("--grad-accum", default="bf16", choices=["fp32", "bf16"])
    ap.add_argument("--wgrad-group", type=int, default=3, help="microbatches per weight-gradient contraction (0 = as many as possible)")
    ap.add_argument("--ckpt-stride", type=int, default=0,
                    help="activation checkpointing stride ac (0 = keep all activations, the default workload)")
    ap.add_argument("--ends", action="store_true",
                    help="second workload: the stage is both the first and the last one (token embedding in front, "
                         "final LayerNorm + LM head + loss behind, vocabulary 51200); forward messages carry token ids")
    ap.add_argument("--bucket-elems", type=int, default=1 << 26)
    ap.add_argument("--overlap-chunk", type=int, default=1,
                    help="chunk size k (buckets) of the extra measurement with the optimizer step overlapped with "
                         "the backward tail; 0 = skip that measurement")
    ap.add_argument("--qkv-input-split", type=int, default=-1,
                    help="1: the QKV projection consumes LayerNorm-1's output as value + rounding remainder; -1 = the "
                         "configuration's own setting (on for 100b, whose gradient parity needs it, off elsewhere)")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the short forward+backward measurements of the 24b and 100b shapes after the default run")
    ap.add_argument("--no-link-probe", action="store_true", help="skip the bare pinned-copy rates of the host link")
    ap.add_argument("--no-optimizer", action="store_true", help="diagnostic: leave the Adam step out of the step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-profile", action="store_true")
    return ap.parse_args()


def cpu_baseline(shape):
    """The fp64 oracle timed on the host: one microbatch of the workload through the whole stage (every layer,
    forward and backward)."""
    import oracle
    from paper_2110_13005_amd import flops
    from paper_2110_13005_amd.inputs import StageShape, make_stage_inputs
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    one = StageShape(shape.n_layers, shape.hidden, shape.n_heads, shape.seq_len, shape.microbatch_size, 1,
                     shape.ffn_hidden)
    layers, xs, dys = make_stage_inputs(one, seed=0)
    t0 = time.perf_counter()
    oracle.stage_batch(xs, dys, layers, one.n_heads, 1e-5)
    dt = time.perf_counter() - t0
    fl = flops.stage_batch_flops(one, causal=True)
    return {"value": fl / dt / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
            "sample": "1 of %d microbatches of the workload through the whole stage (fwd+bwd), fp64 numpy "
                      "oracle, %.1f s; causal FLOP count" % (shape.n_microbatches, dt),
            "tokens_per_s": one.tokens / dt, "seconds": dt}


def message_order(P, M):
    """Message order of a middle stage: P forwards of warm-up, then one backward / one forward, then drain."""
    order, f, b = [], 0, 0
    while f < min(P, M):
        order.append((0, f)); f += 1
    while b < M:
        order.append((1, b)); b += 1
        if f < M:
            order.append((0, f)); f += 1
    return order


def fill_weights(st, g, dev, host_master=None):
    """Synthetic weights ~N(0, 0.02) (LayerNorm gains 1, biases 0), generated on the device in chunks; the fp32
    draws go to `host_master` (pinned), their roundings to the stage's 16-bit parameters."""
    import torch
    from paper_2110_13005_amd import binding as B
    for name, (off, dims) in st.layout.items():
        numel = int(np.prod(dims))
        short = name.split(".")[1]
        if short.startswith("w_"):
            step = 1 << 26
            for o in range(0, numel, step):
                c = min(step, numel - o)
                w = torch.randn(c, generator=g, device=dev, dtype=torch.float32) * 0.02
                st.params[off + o: off + o + c] = w.to(B.torch_elem_dtype())
                if host_master is not None:
                    host_master[off + o: off + o + c] = w.cpu()
        elif host_master is not None:
            host_master[off: off + numel] = st.params[off: off + numel].float().cpu()


def make_messages(sh, g, dev):
    import torch
    from paper_2110_13005_amd import binding as B
    M = sh.n_microbatches
    bsh = (sh.microbatch_size, sh.seq_len, sh.hidden)
    et = B.torch_elem_dtype()
    X = [torch.randn(bsh, generator=g, device=dev, dtype=torch.float32).to(et) for _ in range(M)]
    # upstream gradients ~N(0,1), as a neighbouring stage would send them (any 1/M lives in grad_scale)
    DY = [torch.randn(bsh, generator=g, device=dev, dtype=torch.float32).to(et) for _ in range(M)]
    Y = [torch.empty(bsh, device=dev, dtype=et) for _ in range(M)]
    DX = [torch.empty(bsh, device=dev, dtype=et) for _ in range(M)]
    return X, DY, Y, DX


def stage_flags(args, config):
    """The construction flags of a stage for `config`: what the full-size parity tests use for it."""
    from paper_2110_13005_amd.inputs import PIPELINE_LIMITS, QKV_INPUT_SPLIT
    split = QKV_INPUT_SPLIT.get(config, 0) if args.qkv_input_split < 0 else args.qkv_input_split
    return dict(grad_accum_fp32=1 if args.grad_accum == "fp32" else 0, wgrad_group=args.wgrad_group,
                qkv_input_split=split), PIPELINE_LIMITS


def other_workload(args, config, batches, dev):
    """Forward+backward of another stage shape, `batches` timed batches back to back after one of warm-up (no
    optimizer step: the 12B-shape default run carries that)."""
    import torch
    from paper_2110_13005_amd import binding as B, flops
    from paper_2110_13005_amd.inputs import CONFIGS
    from paper_2110_13005_amd.stage import Stage
    sh = CONFIGS[config]
    flags, limits = stage_flags(args, config)
    M = sh.n_microbatches
    P = limits.get(config, M)
    g = torch.Generator(device=dev)
    g.manual_seed(1)
    st = Stage(sh, pipeline_limit=P, **flags)
    fill_weights(st, g, dev)
    X, DY, Y, DX = make_messages(sh, g, dev)
    order = message_order(P, M)
    stream = torch.cuda.Stream()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(batches + 1)]
    torch.cuda.synchronize()
    for k in range(batches + 1):
        with torch.cuda.stream(stream):
            evs[k][0].record(stream)
            st.zero_grad(stream)
            for kind, i in order:
                st.post(kind, i, X[i] if kind == 0 else DY[i], Y[i] if kind == 0 else DX[i])
            st.run(args.streams, stream)
            st.join(stream)
            evs[k][1].record(stream)
    torch.cuda.synchronize()
    ms = [e[0].elapsed_time(e[1]) for e in evs[1:]]
    st.close()
    del X, DY, Y, DX
    torch.cuda.empty_cache()
    fl = flops.stage_batch_flops(sh, causal=True)
    mean = float(np.mean(ms))
    tf = fl / (mean * 1e-3) / 1e12
    return {"workload": "%s stage: %d layers, h=%d, heads=%d, seq=%d, microbatch=%d, %d microbatches, pipeline_limit=%d"
                        % (config, sh.n_layers, sh.hidden, sh.n_heads, sh.seq_len, sh.microbatch_size, M, P),
            "dtype": B.ELEM, "flags": dict(flags, streams=args.streams, optimizer_in_step=False),
            "batches": batches, "fwd_bwd_ms": mean, "fwd_bwd_ms_min": float(np.min(ms)), "tflops": tf,
            "pct_of_bf16_mfma_peak": 100.0 * tf / flops.PEAK_BF16_DENSE_TFLOPS,
            "tokens_per_s": M * sh.tokens / (mean * 1e-3)}


def host_link_probe(n_bytes=1 << 28, reps=6):
    """Bare rates of the machine's host link for 256 MiB buckets of pinned memory (the library's probe: hipMemcpyAsync
    as the optimizer pipeline issues it): host to device alone, device to host alone, and per direction with both
    running at once on two streams."""
    from paper_2110_13005_amd import binding as B
    h2d, d2h, both = B.axonn_host_link_probe(0, n_bytes, reps)
    return {"bucket_bytes": n_bytes, "h2d_alone_GBps": h2d, "d2h_alone_GBps": d2h, "both_GBps_each_way": both,
            "pcie_gen5_x16_raw_GBps": 64.0}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives or sharding); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2110_13005_amd import binding as B, flops
    from paper_2110_13005_amd.inputs import CONFIGS, OPT_CONFIG
    from paper_2110_13005_amd.stage import Stage

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    B.load()
    sh = CONFIGS[args.config]
    M = sh.n_microbatches
    flags, limits = stage_flags(args, args.config)
    P = args.pipeline_limit or limits.get(args.config, M)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(0)
    g = torch.Generator(device=dev)
    g.manual_seed(0)

    st = Stage(sh, pipeline_limit=P, ckpt_stride=args.ckpt_stride, **flags)
    n = st.n_params
    # fp32 master copy in pinned host memory, bf16 copy = its rounding
    host_ptrs, host_arrs = [], []
    if not args.no_optimizer:
        import ctypes
        for _ in range(3):
            p = B.axonn_pinned_alloc(4 * n)
            host_ptrs.append(p)
            host_arrs.append(torch.from_numpy(np.ctypeslib.as_array((ctypes.c_float * n).from_address(p))))
    fill_weights(st, g, dev, host_arrs[0] if host_arrs else None)
    if host_arrs:
        # mid-training optimizer state: m ~ N(0,1e-4), v = |N(0,1e-6)|
        step = 1 << 26
        for o in range(0, n, step):
            c = min(step, n - o)
            host_arrs[1][o:o + c] = (torch.randn(c, generator=g, device=dev) * 1e-4).cpu()
            host_arrs[2][o:o + c] = (torch.randn(c, generator=g, device=dev) * 1e-6).abs().cpu()
        B.axonn_stage_optimizer_attach(st.handle, host_ptrs[0], host_ptrs[1], host_ptrs[2], n, args.bucket_elems)
    X, DY, Y, DX = make_messages(sh, g, dev)
    embed = head = None
    if args.ends:
        embed = B.axonn_embed_create(0, VOCAB, sh.hidden, sh.seq_len, sh.microbatch_size)
        head = B.axonn_head_create(0, VOCAB, sh.hidden, sh.tokens, M, 1e-5)
        from paper_2110_13005_amd.stage import view_bf16
        for handle, fn in ((embed, B.axonn_embed_buffers), (head, B.axonn_head_buffers)):
            pp, _, nn = fn(handle)
            v = view_bf16(pp, nn)
            lo = 2 * sh.hidden if handle is head else 0          # the final LayerNorm keeps gain 1, shift 0
            for o in range(lo, nn, 1 << 26):
                c = min(1 << 26, nn - o)
                v[o:o + c] = (torch.randn(c, generator=g, device=dev, dtype=torch.float32) * 0.02).to(B.torch_elem_dtype())
            del v
        B.axonn_stage_attach_ends(st.handle, embed, head)
        TOK = [torch.randint(0, VOCAB, (sh.microbatch_size, sh.seq_len), generator=g, device=dev, dtype=torch.int32) for _ in range(M)]
        TGT = [torch.randint(0, VOCAB, (sh.microbatch_size, sh.seq_len), generator=g, device=dev, dtype=torch.int32) for _ in range(M)]
        LOSS = torch.zeros(M, device=dev)
    torch.cuda.synchronize()

    order = message_order(P, M)
    main_stream = torch.cuda.Stream()
    oc = OPT_CONFIG

    def post_all():
        if args.ends:      # every forward message is followed at once by the loss and Backward (Alg. 2, last stage)
            for i in range(M):
                st.post(0, i, TOK[i], None, targets=TGT[i], loss=LOSS[i:i + 1])
        else:
            for kind, i in order:
                st.post(kind, i, X[i] if kind == 0 else DY[i], Y[i] if kind == 0 else DX[i])

    def one_step(step_no, ev, overlap_chunk=0):
        """ev[0]: start, ev[1]: forward+backward work complete, ev[2]: step complete.  overlap_chunk > 0: the
        optimizer step is queued right after the messages are dispatched and starts on the last layers'
        buckets while the backward tail still runs; there is then no ev[1] (a stream that waited for the
        batch alone would hold up whatever shares its hardware queue, the early fetches included)."""
        with torch.cuda.stream(main_stream):
            ev[0].record(main_stream)
            st.zero_grad(main_stream)
            post_all()
            st.run(args.streams, main_stream)
            hyper = (oc["lr"], oc["beta1"], oc["beta2"], oc["eps"], oc["weight_decay"], oc["step"] + step_no, 1.0 / M)
            if overlap_chunk and not args.no_optimizer:
                B.axonn_stage_optimizer_step_overlapped(st.handle, *hyper, overlap_chunk, main_stream)
                st.join(main_stream)
            else:
                st.join(main_stream)
                ev[1].record(main_stream)
                if not args.no_optimizer:
                    B.axonn_stage_optimizer_step(st.handle, *hyper, main_stream)
            ev[2].record(main_stream)

    def events():
        return [torch.cuda.Event(enable_timing=True) for _ in range(3)]

    for w in range(args.warmup):
        one_step(w, events())
    torch.cuda.synchronize()
    evs = [events() for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        one_step(args.warmup + k, evs[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    fb_ms = [e[0].elapsed_time(e[1]) for e in evs]
    opt_ms = [e[1].elapsed_time(e[2]) for e in evs]
    fb_mean = float(np.mean(fb_ms))
    fl = flops.stage_batch_flops(sh, causal=True)
    fl_paper = flops.stage_batch_flops(sh, causal=False)
    fl_head = flops.lm_head_flops(sh, VOCAB) if args.ends else 0    # cf. Eq. 3's V/16lh term
    fl += fl_head
    fl_paper += fl_head
    tflops = fl / (fb_mean * 1e-3) / 1e12
    tokens = M * sh.tokens

    out = {
        "metric": "stage fwd+bwd TFLOP/s per MI355X and % of bf16 MFMA peak; tokens/s",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": B.ELEM, "data": "synthetic",
        "config": {"workload": "%s stage: %d layers, h=%d, heads=%d, ffn=%d, seq=%d, microbatch=%d, %d microbatches, "
                               "pipeline_limit=%d" % (args.config, sh.n_layers, sh.hidden, sh.n_heads, sh.ffn,
                                                      sh.seq_len, sh.microbatch_size, M, P),
                   "streams": args.streams, "grad_accum": args.grad_accum, "wgrad_group": args.wgrad_group,
                   "qkv_input_split": flags["qkv_input_split"], "bucket_elems": args.bucket_elems,
                   "ckpt_stride": args.ckpt_stride, "ends": "embedding + LM head, V=%d" % VOCAB if args.ends else "none",
                   "optimizer_in_step": not args.no_optimizer},
        "pct_of_bf16_mfma_peak": 100.0 * tflops / flops.PEAK_BF16_DENSE_TFLOPS,
        "peak_tflops_used": flops.PEAK_BF16_DENSE_TFLOPS,
        "tokens_per_s": tokens / (fb_mean * 1e-3),
        "tokens_per_s_whole_step": tokens / (wall / args.steps),
        "fwd_bwd_ms": {"mean": fb_mean, "min": float(np.min(fb_ms)), "per_step": [round(float(x), 3) for x in fb_ms]},
        "tflops_paper_convention": fl_paper / (fb_mean * 1e-3) / 1e12,
        "tflops_executed": (fl + flops.regeneration_flops(sh, args.ckpt_stride)) / (fb_mean * 1e-3) / 1e12,
        "device_bytes": dict(zip(("params", "grads", "grad_shadow", "stash", "workspace", "optimizer"),
                                 B.axonn_stage_device_bytes(st.handle))),
        "paper_context": "49.4-54.78% of V100 fp16 peak per GPU on 48-384 V100s (whole system, counts recompute)",
    }
    if not args.no_optimizer:
        om = float(np.mean(opt_ms))
        out["optimizer"] = {"ms": om, "params": n, "host_link_GBps_each_way": 12.0 * n / (om * 1e-3) / 1e9,
                            "buckets": (n + args.bucket_elems - 1) // args.bucket_elems}
        if args.overlap_chunk > 0:
            # the same steps with the optimizer step overlapped with the backward tail (not part of `value`)
            k_steps = max(2, min(args.steps, 5))
            one_step(args.warmup + args.steps, events(), args.overlap_chunk)
            torch.cuda.synchronize()
            evo = [events() for _ in range(k_steps)]
            t1 = time.perf_counter()
            for k in range(k_steps):
                one_step(args.warmup + args.steps + 1 + k, evo[k], args.overlap_chunk)
            torch.cuda.synchronize()
            wall_o = time.perf_counter() - t1
            out["optimizer_overlapped"] = {
                "chunk_buckets": args.overlap_chunk, "steps": k_steps, "ms_per_step": wall_o / k_steps * 1e3,
                "ms_per_step_plain": wall / args.steps * 1e3,
                "tokens_per_s_whole_step": tokens / (wall_o / k_steps)}

    # per-kernel averages: one more batch on a single stream with launch timing on
    if not args.no_kernel_profile:
        B.axonn_profile_enable(True)
        with torch.cuda.stream(main_stream):
            st.zero_grad(main_stream)
            post_all()
            st.run(1, main_stream)
            st.join(main_stream)
            if not args.no_optimizer:    # one more optimizer step, for the Adam kernel's own time
                B.axonn_stage_optimizer_step(st.handle, oc["lr"], oc["beta1"], oc["beta2"], oc["eps"], oc["weight_decay"],
                                             oc["step"] + 10000, 1.0 / M, main_stream)
        torch.cuda.synchronize()
        prof = B.axonn_profile_collect()
        B.axonn_profile_enable(False)
        h, f_, T = sh.hidden, sh.ffn, sh.tokens
        per_layer_mb = 2 * T * (4 * h * h + 2 * h * f_)          # FLOPs of one GEMM layout per layer per microbatch
        LM = sh.n_layers * M
        kern = {}
        for cat, (ms, cnt) in prof.items():
            if cnt:
                kern[cat] = {"launches": int(cnt), "avg_ms": ms / cnt, "total_ms": ms}
        for cat in ("gemm_fwd", "gemm_dgrad", "gemm_wgrad"):
            if cat in kern:
                work = per_layer_mb * LM
                if cat == "gemm_fwd" and flags["qkv_input_split"]:   # the QKV projection then contracts over 2h
                    work += 2 * T * 3 * h * h * LM
                if cat == "gemm_fwd" and args.ckpt_stride:   # regenerated forward GEMMs, one FC2 per segment left out
                    work += work - M * (sh.n_layers // args.ckpt_stride) * 2 * T * h * f_
                if args.ends:                                # each class holds one of the head's three contractions
                    work += fl_head / 3
                kern[cat]["tflops"] = work / (kern[cat]["total_ms"] * 1e-3) / 1e12
                kern[cat]["frac_of_mfma_peak"] = kern[cat]["tflops"] / flops.PEAK_BF16_DENSE_TFLOPS
        if "attention_fwd" in kern and "attention_bwd" in kern:
            # causal-algorithmic FLOPs: 2 b s^2 h forward, 2.5 x that backward (recomputation not counted)
            afl = 2.0 * sh.microbatch_size * sh.seq_len ** 2 * h * LM
            kern["attention_fwd"]["tflops"] = afl / (kern["attention_fwd"]["total_ms"] * 1e-3) / 1e12
            kern["attention_bwd"]["tflops"] = 2.5 * afl / (kern["attention_bwd"]["total_ms"] * 1e-3) / 1e12
            for cat in ("attention_fwd", "attention_bwd"):
                kern[cat]["frac_of_mfma_peak"] = kern[cat]["tflops"] / flops.PEAK_BF16_DENSE_TFLOPS
        if args.ends:
            if "cross_entropy" in kern:   # logits read twice and written once, bf16; the loss reduction is negligible
                kern["cross_entropy"]["GBps"] = 3 * 2.0 * T * VOCAB * M / (kern["cross_entropy"]["total_ms"] * 1e-3) / 1e9
            if "embedding" in kern:
                kern["embedding"]["note"] = "forward gather, table clear (first microbatch), table and position gradients"
        # HBM-bound kernels: algorithmic bytes per call / average time per call (16-bit elements)
        if "layernorm_fwd" in kern:      # read x, write the normalised row + 8 B of statistics per row
            kern["layernorm_fwd"]["GBps"] = (4.0 * T * h + 8.0 * T) / (kern["layernorm_fwd"]["avg_ms"] * 1e-3) / 1e9
        if "layernorm_bwd" in kern:
            # read dout, x and the residual gradient, write dx, read the statistics: the work as defined; the three
            # launches of a call (dx; column partial sums; their reduction) read dout and x a second time
            kern["layernorm_bwd"]["GBps"] = (8.0 * T * h + 8.0 * T) / (kern["layernorm_bwd"]["avg_ms"] * 1e-3) / 1e9
            kern["layernorm_bwd"]["GBps_as_launched"] = 12.0 * T * h / (kern["layernorm_bwd"]["avg_ms"] * 1e-3) / 1e9
        # (the bias gradients have no launches of their own: the weight-gradient GEMMs form them)
        if "adam" in kern:               # theta, m, v read and written (fp32), gradient read and parameter written (bf16)
            kern["adam"]["GBps"] = 28.0 * n / (kern["adam"]["total_ms"] * 1e-3) / 1e9
        for cat in ("layernorm_fwd", "layernorm_bwd", "adam", "cross_entropy"):
            if cat in kern and "GBps" in kern[cat]:
                kern[cat]["frac_of_hbm_peak"] = kern[cat]["GBps"] / flops.PEAK_HBM_GBPS
        out["kernels"] = kern
        # roofline of the largest single kernel by time: the weight-gradient GEMM
        # (gemm_dma_kernel<false,false,5,8> for bf16 accumulators), one launch = one weight of one layer for a
        # group of microbatches; its four shapes average to per_layer_mb/4 FLOP per microbatch
        dom = "gemm_wgrad"
        if dom in kern:
            per_launch = (per_layer_mb * LM + fl_head / 3) / kern[dom]["launches"]
            ach = per_launch / (kern[dom]["avg_ms"] * 1e-3) / 1e12
            out["roofline"] = {"bound": "mfma", "achieved": ach, "peak": flops.PEAK_BF16_DENSE_TFLOPS,
                               "unit": "TFLOP/s", "frac": ach / flops.PEAK_BF16_DENSE_TFLOPS,
                               "traffic": WGRAD_TRAFFIC_BYTES.get((args.config, args.wgrad_group, args.grad_accum)),
                               "kernel": ("axonn::gemm_big_kernel<false,false,4,8>" if args.grad_accum == "fp32"
                                          else "axonn::gemm_dma_kernel<false,false,5,8>") + " (weight gradient)",
                               "avg_launch_ms": kern[dom]["avg_ms"], "flops_per_launch": per_launch,
                               "measured": "launch timing events on the launching stream, one single-stream batch"}
    # a plain device copy of known size (256 MiB read + 256 MiB written): the reference the HBM byte
    # counters of a profiling run are scaled by
    cal = torch.empty(1 << 27, dtype=torch.int16, device=dev)
    cal2 = torch.empty_like(cal)
    cal2.copy_(cal)
    torch.cuda.synchronize()
    del cal, cal2
    st.close()
    if embed:
        B.axonn_embed_destroy(embed)
        B.axonn_head_destroy(head)
    for p in host_ptrs:
        B.axonn_pinned_free(p)
    del X, DY, Y, DX
    torch.cuda.empty_cache()
    if not args.no_link_probe:
        out["host_link"] = host_link_probe()
        if "optimizer" in out:
            hl = out["host_link"]
            o = out["optimizer"]
            # the step moves 12 B per parameter in each direction at once; the denominator is what the box
            # delivers in one direction alone (two bare copy streams with nothing between them serialise on the copy
            # engine: `both_GBps_each_way`; the step's drain copies run as kernels beside the engine's fetches)
            o["frac_of_link_measured"] = o["host_link_GBps_each_way"] / min(hl["h2d_alone_GBps"], hl["d2h_alone_GBps"])
            o["frac_of_link_raw"] = o["host_link_GBps_each_way"] / hl["pcie_gen5_x16_raw_GBps"]
    # the other stage shapes of the benchmark definition, forward+backward only, a few batches each
    default_run = args.config == "12b" and not args.ends and not args.ckpt_stride
    if default_run and not args.no_other_workloads:
        out["other_workloads"] = [other_workload(args, c, 3, dev) for c in ("24b", "100b")]
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(sh)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
