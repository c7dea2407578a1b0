"""Analytic work counts of the stage (host-side bookkeeping, no kernels).

Forward FLOPs of one layer on T = b*s tokens: the four weight GEMMs cost 2*T*(3h^2 + h^2 +
h*f + f*h) (= 24*T*h^2 when f = 4h); attention's two contractions cost 4*b*s^2*h when every
(query, key) pair is counted (the paper's convention: the s/6h term of its Eq. 3) and
half of that when only the causal pairs j <= i are (the work the method has to do).
Forward + backward = 3x forward when activations are stored; with activation checkpointing
(Sec. 5.1) the backward pass first runs the forward pass again (the paper's factor 96 = 4 * 24
contains one, Sec. 6.2), except that this build leaves out the last contraction of every
regenerated segment, whose result nobody reads."""

PEAK_BF16_DENSE_TFLOPS = 2516.6   # MI355X: 256 CU x 2.4 GHz x 4096 flop/clk/CU
PEAK_HBM_GBPS = 8000.0


def layer_forward_flops(h, f, s, b, causal=True):
    T = b * s
    gemm = 2 * T * (3 * h * h + h * h + 2 * h * f)
    attn = 4 * b * s * s * h
    return gemm + (attn // 2 if causal else attn)


def stage_batch_flops(shape, causal=True, n_microbatches=None):
    """fwd + bwd FLOPs of all layers over all microbatches of a batch."""
    M = shape.n_microbatches if n_microbatches is None else n_microbatches
    return 3 * shape.n_layers * M * layer_forward_flops(
        shape.hidden, shape.ffn, shape.seq_len, shape.microbatch_size, causal)


def regeneration_flops(shape, ckpt_stride, causal=True, n_microbatches=None):
    """FLOPs of the forward work that backward passes repeat with checkpointing stride ckpt_stride
    (0: none): one forward per layer minus the second MLP contraction of each segment's last layer."""
    if not ckpt_stride:
        return 0
    M = shape.n_microbatches if n_microbatches is None else n_microbatches
    per_layer = layer_forward_flops(shape.hidden, shape.ffn, shape.seq_len, shape.microbatch_size, causal)
    skipped = 2 * shape.tokens * shape.hidden * shape.ffn
    return M * (shape.n_layers * per_layer - (shape.n_layers // ckpt_stride) * skipped)


def lm_head_flops(shape, vocab, n_microbatches=None):
    """fwd + bwd FLOPs of the last stage's LM head over a batch: three contractions of 2*T*h*V each per
    microbatch (logits, their input gradient, the head's weight gradient): Eq. 3's V/16lh term, 6*b*s*h*V."""
    M = shape.n_microbatches if n_microbatches is None else n_microbatches
    return 3 * 2 * shape.tokens * shape.hidden * vocab * M


def narayanan_flops(b, s, l, h, V=0, recompute=True):
    """The paper's Eq. 3 numerator without the time: 96*b*s*l*h^2*(1 + s/6h + V/16lh), or the
    72-form when there is no recompute forward."""
    c = 96 if recompute else 72
    return c * b * s * l * h * h * (1 + s / (6 * h) + V / (16 * l * h))


def stage_param_count(n_layers, h, f=None):
    f = 4 * h if f is None else f
    return n_layers * (3 * h * h + h * h + 2 * h * f + 3 * h + h + f + h + 4 * h)


def stash_bytes_per_layer(h, f, s, b, a):
    """Activation bytes one layer keeps for backward per microbatch (bf16 tensors + fp32 stats)."""
    T = b * s
    return 2 * T * (5 * h + 3 * h + 2 * f) + 2 * (T * 2 * 4) + b * a * s * 4
