"""fp64 CPU oracle for the AxoNN stage hot path.

TEST INFRASTRUCTURE ONLY.  Nothing under this package is part of the product
path: only `tests/`, `__graft_entry__.smoke()` and the `cpu_baseline` leg of
`bench.py` may import it.  It shares no code with the HIP library and never
imports `paper_2110_13005_amd`.

What it is: the paper's method changes *when* and *where* work happens
(message-driven scheduling of a stage's forward/backward passes, Alg. 2; bucketed
CPU-offloaded optimizer, Sec. 5.2) but never *what* is computed (Sec. 7.1 claims
the loss curve is identical to single-device training).  So the oracle is the plain
definition written out: ordinary forward pass, ordinary reverse-mode gradients
summed over microbatches, ordinary Adam, all in float64, one microbatch at a time,
no buckets, no streams, no tiling.

Modules: transformer (layers, stage, activation checkpointing of Sec. 5.1 with Eq. 1 and
the stride rule), lm_ends (first stage's embedding; last stage's final LayerNorm, LM head
and pre-divided loss, Alg. 2 / Sec. 4.2), adam.

Parity pins (see tests/test_oracle_*.py): every gradient formula is pinned by central
finite differences; softmax, LayerNorm, GeLU, the linear maps, the loss and Adam are
pinned by closed forms, special cases and independent library routines; the regenerating
pass is pinned to the plain one.  No function here is "parity unpinned".
"""
from .transformer import (  # noqa: F401
    layernorm_fwd, layernorm_bwd, gelu, gelu_grad, causal_attention_fwd,
    causal_attention_bwd, layer_forward, layer_backward, stage_forward,
    stage_backward, stage_batch, PARAM_NAMES,
)
from .adam import (adam_step, bf16_round, fp16_round, half_round, loss_scaled_adam_step,  # noqa: F401
                   nonfinite_count)
