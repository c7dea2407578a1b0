"""MI355X-native implementation of the per-GPU hot path of AxoNN (arXiv 2110.13005):
one pipeline stage's forward/backward over a message-driven stream of microbatches and
the bucketed, host-offloaded mixed-precision Adam step.

The compiled HIP library is loaded lazily by `paper_2110_13005_amd.binding`; importing
this package (e.g. for `inputs`) does not need a GPU.
"""
__all__ = ["inputs", "binding", "flops"]
