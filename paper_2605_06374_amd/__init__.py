"""MI355X-native document-masked causal attention (forward + backward) for packed
variable-length microbatches: the quadratic, length-dependent term of the micro-batch
time model (Section 5.2, Eq. 1).

The compute lives in a C-ABI shared library built from ``csrc/`` (HIP, gfx950 only).
``paper_2605_06374_amd.binding`` marshals arguments into it; nothing here computes
attention in Python and there is no CPU fallback.
"""
__all__ = ["workloads"]
