"""MI355X-native per-GPU hot path of a Ulysses-style sequence-parallel layer:
sequence<->head re-layout and causal GQA attention forward/backward.

The compute lives in a C-ABI shared library built from ``csrc/``; the Python
layer (`binding`) only marshals arguments.  Nothing here falls back to a CPU
or PyTorch implementation: a missing library raises.
"""
__all__ = ["binding", "synth"]
