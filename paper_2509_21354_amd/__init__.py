"""MI355X-native gated chunked-KV decode attention (KV-Efficient VLA hot path).

The product is the C-ABI library built from ``csrc/`` (see ``include/kvev.h``);
``binding`` marshals torch device tensors into it and ``synth`` draws the
seeded synthetic workloads.  Nothing here computes on the CPU.
"""
from . import synth  # noqa: F401

__all__ = ["synth", "binding", "build"]
