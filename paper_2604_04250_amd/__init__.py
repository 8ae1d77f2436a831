"""MI355X-native hot path of CAWN's Resonance Layer: fused Temporal-Syntax-Cache conv + gated
phasor + causal phase-accumulation scan (forward, backward, chunked state passing).

`binding` mirrors the C ABI of include/cawn.h; `workloads` draws the seeded synthetic inputs;
`build` compiles csrc/ into libcawn.so with hipcc for gfx950.
"""
from . import workloads  # noqa: F401

__all__ = ["workloads", "binding", "build"]
