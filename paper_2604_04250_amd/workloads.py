"""Seeded synthetic inputs shaped like the paper's 150M-parameter model's Resonance Layer.

This module serves both the CPU oracle's tests and the GPU path.  It holds no arithmetic of
the method: it only draws random tensors with the shapes, ranges and distributions of the
benchmark configurations, with numpy's PCG64 generator, in a fixed draw order
(magnitude, angle, gamma, theta, conv taps, upstream gradients), cast to fp32 once.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    F: int
    L: int
    conv_k: int = 4
    gate_tau: float = 0.1
    gamma_lo: float = 0.95
    gamma_hi: float = 0.9999
    theta_uniform: bool = False   # True: theta ~ U[0, pi); False: caller supplies theta
    chunk: int = 0                # >0: streamed in chunks of this many tokens
    seed: int = 4250

    @property
    def J(self) -> int:
        return self.H * self.F

    @property
    def tokens(self) -> int:
        return self.B * self.L

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


# The five benchmark configurations (index = position in the configuration list) and a sixth shape.
CONFIGS = {
    "cfg1_tiny": Workload("cfg1_tiny", B=1, H=2, F=16, L=256, gate_tau=0.1, gamma_lo=0.90,
                          gamma_hi=0.999, theta_uniform=True, seed=4250),
    "cfg2_layer_fwd": Workload("cfg2_layer_fwd", B=4, H=12, F=64, L=2048, seed=4251),
    "cfg3_train": Workload("cfg3_train", B=8, H=12, F=64, L=8192, seed=4252),
    "cfg4_stream": Workload("cfg4_stream", B=1, H=12, F=64, L=2_000_000, gamma_lo=0.999,
                            gamma_hi=0.99999, chunk=4096, seed=4253),
    "cfg5_wide": Workload("cfg5_wide", B=2, H=32, F=128, L=32768, gate_tau=0.25, seed=4254),
    # the lane shape of the paper's own 150M model (4 heads of 64 harmonics), on the training-step batch
    "cfg6_paper_heads": Workload("cfg6_paper_heads", B=8, H=4, F=64, L=8192, seed=4255),
}


def make_inputs(wl: Workload, theta: Optional[np.ndarray] = None, with_grads: bool = True,
                L: Optional[int] = None) -> dict:
    """Draw one batch of inputs for `wl` (optionally with a different token count L).

    Returns float32 arrays: mag, ang [B,L,J]; gamma, theta [J]; conv_w [2,J,Kc]; conv_b [2,J]
    (zeros); dz_re, dz_im [B,L,J] when with_grads.  `theta`, when given, replaces the drawn
    rotation angles (the uniform draw is still consumed so the other tensors do not shift).
    """
    L = wl.L if L is None else L
    B, J, Kc = wl.B, wl.J, wl.conv_k
    rng = np.random.Generator(np.random.PCG64(wl.seed))
    out = {}
    out["mag"] = rng.standard_normal((B, L, J), dtype=np.float32)
    out["ang"] = rng.standard_normal((B, L, J), dtype=np.float32)
    out["gamma"] = rng.uniform(wl.gamma_lo, wl.gamma_hi, J).astype(np.float32)
    drawn = rng.uniform(0.0, np.pi, J).astype(np.float32)
    if theta is not None:
        theta = np.ascontiguousarray(theta, dtype=np.float32)
        assert theta.shape == (J,)
        out["theta"] = theta
    else:
        assert wl.theta_uniform, "this workload takes the rotation angles from the caller"
        out["theta"] = drawn
    kk = max(Kc, 1)
    out["conv_w"] = (rng.standard_normal((2, J, kk)) / np.sqrt(kk)).astype(np.float32)
    out["conv_b"] = np.zeros((2, J), dtype=np.float32)
    if with_grads:
        out["dz_re"] = rng.standard_normal((B, L, J), dtype=np.float32)
        out["dz_im"] = rng.standard_normal((B, L, J), dtype=np.float32)
    return out


def random_state(wl: Workload, seed: int, scale: float = 1.0):
    """A random incoming state: scan part [B,2,J] and conv tail [B,Kc-1,2,J], float32."""
    rng = np.random.Generator(np.random.PCG64(seed))
    scan = (scale * rng.standard_normal((wl.B, 2, wl.J))).astype(np.float32)
    tail = rng.standard_normal((wl.B, max(wl.conv_k - 1, 0), 2, wl.J)).astype(np.float32)
    return scan, tail
