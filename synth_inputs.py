"""Seeded synthetic inputs for the Markovian next-scale attention path.

This module only draws random tensors and names workloads.  It contains none of the
method's arithmetic (no mask, no softmax, no schedule prefix sums) so that both the
CPU oracle's tests and the HIP path's tests/benchmark can use it without sharing
anything that could hide a common mistake.

Recipe (stand-in for the ImageNet-derived activations of the paper's attention
micro-benchmark, appendix "Efficient Attention Performance", which depends on shapes only): Q, K, V, dO are iid N(0,1),
drawn in fp32 with torch's CPU generator seeded with the workload's seed, in the order
Q, K, V, dO, each of shape [B, H, L, D], then rounded once to bf16 (round to nearest
even).  Both the GPU path and the oracle consume the rounded values.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Tuple

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    sides: Tuple[int, ...]
    B: int
    H: int
    D: int
    seed: int

    @property
    def L(self) -> int:
        return sum(s * s for s in self.sides)


SIDES_TINY = (1, 2, 3, 4)
SIDES_256 = (1, 2, 3, 4, 5, 6, 8, 10, 13, 16)
SIDES_512 = (1, 2, 3, 4, 6, 9, 13, 18, 24, 32)
# SYNTHETIC: the paper times its kernel at 1024px too but never lists that schedule; this one only
# continues the 512px schedule by two scales (L = 8640) to show how the path scales.  Not a
# parity target of the paper's.
SIDES_LARGE_SYNTHETIC = SIDES_512 + (48, 64)

WORKLOADS = {
    "tiny": Workload("tiny", SIDES_TINY, 2, 2, 64, 0),
    "256px_b16_h16": Workload("256px_b16_h16", SIDES_256, 16, 16, 64, 1),
    "256px_b32_h24": Workload("256px_b32_h24", SIDES_256, 32, 24, 64, 2),
    "256px_b32_h30": Workload("256px_b32_h30", SIDES_256, 32, 30, 64, 3),
    "512px_b8_h24": Workload("512px_b8_h24", SIDES_512, 8, 24, 64, 4),
    "large_synthetic_b2_h24": Workload("large_synthetic_b2_h24", SIDES_LARGE_SYNTHETIC, 2, 24, 64, 5),
}


def draw(shape, seed, n_tensors=4, scale=1.0, dtype=torch.bfloat16):
    """n_tensors iid N(0, scale^2) tensors of `shape`, drawn in fp32 on the CPU, in order,
    from one generator seeded with `seed`, each rounded once to `dtype`."""
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    out = []
    for _ in range(n_tensors):
        x = torch.randn(shape, generator=g, dtype=torch.float32)
        if scale != 1.0:
            x = x * scale
        out.append(x.to(dtype))
    return out


def make_inputs(w: Workload, heads=None, dtype=torch.bfloat16):
    """(Q, K, V, dO) for a workload, CPU tensors of `dtype`, shape [B, H, L, D].

    `heads` (optional) limits B*H: the tensors are drawn for B'=1, H'=heads instead;
    used by callers that need a bounded sample of the same shape.
    """
    if heads is None:
        shape = (w.B, w.H, w.L, w.D)
    else:
        shape = (1, int(heads), w.L, w.D)
    return draw(shape, w.seed, 4, 1.0, dtype)


def to_f64(t: torch.Tensor):
    """Widen a tensor (any float dtype, any device) to a float64 numpy array, exactly."""
    return t.detach().to("cpu").to(torch.float64).numpy()
