"""Seeded synthetic inputs for the PMPD decode linear-layer path.

This module only draws random numbers and names shapes.  It holds none of the
method's arithmetic (no packing, no dequantisation, no dot products) so that
both the CPU oracle's tests and the HIP path's tests can feed from it without
sharing any computation.

The real checkpoints the paper evaluates (Section 5, "Models and Datasets")
are replaced by layer stacks of the same shapes with random contents:
4-bit codes uniform on 0..15, one fp16 scale and one fp16 minimum per group of
128 consecutive input features, fp16 activations ~ N(0, 1).

Draw order (fixed, so a seed names one data set):
  weights of (seed, layer, proj):  PCG64(SeedSequence([seed, layer, proj, 0]))
      -> q4  = integers(0, 16, (out, in), uint8)
      -> s   = uniform(1e-3, 1e-2, (out, in/128)) in fp64, rounded to fp16
      -> a   = -8 * s (computed on the fp16 values; exact, a power of two)
  unquantised fp16 weights of (seed, layer, proj): PCG64(SeedSequence([seed, layer, proj, 2]))
      -> W   = 0.02 * standard_normal((out, in)) in fp64, rounded to fp16 (the fp16 baseline's operand)
  activations of (seed, step, layer, proj): PCG64(SeedSequence([seed + step, layer, proj, 1]))
      -> x   = standard_normal((m, in)) in fp64, rounded to fp16

Learned-scheduler inputs of (seed): PCG64(SeedSequence([seed, 0, 0, 3])), in this order
      -> K   = standard_normal((T, D_k)), V = standard_normal((T, D_v)), both rounded to fp16
      -> q   = standard_normal(D_k) * sharpness      (fp32)
      -> W1  = standard_normal((H, D_v)) / sqrt(D_v), b1 = 0.1 * standard_normal(H)
      -> W2  = standard_normal((N, H)) * 4 / sqrt(H), b2 = 0.1 * standard_normal(N)   (all fp32)
  (random parameters stand in for the trained ones, which are not public.)
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Tuple

import numpy as np

GROUP = 128  # input features per quantisation group

# The seven projections of a Llama-style block, in the order the paper's
# latency tables list them (Tables 7 and 8): q, k, v, o, up, down, gate.
PROJ_NAMES = ("q", "k", "v", "o", "up", "down", "gate")


@dataclass(frozen=True)
class StackShape:
    """A decoder stack reduced to the shapes of its linear layers."""

    name: str
    n_blocks: int
    hidden: int
    intermediate: int

    def proj_shapes(self) -> List[Tuple[str, int, int]]:
        """(name, out_features, in_features) of the seven projections of one block."""
        h, f = self.hidden, self.intermediate
        return [
            ("q", h, h),
            ("k", h, h),
            ("v", h, h),
            ("o", h, h),
            ("up", f, h),
            ("down", h, f),
            ("gate", f, h),
        ]

    def layers(self) -> List[Tuple[int, int, str, int, int]]:
        """Flat list of (block, proj_index, name, out, in) over the whole stack."""
        out = []
        for blk in range(self.n_blocks):
            for pi, (nm, o, i) in enumerate(self.proj_shapes()):
                out.append((blk, pi, nm, o, i))
        return out

    def n_weights(self) -> int:
        return self.n_blocks * sum(o * i for _, o, i in self.proj_shapes())


# Shapes of the five workloads.
SINGLE_4096 = StackShape("single-4096x4096", 1, 4096, 4096)  # only its "q" projection is used
LLAMA_7B = StackShape("llama-7b-shaped", 32, 4096, 11008)
MOBILE = StackShape("mobile-1.4b-shaped", 22, 2048, 5632)
LLAMA_13B = StackShape("llama-13b-shaped", 40, 5120, 13824)

STACKS: Dict[str, StackShape] = {
    "7b": LLAMA_7B,
    "mobile": MOBILE,
    "13b": LLAMA_13B,
}

# Progressive schedules of the workloads: (precisions high->low, switch points, steps).
SCHEDULE_7B_256 = ((4, 3, 2), (0, 64, 160), 256)
SCHEDULE_13B_128 = ((3, 2), (0, 48), 128)


def _rng(*key: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence(list(key))))


def draw_codes(seed: int, layer: int, proj: int, out_f: int, in_f: int) -> np.ndarray:
    """4-bit codes, uniform integers 0..15, shape (out, in), uint8."""
    return _rng(seed, layer, proj, 0).integers(0, 16, size=(out_f, in_f), dtype=np.uint8)


def draw_weights(seed: int, layer: int, proj: int, out_f: int, in_f: int,
                 random_min: bool = False):
    """(q4 uint8 [out,in], s fp16 [out,in/128], a fp16 [out,in/128]).

    With random_min the minima are drawn independently of the scales
    (uniform on [-0.12, 0.04]); otherwise a = -8*s as in the headline workloads.
    """
    if in_f % GROUP:
        raise ValueError("in_features must be a multiple of 128")
    g = _rng(seed, layer, proj, 0)
    q4 = g.integers(0, 16, size=(out_f, in_f), dtype=np.uint8)
    s = g.uniform(1e-3, 1e-2, size=(out_f, in_f // GROUP)).astype(np.float16)
    if random_min:
        a = g.uniform(-0.12, 0.04, size=s.shape).astype(np.float16)
    else:
        a = (np.float16(-8.0) * s).astype(np.float16)
    return q4, s, a


def draw_x(seed: int, step: int, layer: int, proj: int, in_f: int, m: int = 1) -> np.ndarray:
    """Activations, fp16, shape (m, in)."""
    return _rng(seed + step, layer, proj, 1).standard_normal(size=(m, in_f)).astype(np.float16)


def draw_fp16_weights(seed: int, layer: int, proj: int, out_f: int, in_f: int) -> np.ndarray:
    """Unquantised weights for the fp16 baseline kernel: fp16, shape (out, in), ~ N(0, 0.02^2)."""
    return (0.02 * _rng(seed, layer, proj, 2).standard_normal(size=(out_f, in_f))).astype(np.float16)


def draw_learned_scheduler(seed: int, T: int, d_k: int, d_v: int, hidden: int, n_classes: int, sharpness: float = 1.0):
    """(K fp16 [T,d_k], V fp16 [T,d_v], q fp32 [d_k], W1 fp32 [hidden,d_v], b1, W2 fp32 [n_classes,hidden], b2)."""
    g = _rng(seed, 0, 0, 3)
    K = g.standard_normal(size=(T, d_k)).astype(np.float16)
    V = g.standard_normal(size=(T, d_v)).astype(np.float16)
    q = (g.standard_normal(size=d_k) * sharpness).astype(np.float32)
    W1 = (g.standard_normal(size=(hidden, d_v)) / np.sqrt(d_v)).astype(np.float32)
    b1 = (0.1 * g.standard_normal(size=hidden)).astype(np.float32)
    W2 = (g.standard_normal(size=(n_classes, hidden)) * 4.0 / np.sqrt(hidden)).astype(np.float32)
    b2 = (0.1 * g.standard_normal(size=n_classes)).astype(np.float32)
    return K, V, q, W1, b1, W2, b2
