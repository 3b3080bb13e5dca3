"""Build the synthetic layer stacks of the benchmark workloads on the GPU.

Generation (numpy, seeded), packing (native host pack) and upload only: no oracle here.
"""
from __future__ import annotations

import sys
import time
from concurrent.futures import ThreadPoolExecutor
from typing import List, Optional, Tuple

import numpy as np

import pmpd_synth as synth

from . import binding


def build_stack(shape: synth.StackShape, seed: int = 0, n_blocks: Optional[int] = None, workers: int = 8,
                keep_host: Optional[set] = None, verbose: bool = False, keep_rows=None):
    """Generate, pack and upload every linear layer of `shape`.

    Returns (stack, layers, kept) where kept[(block, proj)] = (q4, s, a) for the layer
    indices listed in keep_host (host copies for parity checks; everything else is freed).
    With keep_rows(block, proj, out_features) -> row indices, kept[(block, proj)] is instead
    (rows, q4[rows], s[rows], a[rows]) for every layer: a few logical rows per layer, enough to
    check sampled outputs of a full-size stack without holding its codes on the host.
    """
    n_blocks = shape.n_blocks if n_blocks is None else n_blocks
    todo = [(blk, pi, o, i) for blk in range(n_blocks) for pi, (nm, o, i) in enumerate(shape.proj_shapes())]
    keep_host = keep_host or set()
    kept = {}
    t0 = time.time()

    def make(job):
        blk, pi, o, i = job
        q4, s, a = synth.draw_weights(seed, blk, pi, o, i)
        planes, sm = binding.pack(q4, s, a)
        if (blk, pi) in keep_host:
            return job, planes, sm, (q4, s, a)
        if keep_rows is not None:
            rows = np.asarray(keep_rows(blk, pi, o), dtype=np.int64)
            return job, planes, sm, (rows, q4[rows].copy(), s[rows].copy(), a[rows].copy())
        return job, planes, sm, None

    layers: List[binding.PackedLayer] = []
    with ThreadPoolExecutor(max_workers=workers) as pool:
        for n, (job, planes, sm, host) in enumerate(pool.map(make, todo)):
            blk, pi, o, i = job
            layers.append(binding.upload_layer(planes, sm, o, i))
            if host is not None:
                kept[(blk, pi)] = host
            if verbose and (n + 1) % 28 == 0:
                print(f"  built {n + 1}/{len(todo)} layers ({time.time() - t0:.0f} s)", file=sys.stderr, flush=True)
    stack = binding.Stack(layers)
    return stack, layers, kept


def draw_step_activations(shape: synth.StackShape, seed: int, step: int, n_blocks: Optional[int] = None) -> np.ndarray:
    """Concatenated fp16 activations of one decode step, in the stack's default x layout."""
    n_blocks = shape.n_blocks if n_blocks is None else n_blocks
    parts = []
    for blk in range(n_blocks):
        for pi, (nm, o, i) in enumerate(shape.proj_shapes()):
            parts.append(synth.draw_x(seed, step, blk, pi, i)[0])
    return np.concatenate(parts)
