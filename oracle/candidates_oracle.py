"""Plain reference of the candidate formation of a failure event (test infrastructure).

What it follows: the EvoSpec paper, Sec. "Semantic approximation" / "Statistical expansion" and
the appendix paragraph "Runtime candidate formation": the initial pool is the union of the
target-side top candidates at the rejection step and the nearest neighbours of the target hidden
state among the LM-head rows; every seed then contributes up to eight outgoing neighbours of a
sparse token co-occurrence graph; the result is de-duplicated before it goes to the buffer
manager.  The neighbour search here is the exact maximum inner product (the paper's index is an
approximation of exactly this), computed in fp64 on the bf16 bit patterns.

Readings where the paper is silent: the order is target candidates, then retrieved neighbours,
then the successors seed by seed in that same order, each seed's successors in the order the
graph stores them (the graph keeps them by decreasing weight); a duplicate keeps its first place.

Only tests, the smoke check and the benchmark's CPU leg may import this module.
"""
from __future__ import annotations

import numpy as np


def exact_mips(h_bits: np.ndarray, W_bits: np.ndarray, n: int) -> np.ndarray:
    """Ids of the n rows of W with the largest inner product with h (ties: smaller id first)."""
    h = (h_bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64).reshape(-1)
    z = np.empty(W_bits.shape[0], dtype=np.float64)
    for r0 in range(0, W_bits.shape[0], 8192):                  # row blocks: bounded memory
        blk = (W_bits[r0:r0 + 8192].astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        z[r0:r0 + 8192] = blk @ h
    order = sorted(range(z.shape[0]), key=lambda i: (-z[i], i)) if z.shape[0] <= 4096 else \
        np.lexsort((np.arange(z.shape[0]), -z))
    return np.asarray(order[:n], dtype=np.int32)


def form_candidates(target_top, mips_top, row_ptr, col_idx, max_successors=8, cap=None):
    """The ordered, de-duplicated candidate list of one failure event."""
    seeds, seen = [], set()
    for x in list(target_top) + list(mips_top):
        x = int(x)
        if x not in seen:
            seen.add(x)
            seeds.append(x)
    out = list(seeds)
    for s in seeds:
        lo, hi = int(row_ptr[s]), int(row_ptr[s + 1])
        for j in range(lo, min(hi, lo + max_successors)):
            y = int(col_idx[j])
            if y not in seen:
                seen.add(y)
                out.append(y)
    return out if cap is None else out[:cap]
