"""Seeded synthetic inputs for the active-vocabulary LM head.

This module serves both the CPU oracle and the GPU library and holds none of the
method's arithmetic: it only draws random tensors and id sets and rounds them to
bf16.  Everything is numpy on the host; bf16 data is carried as uint16 bit patterns.

The tensors stand in for a Qwen3-8B-shaped LM head (151,936 x 4,096), EAGLE-2 draft
hidden states and a corpus-frequency token ranking, none of which are available
here.  Recipe:
  * W_lm ~ N(0, 0.02^2), h ~ N(0, 1), both rounded to nearest-even bf16;
  * a token-frequency ranking is a seeded shuffle of 0..V-1 with frequency of rank r
    proportional to (r+1)^-1.1 (Zipf); the static core is the first n_core ranks,
    the dynamic (ARC) ids are drawn without replacement from the remaining tail with
    probability proportional to that frequency.
"""
from __future__ import annotations

import numpy as np

SEED_W = 1001
SEED_H = 2000
SEED_IDS = 3000

# Named workloads.  V_act = n_core + n_arc.
CONFIGS = {
    # small case the oracle finishes in well under a second
    "tiny": dict(d=256, V=8192, n_core=1024, n_arc=0, M=8, k=8, ids="sorted_uniform", cfg=1),
    # Qwen3-8B / EAGLE-2 shaped draft step: 60 tree nodes, 32k core + 4k dynamic
    "draft60": dict(d=4096, V=151936, n_core=32768, n_arc=4096, M=60, k=10, ids="zipf", cfg=2),
    # per-depth tree expansion (M in {1,4,8}) + 256-row dynamic-buffer update
    "depth": dict(d=4096, V=151936, n_core=16384, n_arc=2048, M=8, k=10, ids="zipf", cfg=3,
                  Ms=(1, 4, 8), update_rows=256),
    # unpruned head: active ids = 0..V-1
    "fullvocab": dict(d=4096, V=151936, n_core=151936, n_arc=0, M=60, k=10, ids="identity", cfg=4),
    # batched serving: 16 sequences x 60 nodes, shared core + per-sequence extension
    "batched": dict(d=4096, V=151936, n_core=32768, n_arc=2048, M=960, k=10, ids="zipf", cfg=5,
                    S=16, rows_per_seq=60),
}


# Active-set sizes of the paper's own experiments (Table 1 sweeps |V_static| in {8k, 16k, 32k} and
# N_dyn in {256, 512, 1024}; the default setting of the hyper-parameter table is 32,000 + 256) and
# a second model shape (hidden size 2,048, vocabulary 128,256).  (name, d, V, n_core, n_arc, M, k)
SWEEP = [("default_32000+256", 4096, 151936, 32000, 256, 60, 10)]
SWEEP += [(f"{c // 1024}k+{a}", 4096, 151936, c, a, 60, 10) for c in (8192, 16384, 32768) for a in (256, 512, 1024)]
SWEEP += [("d2048_32000+256", 2048, 128256, 32000, 256, 60, 10)]


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(seed: int, stream: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))


def gen_normal_bf16(rows: int, cols: int, seed: int, sigma: float, block_rows: int = 4096) -> np.ndarray:
    """[rows, cols] bf16 bits of N(0, sigma^2); block b of `block_rows` rows comes from
    its own Philox stream, so any row range is reproducible on its own."""
    out = np.empty((rows, cols), dtype=np.uint16)
    for b, r0 in enumerate(range(0, rows, block_rows)):
        r1 = min(rows, r0 + block_rows)
        x = _rng(seed, b).standard_normal((r1 - r0, cols), dtype=np.float32)
        if sigma != 1.0:
            x *= np.float32(sigma)
        out[r0:r1] = f32_to_bf16_bits(x)
    return out


def gen_W_lm(V: int, d: int, seed: int = SEED_W) -> np.ndarray:
    return gen_normal_bf16(V, d, seed, 0.02)


def gen_h(M: int, d: int, seed: int = SEED_H) -> np.ndarray:
    return gen_normal_bf16(M, d, seed, 1.0)


def zipf_ranking(V: int, seed: int) -> np.ndarray:
    """Token ids ordered from most to least frequent (a seeded shuffle of 0..V-1)."""
    return _rng(seed, 0).permutation(V).astype(np.int32)


def zipf_weights(V: int, s: float = 1.1) -> np.ndarray:
    w = (np.arange(V, dtype=np.float64) + 1.0) ** (-s)
    return w


def core_arc_ids(V: int, n_core: int, n_arc: int, seed: int, arc_stream: int = 1,
                 s: float = 1.1):
    """(core[n_core], arc[n_arc]) int32: core = top ranks, arc = Zipf-weighted draw from the tail."""
    rank = zipf_ranking(V, seed)
    core = rank[:n_core].copy()
    if n_arc == 0:
        return core, np.empty((0,), dtype=np.int32)
    tail = rank[n_core:]
    w = zipf_weights(V, s)[n_core:]
    p = w / w.sum()
    pick = _rng(seed, arc_stream).choice(tail.shape[0], size=n_arc, replace=False, p=p)
    return core, tail[pick].astype(np.int32)


def sorted_uniform_ids(V: int, n: int, seed: int) -> np.ndarray:
    return np.sort(_rng(seed, 0).choice(V, size=n, replace=False)).astype(np.int32)


def active_ids(name: str, V: int | None = None, n_core: int | None = None, n_arc: int | None = None):
    """Active id list of a named config (optionally at overridden sizes): core then ARC."""
    c = CONFIGS[name]
    V = c["V"] if V is None else V
    n_core = c["n_core"] if n_core is None else n_core
    n_arc = c["n_arc"] if n_arc is None else n_arc
    seed = SEED_IDS + c["cfg"]
    kind = c["ids"]
    if kind == "identity":
        return np.arange(V, dtype=np.int32)
    if kind == "sorted_uniform":
        return sorted_uniform_ids(V, n_core + n_arc, seed)
    core, arc = core_arc_ids(V, n_core, n_arc, seed)
    return np.concatenate([core, arc]).astype(np.int32)


def batched_ids(V: int, n_core: int, n_arc: int, S: int, seed: int = SEED_IDS + 5):
    """Shared core plus S per-sequence extensions, each disjoint from the core
    (extensions of different sequences may overlap, as independent requests would)."""
    rank = zipf_ranking(V, seed)
    core = rank[:n_core].copy()
    tail = rank[n_core:]
    w = zipf_weights(V)[n_core:]
    p = w / w.sum()
    arcs = np.empty((S, n_arc), dtype=np.int32)
    for s_ in range(S):
        pick = _rng(seed, 100 + s_).choice(tail.shape[0], size=n_arc, replace=False, p=p)
        arcs[s_] = tail[pick]
    return core, arcs


def arc_update(V: int, act_ids: np.ndarray, n_core: int, n_new: int, seed: int):
    """A dynamic-buffer update: n_new ids not currently active, written to n_new distinct
    ARC slots (positions >= n_core).  Returns (slots[n_new], new_ids[n_new]) int32."""
    rng = _rng(seed, 7)
    active = np.zeros(V, dtype=bool)
    active[act_ids] = True
    free = np.flatnonzero(~active)
    new_ids = rng.choice(free, size=n_new, replace=False).astype(np.int32)
    n_arc = act_ids.shape[0] - n_core
    slots = (n_core + rng.choice(n_arc, size=n_new, replace=False)).astype(np.int32)
    return slots, new_ids


def bigram_graph(V: int, seed: int, max_degree: int = 64, mean_degree: float = 12.0):
    """A synthetic stand-in for the token co-occurrence graph (appendix, "Token co-occurrence
    graph": bigram successors, at most 64 per source token, kept by decreasing weight) in CSR
    form: (row_ptr int64 [V+1], col_idx int32).  Out-degrees are geometric, capped; successors are
    drawn Zipf-weighted without repetition; their stored order stands for decreasing weight."""
    rng = _rng(seed, 7)
    deg = np.minimum(rng.geometric(1.0 / mean_degree, size=V) - 1, max_degree).astype(np.int64)
    row_ptr = np.zeros(V + 1, dtype=np.int64)
    np.cumsum(deg, out=row_ptr[1:])
    w = zipf_weights(V)
    cdf = np.cumsum(w / w.sum())
    rank = zipf_ranking(V, seed)
    draws = rank[np.minimum(np.searchsorted(cdf, rng.random(int(row_ptr[-1]) * 2)), V - 1)].astype(np.int32)
    col = np.empty(int(row_ptr[-1]), dtype=np.int32)
    pos = 0
    for u in range(V):                                            # distinct successors per source
        need, got, seen = int(deg[u]), 0, set()
        while got < need:
            if pos >= draws.shape[0]:
                draws = rank[np.minimum(np.searchsorted(cdf, rng.random(4096)), V - 1)].astype(np.int32)
                pos = 0
            y = int(draws[pos]); pos += 1
            if y != u and y not in seen:
                seen.add(y)
                col[row_ptr[u] + got] = y
                got += 1
    return row_ptr, col


def checksum(a: np.ndarray) -> int:
    """64-bit FNV-style fold of the raw bytes (to show two runs consumed the same bits)."""
    b = np.ascontiguousarray(a).view(np.uint8).ravel()
    pad = (-b.shape[0]) % 8
    if pad:
        b = np.concatenate([b, np.zeros(pad, dtype=np.uint8)])
    w = b.view(np.uint64)
    idx = np.arange(1, w.shape[0] + 1, dtype=np.uint64)
    with np.errstate(over="ignore"):
        return int(np.bitwise_xor.reduce(w * (idx * np.uint64(0x9E3779B97F4A7C15) | np.uint64(1))))
