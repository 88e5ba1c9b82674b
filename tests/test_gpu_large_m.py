"""GPU parity of the large-M path (256 x 256 MFMA tiles, taken from 129 draft rows on when the
hidden size is a multiple of 64) against the fp64 oracle.  Needs an MI355X: run with `-m gpu`."""
import numpy as np
import pytest

import evospec_inputs as gi
from helpers import check_head, to_dev_bf16, to_dev_i32
from test_gpu_parity import ev, problem, run_head  # noqa: F401  (fixture and helpers)

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("M,V_act,d,k", [
    (129, 1000, 256, 10),      # one draft-row tile with a tail, 4 active-row tiles with a tail
    (256, 256, 64, 10),        # exactly one tile, two chunks
    (257, 257, 64, 5),         # one row past a tile in both directions, a single pair of chunks
    (300, 100, 192, 10),       # second half of the only active-row tile wholly empty
    (300, 128, 128, 64),       # k above the group filter's range, exactly one slab
    (512, 777, 4096, 10),      # the benchmark's hidden size
    (130, 40, 320, 33),        # fewer rows than a slab, k > 32
    (200, 5, 64, 5),           # k == V_act
])
def test_large_m_shapes(ev, oracle_mod, M, V_act, d, k):
    W, h, ids = problem(300 + M + V_act, V_act, d, M)
    v, i, l = run_head(ev, h, W, ids, k)
    z = oracle_mod.logits(h, W)
    check_head(v, i, l, z, ids, k, f"M={M} V_act={V_act} d={d} k={k}")


def test_large_m_identity_ids_and_fallback_hidden_size(ev, oracle_mod):
    W, h, ids = problem(41, 600, 256, 140)
    v, i, l = run_head(ev, h, W, None, 10)
    z = oracle_mod.logits(h, W)
    check_head(v, i, l, z, np.arange(600, dtype=np.int32), 10, "ids=None")
    # a hidden size that is not a multiple of 64 takes the 64-row passes instead
    W, h, ids = problem(42, 600, 264, 140)
    v, i, l = run_head(ev, h, W, ids, 10)
    check_head(v, i, l, oracle_mod.logits(h, W), ids, 10, "d=264")


def test_large_m_exact_small_integers(ev):
    """Operands whose products and sums are exact in fp32: logits must match exactly, which pins
    the operand layout of the tiles (row/column/hidden-index mapping) bit for bit."""
    rng = np.random.default_rng(5)
    M, V_act, d, k = 261, 391, 128, 7
    Wf = rng.integers(-4, 5, size=(V_act, d)).astype(np.float32)
    hf = rng.integers(-4, 5, size=(M, d)).astype(np.float32)
    W, h = gi.f32_to_bf16_bits(Wf), gi.f32_to_bf16_bits(hf)
    ids = rng.permutation(5000)[:V_act].astype(np.int32)
    v, i, l = run_head(ev, h, W, ids, k)
    z = hf.astype(np.float64) @ Wf.astype(np.float64).T
    # exact top-k under the tie rule (larger logit, then smaller id)
    for m in range(M):
        order = sorted(range(V_act), key=lambda j: (-z[m, j], ids[j]))[:k]
        assert i[m].tolist() == [int(ids[j]) for j in order], f"row {m}"
        assert v[m].tolist() == [float(z[m, j]) for j in order], f"row {m}"
    zmax = z.max(axis=1, keepdims=True)
    ref = (zmax + np.log(np.exp(z - zmax).sum(axis=1, keepdims=True)))[:, 0]
    np.testing.assert_allclose(l, ref, rtol=1e-5)


def test_large_m_matches_row_passes(ev):
    """The same rows through the large-M path and through 64-row passes (split into calls of at
    most 128 rows) give the same ids and, within fp32 summation-order noise, the same values."""
    W, h, ids = problem(77, 2000, 512, 384)
    v0, i0, l0 = run_head(ev, h, W, ids, 10)
    for r0 in range(0, 384, 128):
        v1, i1, l1 = run_head(ev, h[r0:r0 + 128], W, ids, 10)
        np.testing.assert_allclose(v0[r0:r0 + 128], v1, rtol=1e-4, atol=1e-5)
        np.testing.assert_allclose(l0[r0:r0 + 128], l1, rtol=1e-5)
        same = (i0[r0:r0 + 128] == i1).mean()
        assert same > 0.995, same


def seg_check(ev, oracle_mod, V, d, S, n_core, n_arc, row_off, k, seed):
    import torch
    W = gi.gen_normal_bf16(V, d, seed, 0.05)
    core, arcs = gi.batched_ids(V, max(n_core, 1), max(n_arc, 1), S, seed=seed + 1)
    core, arcs = core[:n_core], arcs[:, :n_arc]
    M = int(row_off[-1])
    h = gi.gen_h(M, d, seed + 2)
    W_core = to_dev_bf16(W[core]) if n_core else torch.empty((0, d), dtype=torch.bfloat16, device="cuda")
    W_arc = to_dev_bf16(np.stack([W[arcs[s]] for s in range(S)])) if n_arc else \
        torch.empty((S, 0, d), dtype=torch.bfloat16, device="cuda")
    ids_arc = to_dev_i32(arcs) if n_arc else torch.empty((S, 0), dtype=torch.int32, device="cuda")
    v, i, l = ev.active_lmhead_topk_segmented(to_dev_bf16(h), W_core, to_dev_i32(core) if n_core else None,
                                              W_arc, ids_arc, row_off, k)
    torch.cuda.synchronize()
    v, i, l = v.cpu().numpy(), i.cpu().numpy(), l.cpu().numpy()
    for s in range(S):
        r0, r1 = row_off[s], row_off[s + 1]
        if r1 > r0:
            union = np.concatenate([core, arcs[s]])
            check_head(v[r0:r1], i[r0:r1], l[r0:r1], oracle_mod.logits(h[r0:r1], W[union]), union, k, f"seq {s}")


def test_segmented_large_m_many_short_sequences(ev, oracle_mod):
    """More than 64 chunks (two batched launches), sequences of 0..9 rows, shared core on the large-M path."""
    rng = np.random.default_rng(3)
    lens = rng.integers(0, 10, size=90)
    lens[5] = 70                                                  # one sequence longer than a chunk
    row_off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    assert row_off[-1] >= 129
    seg_check(ev, oracle_mod, 9000, 128, 90, 1500, 130, row_off, 10, 21)


def test_segmented_without_core_or_without_extensions(ev, oracle_mod):
    row_off = np.array([0, 100, 180, 300], dtype=np.int32)
    seg_check(ev, oracle_mod, 5000, 64, 3, 0, 400, row_off, 10, 31)           # extensions only
    seg_check(ev, oracle_mod, 5000, 64, 3, 700, 0, row_off, 10, 41)           # shared core only (large-M path)
    seg_check(ev, oracle_mod, 5000, 64, 3, 700, 0, np.array([0, 10, 40, 100], dtype=np.int32), 10, 51)   # passes
    seg_check(ev, oracle_mod, 5000, 64, 3, 3, 5, row_off, 8, 61)              # k == union size


@pytest.mark.parametrize("k", [16, 17, 40, 64])
def test_large_m_k_range(ev, oracle_mod, k):
    W, h, ids = problem(500 + k, 700, 128, 200)
    v, i, l = run_head(ev, h, W, ids, k)
    check_head(v, i, l, oracle_mod.logits(h, W), ids, k, f"k={k}")


def test_large_m_all_equal_logits(ev):
    """h = 0: every logit is 0, every list overflows; the k smallest ids must come out, exactly."""
    W, h, ids = problem(9, 1000, 64, 150)
    h[:] = 0
    v, i, l = run_head(ev, h, W, ids, 10)
    want = np.sort(ids)[:10]
    assert np.all(i == want[None, :]) and np.all(v == 0)
    np.testing.assert_allclose(l, np.log(1000.0), rtol=1e-6)
