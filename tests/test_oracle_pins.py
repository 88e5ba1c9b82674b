"""Pins for the CPU oracle: everything here is checked against something other than
the oracle itself -- the definition written with numpy/scipy/torch library routines,
closed forms, invariants of Eq. 1, and a hand example.  CPU only.
"""
import math
import os

import numpy as np
import pytest

import evospec_inputs as gi

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "worked_example_eq1.txt")


def f64(bits):
    return gi.bf16_bits_to_f32(bits).astype(np.float64)


def np_topk(z_row, ids, k):
    """Reference order: logits descending, ties by ascending id (numpy lexsort)."""
    order = np.lexsort((ids, -z_row))[:k]
    return z_row[order], ids[order]


def small_problem(seed, V=300, d=40, M=5, n_act=77):
    W = gi.gen_normal_bf16(V, d, seed, 0.5, block_rows=64)
    h = gi.gen_normal_bf16(M, d, seed + 1, 1.0)
    rng = np.random.default_rng(seed)
    ids = rng.choice(V, size=n_act, replace=False).astype(np.int32)
    return W, h, ids


# ---------------------------------------------------------------- hand example
def parse_golden():
    rows = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            rows[key] = vals
    return rows


def test_worked_example(oracle_mod):
    g = parse_golden()
    h = gi.f32_to_bf16_bits(np.array([[float(x) for x in g["h"]]], dtype=np.float32))
    W = gi.f32_to_bf16_bits(np.array([[float(x) for x in g[f"W_lm[{i}]"]] for i in range(5)], dtype=np.float32))
    # the inputs are exactly representable
    assert np.array_equal(gi.bf16_bits_to_f32(W)[3], np.array([-1.0, 0.5], dtype=np.float32))
    z_full = oracle_mod.logits(h, W)
    assert z_full.shape == (1, 5)
    assert z_full[0].tolist() == [float(x) for x in g["z_full"]]
    act = np.array([int(x) for x in g["active"]], dtype=np.int32)
    W_act = np.zeros((3, 2), dtype=np.uint16)
    act_ids = np.full((3,), -1, dtype=np.int32)
    oracle_mod.active_gather(W, act, None, W_act, act_ids)
    vals, ids, lz, z = oracle_mod.active_lmhead_topk(h, W_act, act_ids, 2, return_logits=True)
    assert z[0].tolist() == [float(x) for x in g["z_act"]]
    exp_top = [(float(t.split(":")[0]), int(t.split(":")[1])) for t in g["top2"]]
    assert list(zip(vals[0].tolist(), ids[0].tolist())) == exp_top
    closed = math.log(math.exp(0.0) + math.exp(2.0) + math.exp(3.0))
    assert abs(lz[0] - closed) < 1e-14
    # and the unrestricted normaliser is strictly larger
    assert oracle_mod.logz(z_full)[0] > lz[0]


# ------------------------------------------------- brute force vs the definition
@pytest.mark.parametrize("seed", [11, 12, 13])
def test_pruned_logits_equal_full_vocab_entries(oracle_mod, seed):
    W, h, ids = small_problem(seed)
    z_def = f64(h) @ f64(W).T                       # Eq. 1 with a library matmul
    z_full = oracle_mod.logits(h, W)
    assert z_full.shape == z_def.shape == (h.shape[0], W.shape[0])
    np.testing.assert_allclose(z_full, z_def, rtol=0, atol=1e-12)
    W_act = np.zeros((ids.shape[0], W.shape[1]), dtype=np.uint16)
    act_ids = np.zeros_like(ids)
    oracle_mod.active_gather(W, ids, None, W_act, act_ids)
    assert np.array_equal(W_act, W[ids]) and np.array_equal(act_ids, ids)
    z_act = oracle_mod.logits(h, W_act)
    # same bits, same summation order: restricted logits ARE the full-vocab entries
    assert np.array_equal(z_act, z_full[:, ids])


@pytest.mark.parametrize("k", [1, 7, 32])
def test_all_ids_active_equals_unpruned_topk(oracle_mod, k):
    W, h, _ = small_problem(21)
    V = W.shape[0]
    all_ids = np.arange(V, dtype=np.int32)
    vals, ids, lz = oracle_mod.active_lmhead_topk(h, W, all_ids, k)
    z_def = f64(h) @ f64(W).T
    for m in range(h.shape[0]):
        ev, ei = np_topk(z_def[m], all_ids, k)
        assert np.array_equal(ids[m], ei)
        np.testing.assert_allclose(vals[m], ev, rtol=0, atol=1e-12)
    # ids == NULL is the identity map
    vals2, ids2, lz2 = oracle_mod.active_lmhead_topk(h, W, None, k)
    assert np.array_equal(ids, ids2) and np.array_equal(vals, vals2) and np.array_equal(lz, lz2)


def test_active_topk_is_filtered_full_topk(oracle_mod):
    W, h, ids = small_problem(31)
    k = 9
    W_act = W[ids]
    vals, oid, lz = oracle_mod.active_lmhead_topk(h, W_act, ids, k)
    z_def = f64(h) @ f64(W).T
    member = np.zeros(W.shape[0], dtype=bool)
    member[ids] = True
    for m in range(h.shape[0]):
        order = np.lexsort((np.arange(W.shape[0]), -z_def[m]))
        filt = [i for i in order if member[i]][:k]
        assert oid[m].tolist() == filt
        np.testing.assert_allclose(vals[m], z_def[m][filt], rtol=0, atol=1e-12)


def test_softmax_over_active_set_sums_to_one(oracle_mod):
    W, h, ids = small_problem(41)
    _, _, lz, z = oracle_mod.active_lmhead_topk(h, W[ids], ids, 3, return_logits=True)
    s = np.exp(z - lz[:, None]).sum(axis=1)
    np.testing.assert_allclose(s, 1.0, rtol=0, atol=1e-12)


def test_logz_against_library_routines(oracle_mod):
    from scipy.special import logsumexp
    import torch
    W, h, ids = small_problem(51, V=500, d=64, M=6, n_act=200)
    z_def = f64(h) @ f64(W[ids]).T
    _, _, lz = oracle_mod.active_lmhead_topk(h, W[ids], ids, 1)
    np.testing.assert_allclose(lz, logsumexp(z_def, axis=1), rtol=0, atol=1e-12)
    lsm = torch.log_softmax(torch.from_numpy(z_def), dim=1).numpy()
    vals, oid, lz2 = oracle_mod.active_lmhead_topk(h, W[ids], ids, 4)
    # log-prob of a returned entry = value - logZ  == library log_softmax at that slot
    pos = {int(t): i for i, t in enumerate(ids)}
    for m in range(h.shape[0]):
        for j in range(4):
            assert abs((vals[m, j] - lz2[m]) - lsm[m, pos[int(oid[m, j])]]) < 1e-12
    tv, ti = torch.topk(torch.from_numpy(z_def), 4, dim=1)
    np.testing.assert_allclose(vals, tv.numpy(), rtol=0, atol=1e-12)


# ------------------------------------------------------------ closed forms
def test_zero_hidden_state_closed_form(oracle_mod):
    W, _, ids = small_problem(61)
    h0 = np.zeros((3, W.shape[1]), dtype=np.uint16)
    k = 6
    vals, oid, lz = oracle_mod.active_lmhead_topk(h0, W[ids], ids, k)
    assert np.all(lz == math.log(ids.shape[0]))
    assert np.all(vals == 0.0)
    smallest = np.sort(ids)[:k]
    for m in range(3):
        assert np.array_equal(oid[m], smallest)     # all logits tie -> ascending full-vocab id


def test_one_hot_hidden_state_reads_a_column(oracle_mod):
    W, _, ids = small_problem(71)
    d = W.shape[1]
    one = gi.f32_to_bf16_bits(np.array([1.0], dtype=np.float32))[0]
    for j in (0, 5, d - 1):
        h1 = np.zeros((1, d), dtype=np.uint16)
        h1[0, j] = one
        z = oracle_mod.logits(h1, W[ids])
        assert np.array_equal(z[0], f64(W[ids][:, j]))


def test_scaling_and_sign(oracle_mod):
    """z is linear in h: doubling h (exact in bf16) doubles every logit; negating flips order."""
    W, h, ids = small_problem(81)
    hf = gi.bf16_bits_to_f32(h)
    h2 = gi.f32_to_bf16_bits(hf * 2.0)
    hn = gi.f32_to_bf16_bits(-hf)
    z = oracle_mod.logits(h, W[ids])
    assert np.array_equal(oracle_mod.logits(h2, W[ids]), 2.0 * z)
    assert np.array_equal(oracle_mod.logits(hn, W[ids]), -z)
    v1, i1, _ = oracle_mod.active_lmhead_topk(hn, W[ids], ids, 1)
    assert np.array_equal(i1[:, 0], ids[np.argmin(z, axis=1)])


# ------------------------------------------------------------ invariants
def test_order_of_active_ids_does_not_matter(oracle_mod):
    W, h, ids = small_problem(91)
    k = 8
    v0, i0, l0 = oracle_mod.active_lmhead_topk(h, W[ids], ids, k)
    perm = np.random.default_rng(5).permutation(ids.shape[0])
    ids_p = ids[perm]
    v1, i1, l1 = oracle_mod.active_lmhead_topk(h, W[ids_p], ids_p, k)
    assert np.array_equal(i0, i1) and np.array_equal(v0, v1)
    np.testing.assert_allclose(l0, l1, rtol=0, atol=1e-13)


def test_rows_are_independent(oracle_mod):
    W, h, ids = small_problem(101)
    v, i, l = oracle_mod.active_lmhead_topk(h, W[ids], ids, 5)
    for m in range(h.shape[0]):
        vm, im, lm = oracle_mod.active_lmhead_topk(h[m:m + 1], W[ids], ids, 5)
        assert np.array_equal(vm[0], v[m]) and np.array_equal(im[0], i[m]) and lm[0] == l[m]


def test_logz_grows_with_the_active_set(oracle_mod):
    W, h, ids = small_problem(111, n_act=120)
    prev = None
    for n in (10, 40, 120):
        _, _, lz = oracle_mod.active_lmhead_topk(h, W[ids[:n]], ids[:n], 1)
        if prev is not None:
            assert np.all(lz > prev)
        prev = lz
    full = oracle_mod.logz(oracle_mod.logits(h, W))
    assert np.all(full > prev)


def test_k1_is_argmax_and_k_full_is_a_sort(oracle_mod):
    W, h, ids = small_problem(121, n_act=50)
    z = f64(h) @ f64(W[ids]).T
    v1, i1, _ = oracle_mod.active_lmhead_topk(h, W[ids], ids, 1)
    assert np.array_equal(i1[:, 0], ids[np.argmax(z, axis=1)])
    vf, idf, _ = oracle_mod.active_lmhead_topk(h, W[ids], ids, 50)
    for m in range(h.shape[0]):
        assert sorted(idf[m].tolist()) == sorted(ids.tolist())
        assert np.all(np.diff(vf[m]) <= 0)
        ev, ei = np_topk(z[m], ids, 50)
        assert np.array_equal(idf[m], ei)


def test_exact_ties_break_on_full_vocab_id_not_slot(oracle_mod):
    """Duplicate weight rows under different ids give exactly equal logits; the smaller
    full-vocabulary id must come first whatever the slot order."""
    W, h, _ = small_problem(131, V=64, d=16, M=2, n_act=8)
    W[40] = W[7]
    W[55] = W[7]
    W[3] = W[7]
    ids = np.array([55, 9, 40, 7, 20, 3], dtype=np.int32)      # tied ids out of order
    vals, oid, _ = oracle_mod.active_lmhead_topk(h, W[ids], ids, 6)
    for m in range(2):
        tied = [int(t) for t, v in zip(oid[m], vals[m]) if v == vals[m][list(oid[m]).index(7)]]
        assert tied == [3, 7, 40, 55]


# ------------------------------------------------------------ gather
def test_gather_matches_fancy_indexing_and_incremental_update(oracle_mod):
    W, _, ids = small_problem(141, V=200, d=24, n_act=64)
    W_act = np.zeros((64, 24), dtype=np.uint16)
    act_ids = np.zeros((64,), dtype=np.int32)
    oracle_mod.active_gather(W, ids, None, W_act, act_ids)
    assert np.array_equal(W_act, W[ids]) and np.array_equal(act_ids, ids)
    before = W_act.copy()
    slots, new_ids = gi.arc_update(200, act_ids, n_core=48, n_new=5, seed=3)
    oracle_mod.active_gather(W, new_ids, slots, W_act, act_ids)
    untouched = np.setdiff1d(np.arange(64), slots)
    assert np.array_equal(W_act[untouched], before[untouched])
    assert np.array_equal(W_act[slots], W[new_ids]) and np.array_equal(act_ids[slots], new_ids)
    assert np.unique(act_ids).shape[0] == 64            # still a set (Eq. 3 is a union)


def test_gather_permutation_round_trip(oracle_mod):
    W = gi.gen_normal_bf16(50, 8, 5, 1.0)
    perm = np.random.default_rng(1).permutation(50).astype(np.int32)
    inv = np.argsort(perm).astype(np.int32)
    A = np.zeros_like(W)
    B = np.zeros_like(W)
    tmp = np.zeros((50,), dtype=np.int32)
    oracle_mod.active_gather(W, perm, None, A, tmp)
    oracle_mod.active_gather(A, inv, None, B, tmp)
    assert np.array_equal(B, W)


def test_gather_rejects_out_of_range(oracle_mod):
    W = gi.gen_normal_bf16(10, 8, 5, 1.0)
    A = np.zeros((4, 8), dtype=np.uint16)
    t = np.zeros((4,), dtype=np.int32)
    with pytest.raises(ValueError):
        oracle_mod.active_gather(W, np.array([10], dtype=np.int32), None, A, t)
    with pytest.raises(ValueError):
        oracle_mod.active_gather(W, np.array([1], dtype=np.int32), np.array([4], dtype=np.int32), A, t)


# ------------------------------------------------------------ segmented variant
def test_segmented_equals_definition_on_each_union(oracle_mod):
    V, d, S, n_core, n_arc, k = 400, 32, 3, 60, 12, 5
    W = gi.gen_normal_bf16(V, d, 7, 0.5, block_rows=64)
    core, arcs = gi.batched_ids(V, n_core, n_arc, S, seed=9)
    row_off = np.array([0, 4, 4, 9], dtype=np.int32)           # middle sequence is empty
    h = gi.gen_h(9, d, 8)
    W_arc = np.stack([W[arcs[s]] for s in range(S)])
    vals, oid, lz = oracle_mod.active_lmhead_topk_segmented(h, W[core], core, W_arc, arcs, row_off, k)
    z_def = f64(h) @ f64(W).T
    from scipy.special import logsumexp
    for s in range(S):
        union = np.concatenate([core, arcs[s]])
        assert np.unique(union).shape[0] == union.shape[0]
        for m in range(row_off[s], row_off[s + 1]):
            ev, ei = np_topk(z_def[m][union], union, k)
            assert np.array_equal(oid[m], ei)
            np.testing.assert_allclose(vals[m], ev, rtol=0, atol=1e-12)
            assert abs(lz[m] - logsumexp(z_def[m][union])) < 1e-12


# ------------------------------------------------------------ synthetic-data sanity
def test_synthetic_logz_matches_gaussian_closed_form(oracle_mod):
    """With W ~ N(0, 0.02^2) the logits of a row are ~N(0, s^2), s^2 = 4e-4 |h|^2, so
    logZ ~ ln V_act + s^2/2 (log-normal mean).  A sanity bound, not a parity check."""
    V_act, d, M = 4096, 512, 4
    W = gi.gen_normal_bf16(V_act, d, 77, 0.02)
    h = gi.gen_h(M, d, 78)
    _, _, lz = oracle_mod.active_lmhead_topk(h, W, None, 1)
    s2 = 4e-4 * (f64(h) ** 2).sum(axis=1)
    np.testing.assert_allclose(lz, math.log(V_act) + s2 / 2, rtol=0, atol=0.02)
