"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle, element by element
on the same seeded inputs.  Needs an MI355X: run with `-m gpu`."""
import math

import numpy as np
import pytest

import evospec_inputs as gi
from helpers import bf16_dev_to_bits, check_head, to_dev_bf16, to_dev_i32

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ev():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2605_27390_amd as ev
    return ev


def run_head(ev, h, W_act, ids, k):
    import torch
    v, i, l = ev.active_lmhead_topk(to_dev_bf16(h), to_dev_bf16(W_act), None if ids is None else to_dev_i32(ids), k)
    torch.cuda.synchronize()
    return v.cpu().numpy(), i.cpu().numpy(), l.cpu().numpy()


def problem(seed, V_act, d, M, sigma=0.05, V=None):
    V = V or max(2 * V_act, V_act + 7)
    W = gi.gen_normal_bf16(V_act, d, seed, sigma, block_rows=256)
    h = gi.gen_h(M, d, seed + 1)
    ids = np.random.default_rng(seed).choice(V, size=V_act, replace=False).astype(np.int32)
    return W, h, ids


# ------------------------------------------------------------------ gather
def test_gather_full_and_incremental_bit_exact(ev, oracle_mod):
    import torch
    V, d, n_core, n_arc = 3000, 264, 500, 100
    W = gi.gen_W_lm(V, d)
    ids = np.concatenate(gi.core_arc_ids(V, n_core, n_arc, seed=4))
    Wd = to_dev_bf16(W)
    W_act = torch.zeros((600, d), dtype=torch.bfloat16, device="cuda")
    act_ids = torch.full((600,), -1, dtype=torch.int32, device="cuda")
    ev.active_gather(Wd, to_dev_i32(ids), None, W_act, act_ids)
    ref_W = np.zeros((600, d), dtype=np.uint16)
    ref_ids = np.full((600,), -1, dtype=np.int32)
    oracle_mod.active_gather(W, ids, None, ref_W, ref_ids)
    torch.cuda.synchronize()
    assert np.array_equal(bf16_dev_to_bits(W_act), ref_W)
    assert np.array_equal(act_ids.cpu().numpy(), ref_ids)
    assert ev.validate_ids(act_ids, V)
    for n_new in (1, 32, 100):
        slots, new_ids = gi.arc_update(V, ref_ids, n_core, n_new, seed=10 + n_new)
        ev.active_gather(Wd, to_dev_i32(new_ids), to_dev_i32(slots), W_act, act_ids)
        oracle_mod.active_gather(W, new_ids, slots, ref_W, ref_ids)
        torch.cuda.synchronize()
        assert np.array_equal(bf16_dev_to_bits(W_act), ref_W)
        assert np.array_equal(act_ids.cpu().numpy(), ref_ids)
    # empty update is a no-op; a partial rebuild (n < V_act) touches only the first n slots
    ev.active_gather(Wd, to_dev_i32(np.zeros(0, np.int32)), None, W_act, act_ids)
    ev.active_gather(Wd, to_dev_i32(ids[1:8].copy()), None, W_act, act_ids)
    oracle_mod.active_gather(W, ids[1:8].copy(), None, ref_W, ref_ids)
    torch.cuda.synchronize()
    assert np.array_equal(bf16_dev_to_bits(W_act), ref_W)
    assert not ev.validate_ids(act_ids, V)                 # the partial rebuild duplicated ids
    assert not ev.validate_ids(to_dev_i32(np.array([1, 2, V], np.int32)), V)


def test_gather_skips_out_of_range_entries(ev):
    import torch
    W = gi.gen_W_lm(64, 16)
    W_act = torch.zeros((8, 16), dtype=torch.bfloat16, device="cuda")
    act_ids = torch.full((8,), -1, dtype=torch.int32, device="cuda")
    src = np.array([5, 64, -1, 7], np.int32)
    slots = np.array([0, 1, 2, 8], np.int32)
    ev.active_gather(to_dev_bf16(W), to_dev_i32(src), to_dev_i32(slots), W_act, act_ids)
    torch.cuda.synchronize()
    out = bf16_dev_to_bits(W_act)
    assert np.array_equal(out[0], W[5]) and not out[1:].any()
    assert act_ids.cpu().numpy().tolist() == [5, -1, -1, -1, -1, -1, -1, -1]


# ------------------------------------------------------------------ head, small shapes
def test_tiny_config(ev, oracle_mod):
    c = gi.CONFIGS["tiny"]
    W = gi.gen_W_lm(c["V"], c["d"])
    h = gi.gen_h(c["M"], c["d"], gi.SEED_H + 1)
    ids = gi.active_ids("tiny")
    import torch
    Wd = to_dev_bf16(W)
    W_act = torch.empty((ids.shape[0], c["d"]), dtype=torch.bfloat16, device="cuda")
    act_ids = torch.empty((ids.shape[0],), dtype=torch.int32, device="cuda")
    ev.active_gather(Wd, to_dev_i32(ids), None, W_act, act_ids)
    v, i, l = ev.active_lmhead_topk(to_dev_bf16(h), W_act, act_ids, c["k"])
    torch.cuda.synchronize()
    _, _, _, z = oracle_mod.active_lmhead_topk(h, W[ids], ids, c["k"], return_logits=True)
    st = check_head(v.cpu().numpy(), i.cpu().numpy(), l.cpu().numpy(), z, ids, c["k"], "tiny")
    assert st["max_abs_err"] < 1e-5


@pytest.mark.parametrize("M", [1, 3, 16, 17, 33, 60, 64, 65, 130])
def test_draft_row_counts(ev, oracle_mod, M):
    W, h, ids = problem(100 + M, 777, 264, M)
    k = 10
    v, i, l = run_head(ev, h, W, ids, k)
    z = oracle_mod.logits(h, W)
    check_head(v, i, l, z, ids, k, f"M={M}")


@pytest.mark.parametrize("V_act", [10, 63, 64, 65, 143, 144, 145, 1000, 2309, 9216 + 5])
def test_active_set_sizes_span_slabs_and_ragged_tails(ev, oracle_mod, V_act):
    W, h, ids = problem(200 + V_act, V_act, 512, 60)
    k = 10
    v, i, l = run_head(ev, h, W, ids, k)
    z = oracle_mod.logits(h, W)
    check_head(v, i, l, z, ids, k, f"V_act={V_act}")


@pytest.mark.parametrize("d", [8, 40, 256, 264, 1000, 4096])
def test_hidden_sizes(ev, oracle_mod, d):
    W, h, ids = problem(300 + d, 500, d, 20, sigma=1.0 / math.sqrt(d))
    k = 7
    v, i, l = run_head(ev, h, W, ids, k)
    z = oracle_mod.logits(h, W)
    check_head(v, i, l, z, ids, k, f"d={d}")


@pytest.mark.parametrize("k", [1, 2, 10, 32, 64])
def test_k_values(ev, oracle_mod, k):
    W, h, ids = problem(400 + k, 1500, 128, 33)
    v, i, l = run_head(ev, h, W, ids, k)
    z = oracle_mod.logits(h, W)
    check_head(v, i, l, z, ids, k, f"k={k}")


def test_k_equals_active_size_returns_every_logit(ev, oracle_mod):
    W, h, ids = problem(77, 48, 64, 9)
    v, i, l = run_head(ev, h, W, ids, 48)
    z = oracle_mod.logits(h, W)
    st = check_head(v, i, l, z, ids, 48, "k=V_act")
    for m in range(9):
        assert sorted(i[m].tolist()) == sorted(ids.tolist())
    assert st["max_abs_err"] < 1e-5


def test_identity_ids_when_null(ev, oracle_mod):
    W, h, _ = problem(78, 300, 64, 5)
    v, i, l = run_head(ev, h, W, None, 6)
    z = oracle_mod.logits(h, W)
    check_head(v, i, l, z, None, 6, "ids=NULL")


# ------------------------------------------------------------------ exact cases
def test_zero_hidden_state_is_exact(ev):
    W, _, ids = problem(79, 1000, 256, 4)
    h0 = np.zeros((4, 256), dtype=np.uint16)
    k = 10
    v, i, l = run_head(ev, h0, W, ids, k)
    assert np.all(v == 0.0)
    smallest = np.sort(ids)[:k]
    for m in range(4):
        assert np.array_equal(i[m], smallest)            # every logit ties: ascending full-vocab id
    np.testing.assert_allclose(l, math.log(1000), rtol=2e-6)


def test_one_hot_hidden_state_is_exact(ev):
    W, _, ids = problem(80, 900, 264, 1)
    one = gi.f32_to_bf16_bits(np.array([1.0], dtype=np.float32))[0]
    Wf = gi.bf16_bits_to_f32(W)
    for j in (0, 7, 130, 263):
        h1 = np.zeros((3, 264), dtype=np.uint16)
        h1[1, j] = one
        v, i, l = run_head(ev, h1, W, ids, 5)
        order = np.lexsort((ids, -Wf[:, j].astype(np.float64)))[:5]
        assert np.array_equal(v[1], Wf[order, j])         # zero tolerance: the column itself
        assert np.array_equal(i[1], ids[order])
        assert np.all(v[0] == 0.0) and np.all(v[2] == 0.0)


def test_exact_ties_order_by_full_vocab_id(ev):
    W, h, _ = problem(81, 400, 64, 6)
    ids = np.random.default_rng(3).permutation(5000)[:400].astype(np.int32)
    # 30 copies of one strong row scattered over several 16-row groups and slabs
    strong = gi.f32_to_bf16_bits(gi.bf16_bits_to_f32(h[0]) * 0.25)
    where = np.random.default_rng(4).choice(400, size=30, replace=False)
    W[where] = strong
    v, i, l = run_head(ev, h, W, ids, 12)
    want = np.sort(ids[where])[:12]
    assert np.array_equal(i[0], want)
    assert np.all(v[0] == v[0][0])


def test_bit_identical_across_launches(ev):
    import torch
    W, h, ids = problem(82, 5000, 512, 60)
    hd, Wd, idd = to_dev_bf16(h), to_dev_bf16(W), to_dev_i32(ids)
    ref = None
    for _ in range(5):
        v, i, l = ev.active_lmhead_topk(hd, Wd, idd, 10)
        torch.cuda.synchronize()
        cur = (v.cpu().numpy().tobytes(), i.cpu().numpy().tobytes(), l.cpu().numpy().tobytes())
        assert ref is None or cur == ref
        ref = cur


def test_split_halves_equal_the_fused_call(ev):
    import torch
    W, h, ids = problem(83, 3000, 256, 40)
    hd, Wd, idd = to_dev_bf16(h), to_dev_bf16(W), to_dev_i32(ids)
    k = 10
    v, i, l = ev.active_lmhead_topk(hd, Wd, idd, k)
    ws = torch.empty(ev.workspace_bytes(40, 3000, 256, k), dtype=torch.uint8, device="cuda")
    v2 = torch.empty_like(v)
    i2 = torch.empty_like(i)
    l2 = torch.empty_like(l)
    ev.active_lmhead_partials(hd, Wd, idd, k, ws)
    ev.active_lmhead_merge(40, 3000, 256, k, v2, i2, l2, ws)
    torch.cuda.synchronize()
    assert torch.equal(v, v2) and torch.equal(i, i2) and torch.equal(l, l2)


def test_order_of_active_ids_does_not_change_the_result(ev):
    W, h, ids = problem(84, 2000, 256, 30)
    v0, i0, l0 = run_head(ev, h, W, ids, 10)
    perm = np.random.default_rng(9).permutation(2000)
    v1, i1, l1 = run_head(ev, h, W[perm], ids[perm], 10)
    assert np.array_equal(i0, i1) and np.array_equal(v0, v1)
    np.testing.assert_allclose(l0, l1, rtol=1e-6)


# ------------------------------------------------------------------ segmented variant
def test_segmented_small(ev, oracle_mod):
    V, d, S, n_core, n_arc, k = 6000, 256, 5, 1000, 150, 10
    W = gi.gen_normal_bf16(V, d, 7, 0.05)
    core, arcs = gi.batched_ids(V, n_core, n_arc, S, seed=9)
    row_off = np.array([0, 60, 60, 130, 131, 200], dtype=np.int32)      # empty, 70-row (crosses a pass) and 1-row sequences
    h = gi.gen_h(200, d, 8)
    W_arc = np.stack([W[arcs[s]] for s in range(S)])
    import torch
    v, i, l = ev.active_lmhead_topk_segmented(to_dev_bf16(h), to_dev_bf16(W[core]), to_dev_i32(core),
                                              to_dev_bf16(W_arc), to_dev_i32(arcs), row_off, k)
    torch.cuda.synchronize()
    v, i, l = v.cpu().numpy(), i.cpu().numpy(), l.cpu().numpy()
    for s in range(S):
        r0, r1 = row_off[s], row_off[s + 1]
        if r1 == r0:
            continue
        union = np.concatenate([core, arcs[s]])
        z = oracle_mod.logits(h[r0:r1], W[union])
        check_head(v[r0:r1], i[r0:r1], l[r0:r1], z, union, k, f"seq {s}")
    ov, oi, ol = oracle_mod.active_lmhead_topk_segmented(h, W[core], core, W_arc, arcs, row_off, k)
    np.testing.assert_allclose(l, ol, rtol=1e-3)


# ------------------------------------------------------------------ dynamic buffer -> gather -> head
def test_arc_manager_drives_the_gather(ev, oracle_mod):
    """Failure events go through the C++ buffer manager, its (slot, id) writes through
    `active_gather`; the compact matrix must stay W_lm[ids] on every used slot and the head over
    core + buffer must match the oracle on that active set."""
    import torch
    V, d, n_core, cap, k = 3000, 64, 500, 64, 10
    W = gi.gen_W_lm(V, d)
    core = gi.zipf_ranking(V, 21)[:n_core].astype(np.int32)
    arc = ev.ArcManager(capacity=cap, p0=cap // 2, ghost_cap=cap, max_insert=32, min_residency=2, warmup_events=5,
                        slot_base=n_core, core=core)
    Wd = to_dev_bf16(W)
    W_act = torch.zeros((n_core + cap, d), dtype=torch.bfloat16, device="cuda")
    act_ids = torch.full((n_core + cap,), -1, dtype=torch.int32, device="cuda")
    ev.active_gather(Wd, to_dev_i32(core), None, W_act, act_ids)
    rng = np.random.default_rng(4)
    h = gi.gen_h(20, d, 77)
    for e in range(60):
        slots, ids = arc.event_arrays(rng.integers(0, V, size=int(rng.integers(1, 50))))
        if slots.size:
            ev.active_gather(Wd, to_dev_i32(ids.copy()), to_dev_i32(slots.copy()), W_act, act_ids)
        arc.advance(1)
        if e in (3, 30, 59):
            res = arc.resident()
            n_act = n_core + len(res)
            assert [s for s, _ in res] == list(range(n_core, n_act))
            active = np.concatenate([core, np.array([t for _, t in res], dtype=np.int32)])
            torch.cuda.synchronize()
            assert np.array_equal(act_ids.cpu().numpy()[:n_act], active)
            assert np.array_equal(bf16_dev_to_bits(W_act)[:n_act], W[active])
            assert ev.validate_ids(act_ids[:n_act], V)
            v, i, l = ev.active_lmhead_topk(to_dev_bf16(h), W_act[:n_act], act_ids[:n_act], k)
            torch.cuda.synchronize()
            check_head(v.cpu().numpy(), i.cpu().numpy(), l.cpu().numpy(), oracle_mod.logits(h, W[active]), active, k,
                       f"event {e}")
    assert len(arc.resident()) == cap


@pytest.mark.parametrize("max_insert", [32, 48])   # rows handed to the kernel by value / uploaded first
def test_path_a_event_end_to_end(ev, oracle_mod, max_insert):
    """A failure event through the native entry point (exact inner-product search on the GPU,
    candidate formation, admission, gather) against the same steps done by the oracles."""
    import torch
    from oracle import ArcOracle, exact_mips, form_candidates
    V, d, n_core, cap = 5000, 128, 800, 64
    W = gi.gen_W_lm(V, d)
    core = gi.zipf_ranking(V, 31)[:n_core].astype(np.int32)
    row_ptr, col = gi.bigram_graph(V, 12)
    params = dict(capacity=cap, p0=cap // 2, ghost_cap=cap, max_insert=max_insert, min_residency=1, warmup_events=2,
                  slot_base=n_core, core=core)
    arc, ref = ev.ArcManager(**params), ArcOracle(**params)
    Wd = to_dev_bf16(W)
    W_act = torch.zeros((n_core + cap, d), dtype=torch.bfloat16, device="cuda")
    act_ids = torch.full((n_core + cap,), -1, dtype=torch.int32, device="cuda")
    ev.active_gather(Wd, to_dev_i32(core), None, W_act, act_ids)
    ws = torch.empty(ev.path_a_workspace_bytes(V, d, 10, max_insert), dtype=torch.uint8, device="cuda")
    rng = np.random.default_rng(8)
    most = 0
    for e in range(12):
        h = gi.gen_h(1, d, 500 + e)
        target_top = rng.integers(0, V, 10).astype(np.int32)
        hd = to_dev_bf16(h)
        # the search alone, checked against the exact fp64 search (near-ties at the cut exempt)
        v, i, l = ev.active_lmhead_topk(hd, Wd, None, 10)
        torch.cuda.synchronize()
        z = oracle_mod.logits(h, W)
        check_head(v.cpu().numpy(), i.cpu().numpy(), l.cpu().numpy(), z, np.arange(V, dtype=np.int32), 10, f"search {e}")
        exact = exact_mips(h, W, 11)
        gap = abs(z[0, exact[9]] - z[0, exact[10]]) / max(abs(z[0, exact[9]]), abs(z[0, exact[10]]))
        if gap > 1e-3:
            assert set(i[0].cpu().numpy().tolist()) == set(exact[:10].tolist())
        # the event: its writes are what the oracles derive from the GPU's own neighbours
        got = ev.path_a_event(arc, hd, Wd, target_top, 10, row_ptr, col, 8, W_act, act_ids, ws)
        want = ref.event(form_candidates(target_top, i[0].cpu().numpy(), row_ptr, col, 8))
        assert got == want, e
        most = max(most, len(got))
        arc.advance(1); ref.advance(1)
    torch.cuda.synchronize()
    assert most > 32 or max_insert <= 32                      # the larger limit is actually used
    res = ref.resident()
    n_act = n_core + len(res)
    active = np.concatenate([core, np.array([t for _, t in res], dtype=np.int32)])
    assert np.array_equal(act_ids.cpu().numpy()[:n_act], active)
    assert np.array_equal(bf16_dev_to_bits(W_act)[:n_act], W[active])
    assert len(res) == cap


@pytest.mark.parametrize("M,n_new", [(20, 32), (64, 1), (70, 5), (130, 40), (5, 0)])
def test_head_then_update_equals_the_two_calls(ev, M, n_new):
    """The fused call must leave the outputs of the head on the old matrix and the matrix of the
    separate gather, bit for bit."""
    import torch
    V, d, n_core, n_arc, k = 4000, 256, 700, 100, 10
    W = gi.gen_W_lm(V, d)
    ids = np.concatenate(gi.core_arc_ids(V, n_core, n_arc, seed=6))
    h = to_dev_bf16(gi.gen_h(M, d, 40 + M))
    Wd = to_dev_bf16(W)
    mats = []
    for _ in range(2):
        W_act = torch.empty((ids.shape[0], d), dtype=torch.bfloat16, device="cuda")
        act = torch.empty((ids.shape[0],), dtype=torch.int32, device="cuda")
        ev.active_gather(Wd, to_dev_i32(ids), None, W_act, act)
        mats.append((W_act, act))
    slots, new_ids = gi.arc_update(V, ids, n_core, max(n_new, 1), seed=50 + M)
    slots, new_ids = slots[:n_new], new_ids[:n_new]
    sd, nd = to_dev_i32(slots), to_dev_i32(new_ids)
    v0, i0, l0 = ev.active_lmhead_topk(h, mats[0][0], mats[0][1], k)
    ev.active_gather(Wd, nd, sd, mats[0][0], mats[0][1])
    v1, i1, l1 = ev.active_lmhead_topk_then_update(h, mats[1][0], mats[1][1], k, Wd, nd, sd)
    torch.cuda.synchronize()
    assert torch.equal(v0, v1) and torch.equal(i0, i1) and torch.equal(l0, l1)
    assert torch.equal(mats[0][0].view(torch.int16), mats[1][0].view(torch.int16)) and torch.equal(mats[0][1], mats[1][1])
    want = ids.copy(); want[slots] = new_ids
    assert np.array_equal(mats[1][1].cpu().numpy(), want)
    assert np.array_equal(bf16_dev_to_bits(mats[1][0]), W[want])
