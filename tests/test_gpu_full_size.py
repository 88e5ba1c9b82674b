"""GPU parity at the benchmark's full sizes (Qwen3-8B / EAGLE-2 shapes), in the launch
configuration bench.py times.  The oracle computes every logit at these sizes in seconds on the
host cores (OpenMP): every row of every configuration is checked against it (the batched case on all
960 rows in the packed layout, which bench.py times, and on a sample of rows per sequence in the other)."""
import numpy as np
import pytest

import evospec_inputs as gi
from helpers import bf16_dev_to_bits, check_head, matrix_bits, new_matrix, to_dev_bf16, to_dev_i32

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ev():
    import torch
    assert torch.cuda.is_available()
    import paper_2605_27390_amd as ev
    return ev


@pytest.fixture(scope="module")
def lm_head():
    """The full synthetic LM head (151,936 x 4,096 bf16), host bits and device tensor."""
    c = gi.CONFIGS["draft60"]
    bits = gi.gen_W_lm(c["V"], c["d"])
    return bits, to_dev_bf16(bits)


@pytest.mark.parametrize("layout", ["packed", "row_major"])
def test_draft60_step_with_update(ev, oracle_mod, lm_head, layout):
    """Config 2: gather of the 36,864-id active set, a 32-row ARC update, then the head -- the update
    once as its own call and once behind a head (the call bench.py times)."""
    import torch
    W_bits, W_lm = lm_head
    c = gi.CONFIGS["draft60"]
    V, d, M, k = c["V"], c["d"], c["M"], c["k"]
    ids = gi.active_ids("draft60")
    V_act = ids.shape[0]
    h = gi.gen_h(M, d, gi.SEED_H + 2)
    W_act = new_matrix(ev, V_act, d, layout)
    act_ids = torch.empty((V_act,), dtype=torch.int32, device="cuda")
    ev.active_gather(W_lm, to_dev_i32(ids), None, W_act, act_ids)
    slots, new_ids = gi.arc_update(V, ids, c["n_core"], 32, seed=7000)
    ev.active_gather(W_lm, to_dev_i32(new_ids), to_dev_i32(slots), W_act, act_ids)
    ref_ids = ids.copy()
    ref_ids[slots] = new_ids
    # the head on this state; behind it, in the same call, the next update
    slots2, new_ids2 = gi.arc_update(V, ref_ids, c["n_core"], 32, seed=7001)
    v, i, l = ev.active_lmhead_topk_then_update(to_dev_bf16(h), W_act, act_ids, k, W_lm, to_dev_i32(new_ids2),
                                                to_dev_i32(slots2))
    torch.cuda.synchronize()
    _, _, _, z = oracle_mod.active_lmhead_topk(h, W_bits[ref_ids], ref_ids, k, return_logits=True)
    st = check_head(v.cpu().numpy(), i.cpu().numpy(), l.cpu().numpy(), z, ref_ids, k, "draft60")
    assert st["max_abs_err"] < 1e-4
    assert st["exempt_rows"] < M // 2
    ref_ids[slots2] = new_ids2
    assert np.array_equal(act_ids.cpu().numpy(), ref_ids)
    assert ev.validate_ids(act_ids, V)
    # gathered rows are bit-exact: every row of the matrix after both updates
    assert np.array_equal(matrix_bits(W_act), W_bits[ref_ids])
    v, i, l = ev.active_lmhead_topk(to_dev_bf16(h), W_act, act_ids, k)
    torch.cuda.synchronize()
    _, _, _, z = oracle_mod.active_lmhead_topk(h, W_bits[ref_ids], ref_ids, k, return_logits=True)
    check_head(v.cpu().numpy(), i.cpu().numpy(), l.cpu().numpy(), z, ref_ids, k, "draft60 after the second update")


@pytest.mark.parametrize("layout", ["packed", "row_major"])
@pytest.mark.parametrize("M", [1, 4, 8])
def test_depth_expansion_rows(ev, oracle_mod, lm_head, M, layout):
    """Config 3: 16,384 core + 2,048 ARC ids, M in {1, 4, 8} rows, with a 256-row update."""
    import torch
    W_bits, W_lm = lm_head
    c = gi.CONFIGS["depth"]
    V, d, k = c["V"], c["d"], c["k"]
    ids = gi.active_ids("depth")
    V_act = ids.shape[0]
    assert V_act == 18432
    h = gi.gen_h(M, d, gi.SEED_H + 30 + M)
    W_act = new_matrix(ev, V_act, d, layout)
    act_ids = torch.empty((V_act,), dtype=torch.int32, device="cuda")
    ev.active_gather(W_lm, to_dev_i32(ids), None, W_act, act_ids)
    slots, new_ids = gi.arc_update(V, ids, c["n_core"], c["update_rows"], seed=7100 + M)
    ev.active_gather(W_lm, to_dev_i32(new_ids), to_dev_i32(slots), W_act, act_ids)
    ref_ids = ids.copy()
    ref_ids[slots] = new_ids
    v, i, l = ev.active_lmhead_topk(to_dev_bf16(h), W_act, act_ids, k)
    torch.cuda.synchronize()
    assert gi.checksum(matrix_bits(W_act)) == gi.checksum(W_bits[ref_ids])
    z = oracle_mod.logits(h, W_bits[ref_ids])
    check_head(v.cpu().numpy(), i.cpu().numpy(), l.cpu().numpy(), z, ref_ids, k, f"depth M={M}")


def test_full_vocabulary_head(ev, oracle_mod, lm_head):
    """Config 4: the unpruned head (ids = NULL, W_act = W_lm) -- also Eq. 1 as printed."""
    import torch
    W_bits, W_lm = lm_head
    c = gi.CONFIGS["fullvocab"]
    M, k = c["M"], c["k"]
    h = gi.gen_h(M, c["d"], gi.SEED_H + 4)
    v, i, l = ev.active_lmhead_topk(to_dev_bf16(h), W_lm, None, k)
    torch.cuda.synchronize()
    z = oracle_mod.logits(h, W_bits)
    check_head(v.cpu().numpy(), i.cpu().numpy(), l.cpu().numpy(), z, None, k, "fullvocab")
    # the same head on a packed copy of all of W_lm (1,056 slabs of 10 wavefronts): bit-identical
    W_p = new_matrix(ev, c["V"], c["d"], "packed")
    scratch_ids = torch.empty((c["V"],), dtype=torch.int32, device="cuda")
    ev.active_gather(W_lm, torch.arange(c["V"], dtype=torch.int32, device="cuda"), None, W_p, scratch_ids)
    vp, ip, lp = ev.active_lmhead_topk(to_dev_bf16(h), W_p, None, k)
    torch.cuda.synchronize()
    assert torch.equal(vp, v) and torch.equal(ip, i) and torch.equal(lp, l)
    del W_p, scratch_ids
    # the pruned head's logZ is below the full one, and its top-k is the full top-k filtered to active ids
    ids = gi.active_ids("draft60")
    v2, i2, l2 = ev.active_lmhead_topk(to_dev_bf16(h), to_dev_bf16(W_bits[ids]), to_dev_i32(ids), k)
    torch.cuda.synchronize()
    assert np.all(l2.cpu().numpy() < l.cpu().numpy())
    check_head(v2.cpu().numpy(), i2.cpu().numpy(), l2.cpu().numpy(), z[:, ids], ids, k, "pruned-vs-full")


@pytest.mark.parametrize("layout", ["packed", "row_major"])
def test_batched_serving(ev, oracle_mod, lm_head, layout):
    """Config 5: 16 sequences x 60 rows, shared 32,768-id core + 2,048 ARC ids per sequence.
    Packed layout: the oracle checks all 960 rows.  Row-major: 4 rows of every sequence (first, last
    and two inside) and id membership for the rest."""
    import torch
    W_bits, W_lm = lm_head
    c = gi.CONFIGS["batched"]
    V, d, M, k, S, rps = c["V"], c["d"], c["M"], c["k"], c["S"], c["rows_per_seq"]
    core, arcs = gi.batched_ids(V, c["n_core"], c["n_arc"], S)
    h = gi.gen_h(M, d, gi.SEED_H + 5)
    row_off = np.arange(S + 1, dtype=np.int32) * rps
    W_core = new_matrix(ev, core.shape[0], d, layout)
    ids_core = torch.empty((core.shape[0],), dtype=torch.int32, device="cuda")
    ev.active_gather(W_lm, to_dev_i32(core), None, W_core, ids_core)
    Va = arcs.shape[1]
    W_arc = new_matrix(ev, Va, d, layout, batch=S)
    ids_arc = torch.empty((S * Va,), dtype=torch.int32, device="cuda")
    for s in range(S):
        ev.active_gather(W_lm, to_dev_i32(arcs[s].copy()), None, W_arc.sub(s) if layout == "packed" else W_arc[s],
                         ids_arc[s * Va:(s + 1) * Va])
    v, i, l = ev.active_lmhead_topk_segmented(to_dev_bf16(h), W_core, ids_core, W_arc,
                                              ids_arc.view(S, Va), row_off, k)
    torch.cuda.synchronize()
    v, i, l = v.cpu().numpy(), i.cpu().numpy(), l.cpu().numpy()
    assert np.isfinite(v).all() and np.isfinite(l).all() and (i >= 0).all()
    for s in range(S):
        union = np.concatenate([core, arcs[s]])
        rows = row_off[s] + (np.arange(rps) if layout == "packed" else np.array([0, 17, 41, rps - 1]))
        z = oracle_mod.logits(h[rows], W_bits[union])
        check_head(v[rows], i[rows], l[rows], z, union, k, f"batched seq {s}")
        # every returned id of the sequence's other rows is at least a member of its own union
        member = np.zeros(V, dtype=bool)
        member[union] = True
        assert member[i[row_off[s]:row_off[s + 1]]].all()


@pytest.fixture(scope="module")
def lm_head_d2048():
    """The second synthetic LM head of the sweep (128,256 x 2,048 bf16, its own seed stream)."""
    bits = gi.gen_W_lm(128256, 2048, gi.SEED_W + 1)
    return bits, to_dev_bf16(bits)


@pytest.mark.parametrize("shape", gi.SWEEP, ids=lambda s: s[0])
def test_paper_active_set_sizes(ev, oracle_mod, lm_head, lm_head_d2048, shape):
    """The active-set sizes of the paper's own experiments (Table 1 and the default setting) and the
    d = 2048 shape: gather + head against the oracle on every logit, in the layout bench.py times."""
    import torch
    layout = "packed"
    name, d, V, n_core, n_arc, M, k = shape
    W_bits, W_lm = lm_head if d == 4096 else lm_head_d2048
    assert W_bits.shape == (V, d)
    core, arc = gi.core_arc_ids(V, n_core, n_arc, gi.SEED_IDS + 40)
    ids = np.concatenate([core, arc])
    h = gi.gen_h(M, d, gi.SEED_H + 60)
    W_act = new_matrix(ev, ids.shape[0], d, layout)
    act_ids = torch.empty((ids.shape[0],), dtype=torch.int32, device="cuda")
    ev.active_gather(W_lm, to_dev_i32(ids), None, W_act, act_ids)
    v, i, l = ev.active_lmhead_topk(to_dev_bf16(h), W_act, act_ids, k)
    torch.cuda.synchronize()
    assert np.array_equal(act_ids.cpu().numpy(), ids)
    z = oracle_mod.logits(h, W_bits[ids])
    check_head(v.cpu().numpy(), i.cpu().numpy(), l.cpu().numpy(), z, ids, k, name)
