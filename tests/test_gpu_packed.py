"""GPU parity of the packed (operand-tile) layout of the compact active matrix: the gather that
writes it, bit for bit against the oracle's gather after undoing the documented permutation, and
every head entry point on a packed matrix against the fp64 oracle and against the same call on the
row-major matrix.  Needs an MI355X: run with `-m gpu`."""
import numpy as np
import pytest

import evospec_inputs as gi
from helpers import NAN_BITS, bf16_dev_to_bits, check_head, new_matrix, to_dev_bf16, to_dev_i32, unpack_bits
from test_gpu_parity import ev, problem  # noqa: F401  (fixture and helper)

pytestmark = pytest.mark.gpu



def new_packed(ev, rows, d, batch=None):
    return new_matrix(ev, rows, d, "packed", batch=batch)


def pack(ev, W_bits, batch=None):
    """Packed copy of a row-major matrix (numpy bf16 bits), through the library's gather."""
    import torch
    if batch is None:
        rows, d = W_bits.shape
        P = new_packed(ev, rows, d)
        scratch_ids = torch.empty((max(rows, 1),), dtype=torch.int32, device="cuda")
        if rows:
            ev.active_gather(to_dev_bf16(W_bits), to_dev_i32(np.arange(rows)), None, P, scratch_ids[:rows])
        return P
    S, rows, d = W_bits.shape
    P = new_packed(ev, rows, d, batch=S)
    for s in range(S):
        if rows:
            scratch_ids = torch.empty((rows,), dtype=torch.int32, device="cuda")
            ev.active_gather(to_dev_bf16(W_bits[s]), to_dev_i32(np.arange(rows)), None, P.sub(s), scratch_ids)
    return P


def run_head_packed(ev, h, W, ids, k):
    import torch
    v, i, l = ev.active_lmhead_topk(to_dev_bf16(h), pack(ev, W), None if ids is None else to_dev_i32(ids), k)
    torch.cuda.synchronize()
    return v.cpu().numpy(), i.cpu().numpy(), l.cpu().numpy()


def run_head_rows(ev, h, W, ids, k):
    import torch
    v, i, l = ev.active_lmhead_topk(to_dev_bf16(h), to_dev_bf16(W), None if ids is None else to_dev_i32(ids), k)
    torch.cuda.synchronize()
    return v.cpu().numpy(), i.cpu().numpy(), l.cpu().numpy()


# ------------------------------------------------------------------ gather
@pytest.mark.parametrize("V_act,d", [(600, 256), (37, 72), (16, 8), (1, 520), (1000, 4096)])
def test_packed_gather_full_and_incremental_bit_exact(ev, oracle_mod, V_act, d):
    import torch
    V = 3 * V_act + 50
    W = gi.gen_normal_bf16(V, d, 5, 0.05)
    rng = np.random.default_rng(V_act)
    ids = rng.choice(V, size=V_act, replace=False).astype(np.int32)
    Wd = to_dev_bf16(W)
    P = new_packed(ev, V_act, d)
    act_ids = torch.full((V_act,), -7, dtype=torch.int32, device="cuda")
    ev.active_gather(Wd, to_dev_i32(ids), None, P, act_ids)
    torch.cuda.synchronize()
    ref_W, ref_ids = np.zeros((V_act, d), np.uint16), np.full(V_act, -7, np.int32)
    oracle_mod.active_gather(W, ids, None, ref_W, ref_ids)
    got, full = unpack_bits(bf16_dev_to_bits(P.data), V_act, d)
    assert np.array_equal(got, ref_W) and np.array_equal(act_ids.cpu().numpy(), ref_ids)
    assert np.all(full[0, :V_act, d:] == 0), "pad elements of written rows are zero"
    assert np.all(full[0, V_act:, :] == NAN_BITS), "rows past V_act are never written"
    for step in range(3):                                   # scattered updates: single rows into tiles
        n = min(V_act, 1 + 13 * step)
        slots = rng.choice(V_act, size=n, replace=False).astype(np.int32)
        new_ids = rng.choice(V, size=n, replace=False).astype(np.int32)
        ev.active_gather(Wd, to_dev_i32(new_ids), to_dev_i32(slots), P, act_ids)
        torch.cuda.synchronize()
        oracle_mod.active_gather(W, new_ids, slots, ref_W, ref_ids)
        got, full = unpack_bits(bf16_dev_to_bits(P.data), V_act, d)
        assert np.array_equal(got, ref_W) and np.array_equal(act_ids.cpu().numpy(), ref_ids)
        assert np.all(full[0, :V_act, d:] == 0) and np.all(full[0, V_act:, :] == NAN_BITS)
    # a rebuild of the first rows only must leave the others alone, also inside a shared tile
    m = max(1, V_act // 3)
    ev.active_gather(Wd, to_dev_i32(ids[:m].copy()), None, P, act_ids)
    torch.cuda.synchronize()
    oracle_mod.active_gather(W, ids[:m].copy(), None, ref_W, ref_ids)
    got, _ = unpack_bits(bf16_dev_to_bits(P.data), V_act, d)
    assert np.array_equal(got, ref_W) and np.array_equal(act_ids.cpu().numpy(), ref_ids)


def test_packed_gather_skips_out_of_range_entries(ev):
    import torch
    W = gi.gen_normal_bf16(20, 16, 3, 1.0)
    P = new_packed(ev, 8, 16)
    act_ids = torch.full((8,), -1, dtype=torch.int32, device="cuda")
    src = np.array([3, -1, 20, 5, 7], dtype=np.int32)
    slots = np.array([0, 1, 2, 8, 4], dtype=np.int32)          # id -1, id 20 and slot 8 are out of range
    ev.active_gather(to_dev_bf16(W), to_dev_i32(src), to_dev_i32(slots), P, act_ids)
    ev.active_gather(to_dev_bf16(W), to_dev_i32(np.array([-5, 6, 99], dtype=np.int32)), None, P, act_ids)   # rebuild path
    torch.cuda.synchronize()
    got, _ = unpack_bits(bf16_dev_to_bits(P.data), 8, 16)
    assert act_ids.cpu().numpy().tolist() == [3, 6, -1, -1, 7, -1, -1, -1]
    assert np.array_equal(got[0], W[3]) and np.array_equal(got[1], W[6]) and np.array_equal(got[4], W[7])
    for r in (2, 3, 5, 6, 7):
        assert np.all(got[r] == NAN_BITS)


# ------------------------------------------------------------------ head on a packed matrix
@pytest.mark.parametrize("M,V_act,d,k", [
    (60, 2309, 512, 10),       # several slabs and a ragged tail (not a multiple of 16 either)
    (1, 1, 8, 1),              # one row, one piece
    (17, 15, 72, 5),           # less than a tile, hidden size far from a chunk
    (64, 16, 256, 16),         # exactly a tile, k == V_act
    (33, 145, 264, 10),        # a slab and one row, d one piece past a chunk
    (3, 9216 + 5, 128, 10),    # many slabs, few draft rows
    (100, 1000, 1000, 10),     # two 64-row passes
    (60, 777, 4096, 64),       # the benchmark's hidden size, largest k
    (129, 1000, 256, 10),      # large-M path: a draft-row tile with a tail, 4 active-row tiles with a tail
    (257, 257, 64, 5),         # one row past a tile both ways, a single pair of chunks
    (300, 100, 192, 10),       # second half of the only active-row tile wholly empty
    (200, 5, 64, 5),           # k == V_act on the large-M path
    (512, 777, 4096, 10),
    (130, 40, 320, 33),
])
def test_packed_head_matches_oracle_and_row_major(ev, oracle_mod, M, V_act, d, k):
    W, h, ids = problem(900 + M + V_act, V_act, d, M)
    v, i, l = run_head_packed(ev, h, W, ids, k)
    check_head(v, i, l, oracle_mod.logits(h, W), ids, k, f"packed M={M} V_act={V_act} d={d} k={k}")
    # the layout changes where the operands come from, not the order of the arithmetic
    v0, i0, l0 = run_head_rows(ev, h, W, ids, k)
    assert np.array_equal(v, v0) and np.array_equal(i, i0) and np.array_equal(l, l0)


@pytest.mark.parametrize("M", [40, 261])
def test_packed_exact_small_integers(ev, M):
    """Operands whose products and sums are exact in fp32: the logits must match exactly, which
    pins the packed layout (row / piece / k-step mapping) bit for bit on both kernels."""
    rng = np.random.default_rng(5 + M)
    V_act, d, k = 391, 328, 7
    Wf = rng.integers(-4, 5, size=(V_act, d)).astype(np.float32)
    hf = rng.integers(-4, 5, size=(M, d)).astype(np.float32)
    if M > 128:
        d = 320
        Wf, hf = Wf[:, :d].copy(), hf[:, :d].copy()
    W, h = gi.f32_to_bf16_bits(Wf), gi.f32_to_bf16_bits(hf)
    ids = rng.permutation(5000)[:V_act].astype(np.int32)
    v, i, l = run_head_packed(ev, h, W, ids, k)
    z = hf.astype(np.float64) @ Wf.astype(np.float64).T
    for m in range(M):
        order = sorted(range(V_act), key=lambda j: (-z[m, j], ids[j]))[:k]
        assert i[m].tolist() == [int(ids[j]) for j in order], f"row {m}"
        assert v[m].tolist() == [float(z[m, j]) for j in order], f"row {m}"


def test_packed_identity_ids_and_all_equal_logits(ev, oracle_mod):
    W, h, ids = problem(43, 600, 256, 50)
    v, i, l = run_head_packed(ev, h, W, None, 10)
    check_head(v, i, l, oracle_mod.logits(h, W), np.arange(600, dtype=np.int32), 10, "ids=None")
    h[:] = 0                                                  # every logit 0: the k smallest ids, exactly
    v, i, l = run_head_packed(ev, h, W, ids, 10)
    assert np.all(i == np.sort(ids)[:10][None, :]) and np.all(v == 0)
    np.testing.assert_allclose(l, np.log(600.0), rtol=1e-6)


def test_packed_split_halves_equal_the_fused_call(ev):
    import torch
    W, h, ids = problem(44, 3000, 512, 60)
    P, hd, idd = pack(ev, W), to_dev_bf16(h), to_dev_i32(ids)
    k = 10
    v0, i0, l0 = ev.active_lmhead_topk(hd, P, idd, k)
    ws = torch.empty(ev.workspace_bytes(60, 3000, 512, k), dtype=torch.uint8, device="cuda")
    v1 = torch.empty_like(v0); i1 = torch.empty_like(i0); l1 = torch.empty_like(l0)
    ev.active_lmhead_partials(hd, P, idd, k, ws)
    ev.active_lmhead_merge(60, 3000, 512, k, v1, i1, l1, ws)
    torch.cuda.synchronize()
    assert torch.equal(v0, v1) and torch.equal(i0, i1) and torch.equal(l0, l1)


@pytest.mark.parametrize("M,n_new", [(20, 32), (70, 5), (130, 40), (5, 0)])
def test_packed_head_then_update_equals_the_two_calls(ev, M, n_new):
    import torch
    V, d, n_core, n_arc, k = 4000, 256, 700, 100, 10
    W = gi.gen_W_lm(V, d)
    ids = np.concatenate(gi.core_arc_ids(V, n_core, n_arc, seed=6))
    h = to_dev_bf16(gi.gen_h(M, d, 40 + M))
    Wd = to_dev_bf16(W)
    mats = []
    for _ in range(2):
        P = new_packed(ev, ids.shape[0], d)
        act = torch.empty((ids.shape[0],), dtype=torch.int32, device="cuda")
        ev.active_gather(Wd, to_dev_i32(ids), None, P, act)
        mats.append((P, act))
    slots, new_ids = gi.arc_update(V, ids, n_core, max(n_new, 1), seed=50 + M)
    slots, new_ids = slots[:n_new], new_ids[:n_new]
    sd, nd = to_dev_i32(slots), to_dev_i32(new_ids)
    v0, i0, l0 = ev.active_lmhead_topk(h, mats[0][0], mats[0][1], k)
    ev.active_gather(Wd, nd, sd, mats[0][0], mats[0][1])
    v1, i1, l1 = ev.active_lmhead_topk_then_update(h, mats[1][0], mats[1][1], k, Wd, nd, sd)
    torch.cuda.synchronize()
    assert torch.equal(v0, v1) and torch.equal(i0, i1) and torch.equal(l0, l1)
    assert torch.equal(mats[0][0].data.view(torch.int16), mats[1][0].data.view(torch.int16))
    want = ids.copy(); want[slots] = new_ids
    assert np.array_equal(mats[1][1].cpu().numpy(), want)
    got, _ = unpack_bits(bf16_dev_to_bits(mats[1][0].data), ids.shape[0], d)
    assert np.array_equal(got, W[want])


# ------------------------------------------------------------------ segmented variant
def seg_check_packed(ev, oracle_mod, V, d, S, n_core, n_arc, row_off, k, seed):
    import torch
    W = gi.gen_normal_bf16(V, d, seed, 0.05)
    core, arcs = gi.batched_ids(V, max(n_core, 1), max(n_arc, 1), S, seed=seed + 1)
    core, arcs = core[:n_core], arcs[:, :n_arc]
    M = int(row_off[-1])
    h = gi.gen_h(M, d, seed + 2)
    W_core = pack(ev, W[core])
    W_arc = pack(ev, np.stack([W[arcs[s]] for s in range(S)]), batch=S)
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


def test_packed_segmented(ev, oracle_mod):
    # 64-row passes: empty, 70-row (crosses a pass) and 1-row sequences; extensions of 150 rows (padded tiles)
    seg_check_packed(ev, oracle_mod, 6000, 256, 5, 1000, 150, np.array([0, 60, 60, 130, 131, 200], dtype=np.int32), 10, 7)
    seg_check_packed(ev, oracle_mod, 6000, 72, 3, 100, 37, np.array([0, 10, 40, 100], dtype=np.int32), 10, 8)
    # shared core on the large-M path, more than 64 chunks
    rng = np.random.default_rng(3)
    lens = rng.integers(0, 10, size=90)
    lens[5] = 70
    row_off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    seg_check_packed(ev, oracle_mod, 9000, 128, 90, 1500, 130, row_off, 10, 21)
    row_off = np.array([0, 100, 180, 300], dtype=np.int32)
    seg_check_packed(ev, oracle_mod, 5000, 64, 3, 0, 400, row_off, 10, 31)           # extensions only
    seg_check_packed(ev, oracle_mod, 5000, 64, 3, 700, 0, row_off, 10, 41)           # shared core only


# ------------------------------------------------------------------ Path-A event into a packed matrix
def test_packed_path_a_event(ev, oracle_mod):
    """Failure events through the native entry point with a packed W_act: admissions as the oracles
    derive them from the GPU's own neighbours, matrix and id list bit-exact afterwards."""
    import torch
    from oracle import ArcOracle, form_candidates
    V, d, n_core, cap = 5000, 128, 800, 64
    W = gi.gen_W_lm(V, d)
    core = gi.zipf_ranking(V, 31)[:n_core].astype(np.int32)
    row_ptr, col = gi.bigram_graph(V, 12)
    params = dict(capacity=cap, p0=cap // 2, ghost_cap=cap, max_insert=32, min_residency=1, warmup_events=2,
                  slot_base=n_core, core=core)
    arc, ref = ev.ArcManager(**params), ArcOracle(**params)
    Wd = to_dev_bf16(W)
    P = new_packed(ev, n_core + cap, d)
    act_ids = torch.full((n_core + cap,), -1, dtype=torch.int32, device="cuda")
    ev.active_gather(Wd, to_dev_i32(core), None, P, act_ids)
    ws = torch.empty(ev.path_a_workspace_bytes(V, d, 10, 32), dtype=torch.uint8, device="cuda")
    rng = np.random.default_rng(8)
    for e in range(12):
        hd = to_dev_bf16(gi.gen_h(1, d, 500 + e))
        target_top = rng.integers(0, V, 10).astype(np.int32)
        v, i, l = ev.active_lmhead_topk(hd, Wd, None, 10)
        got = ev.path_a_event(arc, hd, Wd, target_top, 10, row_ptr, col, 8, P, act_ids, ws)
        want = ref.event(form_candidates(target_top, i[0].cpu().numpy(), row_ptr, col, 8))
        assert got == want, e
        arc.advance(1); ref.advance(1)
    torch.cuda.synchronize()
    res = ref.resident()
    n_act = n_core + len(res)
    active = np.concatenate([core, np.array([t for _, t in res], dtype=np.int32)])
    assert np.array_equal(act_ids.cpu().numpy()[:n_act], active)
    got_W, _ = unpack_bits(bf16_dev_to_bits(P.data), n_core + cap, d)
    assert np.array_equal(got_W[:n_act], W[active])
    # and the head over the packed matrix sees exactly that active set
    h = gi.gen_h(7, d, 77)
    v, i, l = ev.active_lmhead_topk(to_dev_bf16(h), ev.PackedMatrix(n_act, d, data=P.data), act_ids[:n_act], 10)
    torch.cuda.synchronize()
    check_head(v.cpu().numpy(), i.cpu().numpy(), l.cpu().numpy(), oracle_mod.logits(h, W[active]), active, 10, "after events")


# ------------------------------------------------------------------ stream capture
def test_step_is_capturable_in_a_graph(ev, oracle_mod):
    """The calls allocate nothing and never synchronise, so a decode step (head + update behind it)
    can be captured in a HIP graph: every replay, with eager work and synchronisations in between,
    must reproduce the eager result bit for bit."""
    import torch
    V, d, n_core, n_arc, k, M = 4000, 256, 700, 100, 10, 60
    W = gi.gen_W_lm(V, d)
    ids = np.concatenate(gi.core_arc_ids(V, n_core, n_arc, seed=6))
    Wd = to_dev_bf16(W)
    P = new_packed(ev, ids.shape[0], d)
    act = torch.empty((ids.shape[0],), dtype=torch.int32, device="cuda")
    ev.active_gather(Wd, to_dev_i32(ids), None, P, act)
    slots, new_ids = gi.arc_update(V, ids, n_core, 32, seed=77)
    sd, nd = to_dev_i32(slots), to_dev_i32(new_ids)
    h = to_dev_bf16(gi.gen_h(M, d, 91))
    ws = torch.empty(ev.workspace_bytes(M, ids.shape[0], d, k), dtype=torch.uint8, device="cuda")
    ov = torch.empty((M, k), dtype=torch.float32, device="cuda")
    oi = torch.empty((M, k), dtype=torch.int32, device="cuda")
    ol = torch.empty((M,), dtype=torch.float32, device="cuda")

    def step():
        ev.active_lmhead_topk_then_update(h, P, act, k, Wd, nd, sd, ov, oi, ol, ws)

    step()                                         # eager: applies the update; later steps see the updated set
    step()
    torch.cuda.synchronize()
    want = (ov.clone(), oi.clone(), ol.clone())
    ref_ids = ids.copy(); ref_ids[slots] = new_ids
    check_head(ov.cpu().numpy(), oi.cpu().numpy(), ol.cpu().numpy(), oracle_mod.logits(gi.gen_h(M, d, 91), W[ref_ids]),
               ref_ids, k, "eager step on the updated set")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    for r in range(4):
        ov.zero_(); oi.zero_(); ol.zero_()         # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(ov, want[0]) and torch.equal(oi, want[1]) and torch.equal(ol, want[2]), f"replay {r}"
    assert np.array_equal(act.cpu().numpy(), ref_ids)


def test_two_host_threads_on_their_own_streams(ev):
    """The library keeps no per-call state: two host threads, each with its own stream, workspace and
    outputs, can run heads on the same matrices at the same time (ctypes drops the GIL in a call)."""
    import threading
    import torch
    W, h, ids = problem(4242, 3000, 512, 60)
    P, idd = pack(ev, W), to_dev_i32(ids)
    hs = [to_dev_bf16(h), to_dev_bf16(h[::-1].copy())]
    k = 10
    want = []
    for t in range(2):
        v, i, l = ev.active_lmhead_topk(hs[t], P, idd, k)
        torch.cuda.synchronize()
        want.append((v.clone(), i.clone(), l.clone()))
    errors = []

    def worker(t):
        try:
            st = torch.cuda.Stream()
            with torch.cuda.stream(st):
                ws = torch.empty(ev.workspace_bytes(60, 3000, 512, k), dtype=torch.uint8, device="cuda")
                for _ in range(25):
                    v, i, l = ev.active_lmhead_topk(hs[t], P, idd, k, workspace=ws)
                    st.synchronize()
                    if not (torch.equal(v, want[t][0]) and torch.equal(i, want[t][1]) and torch.equal(l, want[t][2])):
                        errors.append(f"thread {t}: result differs")
                        return
        except Exception as exc:            # surfaced in the main thread
            errors.append(f"thread {t}: {exc!r}")

    threads = [threading.Thread(target=worker, args=(t,)) for t in range(2)]
    for th in threads:
        th.start()
    for th in threads:
        th.join(timeout=100)
    assert not any(th.is_alive() for th in threads), "a worker did not finish"
    assert not errors, errors
