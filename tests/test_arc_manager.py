"""The C++ dynamic-buffer manager (through its C ABI) against the plain oracle: the same
hand-worked trace, and identical writes and state, event by event, on random request streams
with the paper's parameters.  Host only: no GPU needed."""
import ctypes

import numpy as np
import pytest

import evospec_inputs as gi
from oracle import ArcOracle
from test_arc_oracle import run_trace


@pytest.fixture(scope="module")
def ArcManager():
    import paper_2605_27390_amd as ev
    return ev.ArcManager


def test_hand_worked_trace(ArcManager):
    run_trace(ArcManager)


def same_state(a, b):
    sa, sb = a.state(), b.state()
    for key in ("p", "T1", "T2", "B1", "B2", "slots", "step", "events"):
        assert sa[key] == sb[key], key
    assert a.resident() == b.resident()


@pytest.mark.parametrize("params", [
    dict(),                                                      # the paper's setting
    dict(capacity=16, p0=3, ghost_cap=5, max_insert=4, min_residency=2, warmup_events=0, slot_base=7),
    dict(capacity=8, p0=8, ghost_cap=0, max_insert=8, min_residency=0, warmup_events=3),
    dict(capacity=32, p0=0, ghost_cap=64, max_insert=1, min_residency=5, warmup_events=10),
])
def test_matches_the_oracle_event_by_event(ArcManager, params):
    rng = np.random.default_rng(11)
    V = 4000
    core = gi.zipf_ranking(V, 5)[:300]
    a, b = ArcManager(core=core, **params), ArcOracle(core=core, **params)
    weights = gi.zipf_weights(V)
    weights = weights / weights.sum()
    perm = gi.zipf_ranking(V, 5)
    for ev in range(1500):
        n = int(rng.integers(0, 90))
        cands = perm[rng.choice(V, size=n, p=weights)]           # Zipf-distributed token ids, repeats included
        if ev % 97 == 0:
            cands = np.concatenate([cands, [-1, -7]]).astype(np.int32)
        assert a.event(cands) == b.event(cands), ev
        if ev % 10 == 0:
            same_state(a, b)
        steps = int(rng.integers(0, 4))
        a.advance(steps); b.advance(steps)
        if rng.random() < 0.3:
            t = perm[rng.choice(V, size=6, p=weights)]
            a.touch(t); b.touch(t)
    same_state(a, b)
    assert len(a.resident()) == params.get("capacity", 256)


def test_argument_errors(ArcManager):
    import paper_2605_27390_amd as ev
    L = ev.lib
    with pytest.raises(ev.EvospecError):
        ArcManager(capacity=0)
    with pytest.raises(ev.EvospecError):
        ArcManager(capacity=4, p0=5)
    m = ArcManager(capacity=4, p0=2, max_insert=2)
    n = ctypes.c_int(0)
    assert L.evospec_arc_event(None, None, 0, None, None, ctypes.byref(n)) == 1
    assert L.evospec_arc_event(m._h, None, 3, None, None, ctypes.byref(n)) == 1
    assert L.evospec_arc_event(m._h, None, -1, None, None, ctypes.byref(n)) == 2
    assert L.evospec_arc_advance(m._h, -1) == 2
    assert L.evospec_arc_list(m._h, 4, None, 0, ctypes.byref(n)) == 2
    assert m.event([]) == [] and m.state()["events"] == 1


def test_candidate_formation_matches_the_oracle():
    import paper_2605_27390_amd as ev
    from oracle import form_candidates
    V = 6000
    row_ptr, col = gi.bigram_graph(V, 8)
    rng = np.random.default_rng(2)
    for trial in range(200):
        t = rng.integers(0, V, int(rng.integers(0, 12)))
        m = rng.integers(0, V, int(rng.integers(0, 12)))
        ms = int(rng.integers(0, 10))
        cap = int(rng.choice([4096, 5, 25, 0]))
        assert ev.form_candidates(t, m, row_ptr, col, V, ms, cap) == form_candidates(t, m, row_ptr, col, ms, cap), trial
    # the hand-worked case of the oracle's pins
    rp = np.array([0, 3, 3, 7, 8, 8, 8, 8, 8, 8, 8], dtype=np.int64)
    ci = np.array([5, 6, 7, 6, 0, 9, 8, 1], dtype=np.int32)
    assert ev.form_candidates([2, 0], [0, 3], rp, ci, 10, 2) == [2, 0, 3, 6, 5, 1]
    # seeds outside the vocabulary are dropped
    assert ev.form_candidates([2, 10, -1], [3], rp, ci, 10, 0) == [2, 3]
    # no successors asked for: the graph may be absent altogether
    assert ev.form_candidates([2, 0], [0, 3], None, None, 10, 0) == [2, 0, 3]
    L = ev.lib
    n = ctypes.c_int(0)
    seeds = (ctypes.c_int32 * 2)(2, 0)
    out = (ctypes.c_int32 * 8)()
    assert L.evospec_form_candidates(seeds, 2, None, 0, None, None, 10, 0, out, 8, ctypes.byref(n)) == 0 and n.value == 2
    assert L.evospec_form_candidates(seeds, 2, None, 0, None, None, 10, 3, out, 8, ctypes.byref(n)) == 1   # graph needed
    # successors outside the vocabulary never become candidates (they could not be gathered)
    ci_bad = np.array([5, 60, -7, 6, 0, 9, 8, 1], dtype=np.int32)
    assert ev.form_candidates([0], [], rp, ci_bad, 10, 3) == [0, 5]


def test_get_config_round_trip(ArcManager):
    import paper_2605_27390_amd as ev
    m = ArcManager(capacity=16, p0=3, ghost_cap=5, max_insert=4, min_residency=2, warmup_events=0, slot_base=7)
    cfg = ev.arc._Config()
    assert ev.lib.evospec_arc_get_config(ctypes.c_void_p(m._h) if not isinstance(m._h, ctypes.c_void_p) else m._h, ctypes.byref(cfg)) == 0
    assert (cfg.capacity, cfg.p0, cfg.ghost_capacity, cfg.max_insert, cfg.min_residency, cfg.warmup_events, cfg.slot_base) == (16, 3, 5, 4, 2, 0, 7)
    assert ev.lib.evospec_arc_get_config(None, ctypes.byref(cfg)) == 1
