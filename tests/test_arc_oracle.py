"""Pins of the dynamic-buffer manager's oracle (no GPU): a trace worked by hand, special cases
that reduce to a plain LRU, and invariants under random request streams."""
import collections
import os

import numpy as np
import pytest

from oracle import ArcOracle

HERE = os.path.dirname(os.path.abspath(__file__))


def parse_list(s):
    s = s.strip()
    return [] if s in ("-", "") else [int(x) for x in s.split()]


def run_trace(make, path=os.path.join(HERE, "golden", "arc_worked_example.txt")):
    """Replays the hand-worked trace on a manager built by `make`; yields after every line."""
    arc = make(capacity=4, p0=2, ghost_cap=2, max_insert=3, min_residency=1, warmup_events=2, slot_base=100)
    n = 0
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        kind, rest = line[0], line[1:]
        if kind == "A":
            arc.advance(int(rest))
            continue
        f = [x.strip() for x in rest.split("|")]
        if kind == "E":
            writes = arc.event(parse_list(f[0]))
            want = [] if f[1] == "-" else [tuple(int(v) for v in w.split(":")) for w in f[1].split()]
            assert [tuple(w) for w in writes] == want, line
        else:
            arc.touch(parse_list(f[0]))
        st = arc.state()
        assert st["p"] == int(f[2]), line
        for name, col in zip(("T1", "T2", "B1", "B2"), f[3:7]):
            assert list(st[name]) == parse_list(col), (name, line)
        n += 1
    assert n == 8


def test_hand_worked_trace():
    run_trace(ArcOracle)


def lru_writes(stream, capacity):
    """Plain LRU cache with slot reuse: what the manager must do when nothing is ever promoted."""
    od, out = collections.OrderedDict(), []
    for x in stream:
        if x in od:
            continue                                            # (a repeat would promote: excluded by the caller)
        if len(od) >= capacity:
            _, s = od.popitem(last=False)
        else:
            s = len(od)
        od[x] = s
        out.append((s, x))
    return out


def test_reduces_to_lru_when_no_token_repeats():
    # all tokens distinct, one per event, target frozen at the capacity: T1 alone, oldest out
    rng = np.random.default_rng(3)
    stream = rng.permutation(5000)[:600].tolist()
    arc = ArcOracle(capacity=32, p0=0, ghost_cap=16, max_insert=1, min_residency=0, warmup_events=10**9)
    got = []
    for x in stream:
        got += arc.event([x])
    assert got == lru_writes(stream, 32)
    st = arc.state()
    assert st["T2"] == [] and st["T1"] == stream[-32:] and st["B1"] == stream[-48:-32] and st["B2"] == []


def test_second_hit_promotes_and_frequent_tokens_survive_a_scan():
    arc = ArcOracle(capacity=8, p0=4, ghost_cap=8, max_insert=8, min_residency=0, warmup_events=0)
    arc.event([1, 2, 3, 4])
    arc.event([1, 2, 3, 4])                                    # second hit: all four in T2
    assert arc.state()["T2"] == [1, 2, 3, 4] and arc.state()["T1"] == []
    for i in range(20):                                         # a scan of one-off tokens
        arc.event([100 + 8 * i + j for j in range(8)])
    st = arc.state()
    # the first eviction finds |T1| = 4 > p = 4 false and takes the LRU of T2; from then on
    # |T1| = 5 > p and the scan only ever evicts its own one-off tokens from T1
    assert st["T2"] == [2, 3, 4] and len(st["T1"]) == 5 and st["p"] == 4
    assert st["T1"] == [100 + 8 * 19 + j for j in range(3, 8)]


def test_ghost_hits_move_the_target_both_ways_and_respect_the_bounds():
    arc = ArcOracle(capacity=4, p0=2, ghost_cap=4, max_insert=4, min_residency=0, warmup_events=0)
    arc.event([1, 2, 3, 4])
    arc.event([5, 6])                                           # 1, 2 -> B1
    assert arc.state()["B1"] == [1, 2]
    arc.event([1])                                              # B1 hit: p 2 -> 3, 1 enters T2
    assert arc.state()["p"] == 3 and arc.state()["T2"] == [1]
    arc.event([2])                                              # B1 hit again: p -> 4 (the capacity)
    arc.event([3])                                              # 3 was evicted to B1 meanwhile: p stays at 4
    assert arc.state()["p"] == 4
    st = arc.state()
    assert set(st["T1"]) | set(st["T2"]) == set(st["slots"]) and len(st["slots"]) == 4
    # drive evictions from T2 so that B2 fills, then hit it: p comes down
    arc2 = ArcOracle(capacity=2, p0=2, ghost_cap=4, max_insert=4, min_residency=0, warmup_events=0)
    arc2.event([1, 2]); arc2.event([1, 2])                      # both in T2
    arc2.event([3])                                             # |T1| = 0 > 2 false -> evict 1 from T2 to B2
    assert arc2.state()["B2"] == [1]
    arc2.event([1])                                             # B2 hit: p = max(0, 2 - max(1, 0 // 1)) = 1
    assert arc2.state()["p"] == 1


def test_safeguards_cap_residency_warmup_core_and_dedup():
    arc = ArcOracle(capacity=8, p0=4, ghost_cap=8, max_insert=3, min_residency=2, warmup_events=3, core=[5, 6])
    w = arc.event([5, 1, 1, 6, 2, -4, 3, 4])                    # core ids, a duplicate and a negative id dropped; cap 3
    assert w == [(0, 1), (1, 2), (2, 3)]
    arc.event([4, 7, 8]); arc.event([9, 10])                    # full (8 residents), still step 0
    assert len(arc.state()["slots"]) == 8
    assert arc.event([11]) == []                                # nobody has been resident for 2 steps
    arc.advance(1)
    assert arc.event([11]) == []
    arc.advance(1)
    assert arc.event([11]) == [(0, 11)]                         # 1 (slot 0, LRU of T1) goes
    assert arc.state()["B1"] == [1]
    # events so far: 6 > warm-up of 3 -> a ghost hit adapts p now
    p_before = arc.state()["p"]
    arc.event([1])
    assert arc.state()["p"] == p_before + 1
    # within the warm-up nothing adapts
    a2 = ArcOracle(capacity=2, p0=1, ghost_cap=4, max_insert=4, min_residency=0, warmup_events=50)
    a2.event([1, 2]); a2.event([3]); a2.event([1])
    assert a2.state()["p"] == 1 and 1 in a2.state()["T2"]


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_invariants_under_random_streams(seed):
    rng = np.random.default_rng(seed)
    arc = ArcOracle(capacity=64, p0=32, ghost_cap=48, max_insert=32, min_residency=3, warmup_events=5,
                    slot_base=1000, core=range(10))
    shadow = {}                                                 # slot -> id, rebuilt from the writes alone
    for ev in range(400):
        n = int(rng.integers(0, 60))
        cands = (rng.zipf(1.3, size=n) % 700).tolist()
        writes = arc.event(cands)
        assert len(writes) <= 32 and len({s for s, _ in writes}) == len(writes)
        for s, x in writes:
            assert x not in shadow.values() or shadow.get(s) == x
            shadow[s] = x
        st = arc.state()
        T1, T2, B1, B2 = st["T1"], st["T2"], st["B1"], st["B2"]
        res = T1 + T2
        assert len(res) == len(set(res)) <= 64 and not (set(res) & set(B1 + B2)) and not (set(B1) & set(B2))
        assert len(B1) <= 48 and len(B2) <= 48 and 0 <= st["p"] <= 64
        assert not (set(res) & set(range(10)))
        # the writes alone reproduce the resident set, and the used slots are dense
        assert sorted(shadow.items()) == arc.resident()
        assert sorted(shadow) == list(range(1000, 1000 + len(res)))
        if rng.random() < 0.5:
            arc.advance(int(rng.integers(0, 3)))
        if rng.random() < 0.3 and res:
            arc.touch(rng.choice(res, size=min(4, len(res)), replace=False).tolist())
