"""Plain reference of the dynamic-buffer manager (test infrastructure, not the product).

What it follows: the EvoSpec paper's appendix paragraphs "ARC-based dynamic vocabulary
maintenance" and "Additional safeguards" and the hyper-parameter table (capacity 256, initial
target p = 128 kept in [0, capacity], ghost lists of 256 each, at most 32 insertions per failure
event, a minimum residency of 8 decoding steps before eviction, the target frozen during the
first 50 events), on top of the textbook Adaptive Replacement Cache (recent list T1, frequent
list T2, ghost lists B1 and B2).

Everything is a Python list ordered from least to most recently used; every operation is a linear
scan.  Only tests, the smoke check and the benchmark's CPU leg may import this module.

Readings where the paper is silent (the same ones the C++ manager takes):
  * the request stream is the de-duplicated candidate list of a failure event, in the given
    order, minus tokens of the static core; `touch` feeds extra hits on resident tokens;
  * a candidate found in a ghost list adapts p the textbook way (by max(1, |other ghost| /
    |this ghost|), integer division) once the warm-up is over, and re-enters at T2;
  * when the buffer is full the victim is the least recently used token of T1 if |T1| > p, else of
    T2, that has been resident for the minimum number of decoding steps; if the chosen list has
    none, the other list is searched; if no token qualifies, the candidate is dropped and
    nothing changes;
  * the candidate leaves its ghost list before its victim enters one (and the ghost list is
    trimmed to its capacity);
  * a candidate beyond the insertion cap is dropped without touching p or the ghost lists;
  * a new token takes the slot its victim leaves, or the next unused slot while the buffer is
    filling, so the used slots stay dense; slots are reported with `slot_base` added.
"""
from __future__ import annotations


class ArcOracle:
    def __init__(self, capacity=256, p0=128, ghost_cap=256, max_insert=32, min_residency=8,
                 warmup_events=50, slot_base=0, core=()):
        assert capacity >= 1 and 0 <= p0 <= capacity and ghost_cap >= 0 and max_insert >= 0
        self.c, self.p, self.ghost_cap = capacity, p0, ghost_cap
        self.max_insert, self.min_res, self.warmup = max_insert, min_residency, warmup_events
        self.slot_base = slot_base
        self.core = set(int(x) for x in core)
        self.T1, self.T2, self.B1, self.B2 = [], [], [], []     # LRU ... MRU
        self.slot, self.born = {}, {}                           # resident token -> slot, insertion step
        self.step, self.events = 0, 0

    # ---- clock and extra hits
    def advance(self, steps=1):
        assert steps >= 0
        self.step += steps

    def touch(self, ids):
        for x in ids:
            x = int(x)
            if x in self.T1:
                self.T1.remove(x)
                self.T2.append(x)
            elif x in self.T2:
                self.T2.remove(x)
                self.T2.append(x)

    # ---- one failure event
    def _victim(self):
        order = (self.T1, self.T2) if len(self.T1) > self.p else (self.T2, self.T1)
        for lst in order:
            for tok in lst:                                     # from the LRU end
                if self.step - self.born[tok] >= self.min_res:
                    return tok, lst
        return None, None

    def event(self, candidates):
        """Returns the list of (slot, id) writes this event causes, in insertion order."""
        self.events += 1
        adapt = self.events > self.warmup
        seen, cands = set(), []
        for x in candidates:
            x = int(x)
            if x < 0 or x in self.core or x in seen:
                continue
            seen.add(x)
            cands.append(x)
        writes = []
        for x in cands:
            if x in self.T1:
                self.T1.remove(x)
                self.T2.append(x)
                continue
            if x in self.T2:
                self.T2.remove(x)
                self.T2.append(x)
                continue
            if len(writes) >= self.max_insert:
                continue
            full = len(self.T1) + len(self.T2) >= self.c
            if full and self._victim()[0] is None:
                continue
            in_b1, in_b2 = x in self.B1, x in self.B2
            if adapt and in_b1:
                self.p = min(self.c, self.p + max(1, len(self.B2) // len(self.B1)))
            if adapt and in_b2:
                self.p = max(0, self.p - max(1, len(self.B1) // len(self.B2)))
            if in_b1:                                           # leaves its ghost list before the victim
                self.B1.remove(x)                               # enters one (the trim must not meet it)
            if in_b2:
                self.B2.remove(x)
            if full:
                v, lst = self._victim()
                lst.remove(v)
                ghost = self.B1 if lst is self.T1 else self.B2
                ghost.append(v)
                if len(ghost) > self.ghost_cap:
                    ghost.pop(0)
                s = self.slot.pop(v)
                del self.born[v]
            else:
                s = len(self.slot)
            (self.T2 if (in_b1 or in_b2) else self.T1).append(x)
            self.slot[x], self.born[x] = s, self.step
            writes.append((self.slot_base + s, x))
        return writes

    # ---- inspection
    def state(self):
        return {"p": self.p, "T1": list(self.T1), "T2": list(self.T2), "B1": list(self.B1), "B2": list(self.B2),
                "slots": {t: self.slot_base + s for t, s in self.slot.items()}, "step": self.step,
                "events": self.events}

    def resident(self):
        """(slot, id) of every resident token, by slot."""
        return sorted((self.slot_base + s, t) for t, s in self.slot.items())
