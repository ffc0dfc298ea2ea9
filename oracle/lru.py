"""CPU oracle: least-recently-used residency of models under a byte budget.

TEST INFRASTRUCTURE ONLY (never imported by the product path).

Section 3 of the paper describes demand paging of whole models: a request
for a model that is not in device memory makes a replacement policy choose a
resident model to swap out, then the requested one is swapped in; Section 4
names the policy (LRU).  The paper caps the *number* of resident models
(Section 5); here the cap is a byte budget, which coincides with a count when
all models have the same size.

State machine (readings of points the paper leaves open):
  * "use" = dispatch of an inference or an explicit swap-in; each use stamps
    the model with a strictly increasing counter, so there are no ties;
  * eviction is lazy: victims are taken, least recently used first, only
    while `resident_bytes + bytes(m) > budget`;
  * a model larger than the budget is an error;
  * an explicit swap-out of any resident model is allowed and is no "use".

Parity status: fully pinned (budget invariant, equality with the textbook
stack-distance characterisation of LRU for equal sizes, brute-force replay).
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

# event = (kind, model, victims) with kind in {"hit", "miss", "out"}
Event = Tuple[str, int, Tuple[int, ...]]


class LruResidency:
    def __init__(self, budget: int, sizes: Sequence[int]):
        self.budget = int(budget)
        self.sizes = [int(s) for s in sizes]
        self.last_use: Dict[int, int] = {}     # resident model -> stamp
        self.clock = 0
        self.resident_bytes = 0
        self.peak_resident = 0
        self.events: List[Event] = []

    def is_resident(self, m: int) -> bool:
        return m in self.last_use

    def touch(self, m: int) -> Event:
        """A use of model `m` (inference dispatch or explicit swap-in)."""
        if not 0 <= m < len(self.sizes):
            raise KeyError(m)
        self.clock += 1
        if m in self.last_use:
            self.last_use[m] = self.clock
            ev: Event = ("hit", m, ())
            self.events.append(ev)
            return ev
        need = self.sizes[m]
        if need > self.budget:
            raise ValueError("model larger than the budget")
        victims = []
        while self.resident_bytes + need > self.budget:
            v = min(self.last_use, key=self.last_use.get)
            del self.last_use[v]
            self.resident_bytes -= self.sizes[v]
            victims.append(v)
        self.last_use[m] = self.clock
        self.resident_bytes += need
        self.peak_resident = max(self.peak_resident, self.resident_bytes)
        ev = ("miss", m, tuple(victims))
        self.events.append(ev)
        return ev

    def swap_out(self, m: int) -> Event:
        if m in self.last_use:
            del self.last_use[m]
            self.resident_bytes -= self.sizes[m]
            ev: Event = ("out", m, (m,))
        else:
            ev = ("out", m, ())
        self.events.append(ev)
        return ev


def replay(budget: int, sizes: Sequence[int], trace: Sequence[int]) -> List[Event]:
    r = LruResidency(budget, sizes)
    for m in trace:
        r.touch(int(m))
    return r.events
