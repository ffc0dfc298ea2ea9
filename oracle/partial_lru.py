"""CPU oracle: LRU residency at the granularity of transfer blocks.

TEST INFRASTRUCTURE ONLY (never imported by the product path).

Section 3 of the paper swaps whole models; its closing section names smarter
load/offload decisions as the way to cut on-demand swaps.  This is the
block-granular refinement the library offers as an option: a model is a list
of transfer blocks in forward order (embeddings, then one block per decoder
layer), the part of a model that stays in device memory is always a *prefix*
of that list, and an eviction takes away only as many blocks as the incoming
model needs, from the tail of the least recently used model.  A later request
for the shortened model reloads just the missing tail while its forward pass
already runs on the prefix.

State machine (this oracle's definition; the paper has none for it):
  * `k[m]` = number of resident blocks of model m (a prefix), 0 <= k <= n_m;
  * a use of m with k[m] == n_m is a hit;
  * otherwise it is a miss: `need` = bytes of blocks k[m]..n_m-1; while
    `resident_bytes + need > budget`, the victim is the model with the
    smallest last-use stamp among those with k > 0 other than m, and its last
    resident block is dropped (k[v] -= 1); then m's missing blocks are loaded;
  * a model whose k reaches 0 leaves the recency order;
  * stamps as in the whole-model policy: a strictly increasing counter, set on
    every use; an explicit swap-out drops all blocks and is no use.

With one block per model this is exactly the whole-model policy.

Parity status: pinned by (tests/test_oracle_partial_lru.py) equality with the
whole-model oracle for single-block models, the budget and prefix invariants,
minimality of every eviction, the structural fact that at most one model is
partially resident and it is the least recently used one, dominance over the
whole-model policy (never fewer hits, never more bytes loaded), and an
independently written flat-priority-list simulation on small cases.
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

# (victim, first_block, end_block): blocks [first, end) of the victim leave device memory
Eviction = Tuple[int, int, int]
# (kind, model, first_loaded_block, evictions) with kind in {"hit", "miss", "out"};
# a miss loads blocks [first_loaded_block, n_m)
Event = Tuple[str, int, int, Tuple[Eviction, ...]]


class PartialLruResidency:
    def __init__(self, budget: int, block_bytes: Sequence[Sequence[int]]):
        self.budget = int(budget)
        self.blocks = [[int(b) for b in bs] for bs in block_bytes]
        self.k = [0] * len(self.blocks)
        self.last_use: Dict[int, int] = {}     # model with k > 0 -> stamp
        self.clock = 0
        self.resident_bytes = 0
        self.peak_resident = 0
        self.bytes_loaded = 0
        self.events: List[Event] = []

    def n_blocks(self, m: int) -> int:
        return len(self.blocks[m])

    def is_resident(self, m: int) -> bool:
        return self.k[m] == self.n_blocks(m)

    def touch(self, m: int) -> Event:
        if not 0 <= m < len(self.blocks):
            raise KeyError(m)
        self.clock += 1
        n = self.n_blocks(m)
        if self.k[m] == n:
            self.last_use[m] = self.clock
            ev: Event = ("hit", m, n, ())
            self.events.append(ev)
            return ev
        if sum(self.blocks[m]) > self.budget:
            raise ValueError("model larger than the budget")
        first = self.k[m]
        need = sum(self.blocks[m][first:])
        dropped: Dict[int, List[int]] = {}     # victim -> [new k, old k], insertion order = eviction order
        while self.resident_bytes + need > self.budget:
            candidates = {v: s for v, s in self.last_use.items() if v != m}
            v = min(candidates, key=candidates.get)
            self.k[v] -= 1
            self.resident_bytes -= self.blocks[v][self.k[v]]
            if v in dropped:
                dropped[v][0] = self.k[v]
            else:
                dropped[v] = [self.k[v], self.k[v] + 1]
            if self.k[v] == 0:
                del self.last_use[v]
        self.k[m] = n
        self.last_use[m] = self.clock
        self.resident_bytes += need
        self.bytes_loaded += need
        self.peak_resident = max(self.peak_resident, self.resident_bytes)
        ev = ("miss", m, first, tuple((v, lo, hi) for v, (lo, hi) in dropped.items()))
        self.events.append(ev)
        return ev

    def swap_out(self, m: int) -> Event:
        if self.k[m] > 0:
            ev: Event = ("out", m, 0, ((m, 0, self.k[m]),))
            self.resident_bytes -= sum(self.blocks[m][:self.k[m]])
            self.k[m] = 0
            del self.last_use[m]
        else:
            ev = ("out", m, 0, ())
        self.events.append(ev)
        return ev


def replay(budget: int, block_bytes: Sequence[Sequence[int]], trace: Sequence[int]) -> List[Event]:
    r = PartialLruResidency(budget, block_bytes)
    for m in trace:
        r.touch(int(m))
    return r.events
