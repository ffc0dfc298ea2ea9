"""CPU oracle: the engine's request scheduling, on a simulated clock.

TEST INFRASTRUCTURE ONLY (never imported by the product path).

Section 3.1 of the paper: every request is pushed, with a timestamp, into a
queue of its own model; the engine repeatedly picks a queue, pops its oldest
requests and submits them as one batch entry.  Section 4: requests are
scheduled in batches based on the oldest timestamp, and swapping follows LRU.
Section 5.2 fixes the maximum batch size per experiment (8 and 32).

Reading taken where the text leaves room:
  * the engine is serial on one GPU: it dispatches the next batch when the
    previous one has completed;
  * "based on the oldest timestamp": among the non-empty queues the one whose
    head request is oldest is served (ties: lower model index);
  * a batch takes the min(max_batch, queue length) oldest requests of that
    queue that have arrived by the dispatch time;
  * dispatching a batch is one "use" of the model for the LRU policy.

Time is simulated: the caller supplies `service(model, batch, miss)`, the
duration of one batch.  Everything else is deterministic bookkeeping, which is
what the library's scheduler is compared with.

Parity status: pinned by invariants (every request served exactly once, in
arrival order within its model, batches single-model and within the cap,
oldest-head-first at every dispatch, no dispatch before arrival) and by
brute-force enumeration on small cases (tests/test_oracle_engine.py).
"""
from __future__ import annotations

from typing import Callable, List, Sequence, Tuple

from .lru import LruResidency

# one dispatched batch: (dispatch_time, finish_time, model, request indices, was_miss)
Batch = Tuple[float, float, int, Tuple[int, ...], bool]


def simulate(arrival: Sequence[float], model_of: Sequence[int], n_models: int, max_batch: int,
             budget: int, sizes: Sequence[int],
             service: Callable[[int, int, bool], float]) -> Tuple[List[Batch], LruResidency]:
    """Runs the engine over a trace sorted by arrival time."""
    n = len(arrival)
    queues: List[List[int]] = [[] for _ in range(n_models)]
    lru = LruResidency(budget, sizes)
    batches: List[Batch] = []
    now = 0.0
    nxt = 0                      # next request of the trace not yet in a queue
    served = 0
    while served < n:
        while nxt < n and arrival[nxt] <= now:          # everything that has arrived is queued
            queues[model_of[nxt]].append(nxt)
            nxt += 1
        heads = [(arrival[q[0]], m) for m, q in enumerate(queues) if q]
        if not heads:
            now = arrival[nxt]                          # idle until the next arrival
            continue
        _, m = min(heads)
        take = tuple(queues[m][:max_batch])
        del queues[m][:len(take)]
        miss = lru.touch(m)[0] == "miss"
        finish = now + service(m, len(take), miss)
        batches.append((now, finish, m, take, miss))
        served += len(take)
        now = finish
    return batches, lru


def latencies(arrival: Sequence[float], batches: Sequence[Batch]) -> List[float]:
    out = [0.0] * len(arrival)
    for _, finish, _, reqs, _ in batches:
        for r in reqs:
            out[r] = finish - arrival[r]
    return out
