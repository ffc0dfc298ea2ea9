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

`simulate_async` is the engine of Section 3.2 proper: load entries are
asynchronous, so a batch of one model need not wait for the load of another.
On one GPU this becomes two
lanes that run side by side:
  * the hit lane executes batches of models that are completely loaded, one
    batch at a time;
  * the load lane takes one miss at a time: the swap-in of the model followed
    by that model's batch (a batch is only evaluated on loaded parameters);
  * a model whose miss is in flight on the load lane is not dispatched again
    until that batch has completed;
  * at every decision time the non-empty queues are scanned oldest head first
    (ties: lower model index) and the first one that can be dispatched (its
    lane is free, its model is not loading) is; the scan repeats until nothing
    more can be dispatched; the clock then moves to the next arrival or
    completion.

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


# one dispatched batch of the two-lane engine: (dispatch, finish, model, requests, was_miss, lane)
AsyncBatch = Tuple[float, float, int, Tuple[int, ...], bool, int]
HIT_LANE, LOAD_LANE = 0, 1


def simulate_async(arrival: Sequence[float], model_of: Sequence[int], n_models: int, max_batch: int,
                   budget: int, sizes: Sequence[int],
                   service: Callable[[int, int, bool], float]) -> Tuple[List[AsyncBatch], LruResidency]:
    """The two-lane engine over a trace sorted by arrival time (see the module text)."""
    n = len(arrival)
    queues: List[List[int]] = [[] for _ in range(n_models)]
    lru = LruResidency(budget, sizes)
    batches: List[AsyncBatch] = []
    lane_free = [0.0, 0.0]
    loading = {}                 # model -> time its batch on the load lane completes
    now, nxt, dispatched = 0.0, 0, 0
    while dispatched < n:
        while nxt < n and arrival[nxt] <= now:
            queues[model_of[nxt]].append(nxt)
            nxt += 1
        for m in [m for m, t in loading.items() if t <= now]:
            del loading[m]
        progress = True
        while progress:
            progress = False
            for _, m in sorted((arrival[q[0]], m) for m, q in enumerate(queues) if q):
                if m in loading:
                    continue
                hit = lru.is_resident(m)
                lane = HIT_LANE if hit else LOAD_LANE
                if lane_free[lane] > now:
                    continue
                take = tuple(queues[m][:max_batch])
                del queues[m][:len(take)]
                lru.touch(m)
                finish = now + service(m, len(take), not hit)
                lane_free[lane] = finish
                if not hit:
                    loading[m] = finish
                batches.append((now, finish, m, take, not hit, lane))
                dispatched += len(take)
                progress = True
                break
        if dispatched == n:
            break
        ahead = [t for t in lane_free if t > now]
        if nxt < n:
            ahead.append(arrival[nxt])
        now = min(ahead)
    return batches, lru


def latencies(arrival: Sequence[float], batches: Sequence[Batch]) -> List[float]:
    out = [0.0] * len(arrival)
    for _, finish, _, reqs, _ in batches:
        for r in reqs:
            out[r] = finish - arrival[r]
    return out
