"""Serial oldest-request-first serving loop over a swapping context.

Section 3.1 / 4 of the paper: the engine keeps one queue per model, always serves the oldest
pending request and swaps models on demand with LRU replacement.  With a maximum batch size of
one and one GPU this is a single FIFO over the merged arrival stream; the loop below replays an
arrival trace in real time (open loop: latency includes queueing behind earlier requests) and
calls `ctn_infer` for each request.  All swapping decisions are taken inside the library.
"""
from __future__ import annotations

import time
from typing import Callable, Sequence

import numpy as np


def serve_trace(ctx, models: Sequence[int], arrival_s: np.ndarray, model_of: np.ndarray,
                ids_of: Callable[[int], np.ndarray], out, time_scale: float = 1.0,
                progress: Callable[[int], None] = None, missing_blocks: list = None):
    """Replays the trace; returns (latency_s, service_s, was_miss) arrays.  `missing_blocks`, if
    given, receives per request the number of transfer blocks that had to be loaded.

    `out` is a device tensor receiving the logits of each request (overwritten every time);
    a request is complete when its logits are complete on the compute stream.
    """
    n = len(arrival_s)
    lat = np.zeros(n)
    svc = np.zeros(n)
    miss = np.zeros(n, dtype=bool)
    arr = np.asarray(arrival_s, dtype=np.float64) * time_scale
    t0 = time.perf_counter()
    for i in range(n):
        now = time.perf_counter() - t0
        if now < arr[i]:
            time.sleep(arr[i] - now)
        m = models[int(model_of[i])]
        start = time.perf_counter() - t0
        miss[i] = not ctx.is_resident(m)
        if missing_blocks is not None:
            k, nb = ctx.resident_blocks(m)
            missing_blocks.append(nb - k)
        ctx.infer(m, ids_of(i), out=out)
        ctx.stream_compute.synchronize()
        end = time.perf_counter() - t0
        lat[i] = end - arr[i]
        svc[i] = end - start
        if progress is not None:
            progress(i)
    return lat, svc, miss


def serve_engine(ctx, engine, models: Sequence[int], arrival_s: np.ndarray, model_of: np.ndarray,
                 ids_of: Callable[[int], np.ndarray], out, on_batch: Callable = None):
    """Real-time replay through the library's engine (per-model queues, oldest-first batches of at
    most `engine.max_batch`, Sections 3.1 / 4 / 5.2).  Requests are submitted when their arrival
    time has passed; the loop dispatches one batch at a time and waits for its logits.
    Returns (latency_s per request, list of (n_requests, model, was_miss, service_s) per batch)."""
    n = len(arrival_s)
    lat = np.zeros(n)
    batches = []
    nxt = done = 0
    base = None                      # the engine's id of trace request 0 (earlier submissions shift it)
    t0 = time.perf_counter()
    while done < n:
        now = time.perf_counter() - t0
        while nxt < n and arrival_s[nxt] <= now:
            rid = engine.submit(models[int(model_of[nxt])], ids_of(nxt), float(arrival_s[nxt]))
            if base is None:
                base = rid
            assert rid - base == nxt
            nxt += 1
        start = time.perf_counter() - t0
        r = engine.step(out)
        if r is None:
            engine.idle()            # nothing queued: the engine may load the predicted next model ahead
            pause = arrival_s[nxt] - (time.perf_counter() - t0)
            if pause > 0:
                time.sleep(pause)
            continue
        ctx.stream_compute.synchronize()
        end = time.perf_counter() - t0
        served, m, miss = r
        served = [rid - base for rid in served]
        for rid in served:
            lat[rid] = end - arrival_s[rid]
        done += len(served)
        batches.append((len(served), m, miss, end - start))
        if on_batch is not None:
            on_batch(served, m, miss)
    return lat, batches


def serve_engine_async(ctx, engine, models: Sequence[int], arrival_s: np.ndarray, model_of: np.ndarray,
                       ids_of: Callable[[int], np.ndarray], out_hit, out_load, on_batch: Callable = None):
    """Real-time replay through the two-lane engine (Section 3.2: batches of loaded models go on
    while another model loads).  The loop submits requests as they arrive, dispatches whatever can
    go, and notes a batch's completion when its lane reports idle.
    Returns (latency_s per request, list of (n_requests, model, was_miss, service_s, lane) per batch).
    `on_batch(request indices, model, was_miss, lane, logits_intact)` is called at every completion."""
    n = len(arrival_s)
    lat = np.zeros(n)
    batches = []
    nxt = done = 0
    base = None
    flying = [None, None]            # per lane: (request indices, model, miss, start time)
    t0 = time.perf_counter()

    def finished(lane, intact=True):
        """The batch that was in flight on `lane` has completed; `intact`: its logits are still in
        the lane's buffer (no newer batch has been dispatched there)."""
        nonlocal done
        end = time.perf_counter() - t0
        served, m, miss, start = flying[lane]
        flying[lane] = None
        for rid in served:
            lat[rid] = end - arrival_s[rid]
        done += len(served)
        batches.append((len(served), m, miss, end - start, lane))
        if on_batch is not None:
            on_batch(served, m, miss, lane, intact)

    while done < n:
        now = time.perf_counter() - t0
        while nxt < n and arrival_s[nxt] <= now:
            rid = engine.submit(models[int(model_of[nxt])], ids_of(nxt), float(arrival_s[nxt]))
            if base is None:
                base = rid
            assert rid - base == nxt
            nxt += 1
        if flying[0] is not None or flying[1] is not None:
            busy = engine.lanes_busy()
            ready = [lane for lane in (0, 1) if flying[lane] is not None and not busy[lane]]
            for lane in sorted(ready, key=lambda l: flying[l][3]):     # noticed together: report in dispatch order
                finished(lane)
        if done == n:
            break
        start = time.perf_counter() - t0
        r = engine.dispatch(out_hit, out_load)
        if r is not None:
            served, m, miss, lane = r
            if flying[lane] is not None:     # the engine saw that lane's batch complete just now and reused the lane
                finished(lane, intact=False)
            flying[lane] = ([rid - base for rid in served], m, miss, start)
            continue
        if flying[0] is None and flying[1] is None and nxt < n:
            engine.idle()
            pause = arrival_s[nxt] - (time.perf_counter() - t0)
            if pause > 0:
                time.sleep(min(pause, 0.002))
    return lat, batches
