"""`bench.py --workload serve`: multi-model serving on one GPU under an HBM budget.

8 distinct shards of the opt6.7b TP=2 shape (6.67 GB each) in pinned host memory, budget
20,000,000,000 B so at most two are resident; 2000 requests (batch 1 x seq 64) from independent
Gamma arrival processes (CV 4) with Zipf(1.5) popularity, 20 requests/s in total (Section 5.2 of
the paper, sized for one rank); serial oldest-first engine, LRU swapping.
"""
from __future__ import annotations

import json
import sys
import time

import numpy as np


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def serve_setup(host_layout="separate"):
    """The eight shards of the serving workload in pinned host memory: (config, pool, tensor lists)."""
    import paper_2306_13835_amd as P
    from synth import CONFIGS, fill_shard, shard_bytes, param_list
    c = CONFIGS["serve8x6.7b_tp2"]
    desc, n_models = c["desc"], c["n_models"]
    nbytes = shard_bytes(desc)
    gap = 4096 if host_layout == "separate" else 0
    n_t = len(param_list(desc))
    pool = P.HostPool(n_models * (nbytes + n_t * (256 + gap)) + 8192)
    t0 = time.time()
    keep = [fill_shard(desc, c["wseed"] + k, alloc=lambda s: pool.take(s, gap=gap), threads=16) for k in range(n_models)]
    log(f"[serve] {n_models} shards ({n_models * nbytes / 1e9:.1f} GB pinned) ready in {time.time() - t0:.1f}s")
    return c, pool, keep


def run_serve(args):
    import torch
    torch.cuda.set_device(0)
    torch.zeros(1, device="cuda")
    c, pool, keep = serve_setup(args.host_layout)
    res = serve_once(c, keep, args.requests or c["n_requests"], args.transfer, args.host_layout,
                     blocks=bool(getattr(args, "block_residency", False)), two_lanes=bool(getattr(args, "two_lane", False)),
                     load_ahead=bool(getattr(args, "load_ahead", False)))
    del keep
    pool.close()
    print(json.dumps(res), flush=True)


TRANSFER_MODES = {"dma": 0, "kernel": 1, "auto": 2, "dma_in_kernel_out": 3, "kernel_in_dma_out": 4, "dma_runs": 5}


def serve_once(c, keep, n_req, transfer="auto", host_layout="separate", blocks=False, two_lanes=False, load_ahead=False):
    """One real-time replay of the first n_req requests of the serving trace over the registered shards;
    returns the result record (latency percentiles, misses, whether every decision equals the policy replay)."""
    import torch
    import paper_2306_13835_amd as P
    from paper_2306_13835_amd.serving import serve_trace
    from synth import token_ids, shard_bytes, param_list, gamma_zipf_trace

    desc, batch, seq, n_models = c["desc"], c["batch"], c["seq"], c["n_models"]
    nbytes = shard_bytes(desc)
    budget = c["budget"]
    # The budget caps the bytes of models *marked resident* (at most two here).  The arena holds one
    # more range so that a victim can still be streaming out of its range while the requested model
    # streams into another one, as the paper's overlapped offload and load do (Sections 3.2, 5.1).
    resident_max = budget // nbytes
    # Block residency: every transfer block takes one slot; the slack of the budget below another whole
    # model holds a prefix of one more model, so the arena gets one more range than the whole-model case.
    one = P.slot_bytes(desc) * (desc.layers + 1) if blocks else P.arena_bytes(desc)
    arena = torch.empty((resident_max + (2 if blocks else 1)) * one, dtype=torch.uint8, device="cuda")
    ws = torch.empty(P.workspace_bytes(desc, batch * seq) * (2 if two_lanes else 1) + 512, dtype=torch.uint8, device="cuda")
    logits = torch.empty(batch, seq, desc.vocab // desc.tp, dtype=torch.float32, device="cuda")
    logits2 = torch.empty_like(logits)
    ctx = P.Context(budget, arena, ws, transfer_mode=TRANSFER_MODES[transfer], pipeline=True, block_residency=blocks)
    models = [ctx.register_model(desc, t) for t in keep]
    arr, mod = gamma_zipf_trace(n_models, c["rate"], c["cv"], c["zipf"], c["n_requests"], c["trace_seed"])
    arr, mod = arr[:n_req], mod[:n_req]
    ids = [token_ids(c["idseed"] + i, batch, seq, desc.vocab) for i in range(n_req)]
    # warm-up requests that are not recorded (Section 5.2): one hit-path and one miss-path inference
    for k in (0, 1, 0):
        ctx.infer(models[k], ids[0], out=logits)
    ctx.sync()
    for m in models:
        ctx.swap_out(m)
    ctx.sync()
    ev0 = len(ctx.events())
    bev0 = len(ctx.block_events())
    st0 = ctx.stats()
    last = [time.time()]

    def progress(i):
        if time.time() - last[0] > 20:
            last[0] = time.time()
            log(f"[serve] request {i + 1}/{n_req}")

    t0 = time.perf_counter()
    missing = []
    if two_lanes:
        # the asynchronous engine of Section 3.2 (batch size 1 as in this workload): hits go on while a model loads
        from paper_2306_13835_amd.serving import serve_engine_async
        eng = P.Engine(ctx, batch, seq, two_lanes=True)
        if load_ahead:
            eng.set_prefetch(True, min_count=3, min_share_percent=60)
        miss = np.zeros(n_req, dtype=bool)
        count = [0]

        def on_batch(served, m, was_miss, lane, intact):
            miss[served] = was_miss
            count[0] += len(served)
            progress(count[0] - 1)
        lat, batches = serve_engine_async(ctx, eng, models, arr, mod, lambda i: ids[i], logits, logits2, on_batch)
        eng.close()
        # time from dispatch to completion of each request's batch (requests are batches of one here)
        svc_hit = np.array([b[3] for b in batches if not b[2]])
        svc_miss = np.array([b[3] for b in batches if b[2]])
        svc = np.zeros(n_req)
        svc[~miss] = np.resize(svc_hit, int((~miss).sum())) if svc_hit.size else 0.0
        svc[miss] = np.resize(svc_miss, int(miss.sum())) if svc_miss.size else 0.0
        missing = np.where(miss, desc.layers + 1, 0)
    else:
        lat, svc, miss = serve_trace(ctx, models, arr, mod, lambda i: ids[i], logits, progress=progress,
                                     missing_blocks=missing)
        missing = np.asarray(missing)
    whole_miss = missing == desc.layers + 1
    part_miss = (missing > 0) & ~whole_miss
    wall = time.perf_counter() - t0
    ctx.sync()
    st = ctx.stats()
    events = ctx.events()[ev0:]
    # the decisions taken on the GPU path must be the ones the policy takes on the bare trace
    if two_lanes:
        # requests overtake one another, so the policy is replayed on the order of dispatch
        order = [e[1] for e in events]
        if blocks:
            n = [2 * int(np.prod(shape)) for _, shape, _ in param_list(desc)]
            bb = [n[0] + n[1] + n[-2] + n[-1]] + [sum(n[2 + 16 * l:18 + 16 * l]) for l in range(desc.layers)]
            replay = P.block_residency_replay(budget, [bb] * n_models, order)[0]
        else:
            replay = P.residency_replay(budget, [nbytes] * n_models, order)
        decisions_match = [(e[0], e[1], e[2]) for e in events] == replay
    elif blocks:
        n = [2 * int(np.prod(shape)) for _, shape, _ in param_list(desc)]
        bb = [n[0] + n[1] + n[-2] + n[-1]] + [sum(n[2 + 16 * l:18 + 16 * l]) for l in range(desc.layers)]
        replay, block_replay = P.block_residency_replay(budget, [bb] * n_models, [int(x) for x in mod])
        got_blocks = [(k, m, lo, hi, use - ev0) for k, m, lo, hi, use in ctx.block_events()[bev0:]]
        decisions_match = [(e[0], e[1], e[2]) for e in events] == replay and got_blocks == block_replay
    else:
        replay = P.residency_replay(budget, [nbytes] * n_models, [int(x) for x in mod])
        decisions_match = [(e[0], e[1], e[2]) for e in events] == replay
    n_miss = st["n_miss"] - st0["n_miss"]
    res = {
        "metric": "p99 request latency under swap (8 models, budget 20e9 B, Gamma CV=4 / Zipf 1.5 arrivals)",
        "value": round(float(np.percentile(lat, 99)), 4), "unit": "s", "n_gpus": 1, "steps": n_req, "warmup": 3,
        "ms_per_step": round(wall / n_req * 1e3, 3), "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"serve8x6.7b_tp2: {n_models} shards x {nbytes} B, budget {budget} B, {n_req} requests "
                               f"batch {batch} x seq {seq}, "
                               + ("two-lane engine (hits go on while a model loads)" if two_lanes else "serial oldest-first engine")
                               + ", LRU",
                   "transfer": transfer, "host_layout": host_layout,
                   "residency": "per transfer block (prefix kept)" if blocks else "whole models (2 resident)",
                   "load_ahead": bool(load_ahead),
                   "arena_bytes": int(arena.numel()), "arena_note": "budget + one transit range"},
        "latency_s": {"mean": round(float(lat.mean()), 4), "p50": round(float(np.percentile(lat, 50)), 4),
                      "p90": round(float(np.percentile(lat, 90)), 4), "p99": round(float(np.percentile(lat, 99)), 4),
                      "max": round(float(lat.max()), 4)},
        "service_ms": {"hit_p50": round(float(np.median(svc[~miss]) * 1e3), 3) if (~miss).any() else None,
                       "miss_p50": round(float(np.median(svc[miss]) * 1e3), 3) if miss.any() else None,
                       "miss_max": round(float(svc[miss].max() * 1e3), 3) if miss.any() else None,
                       "whole_miss_p50": round(float(np.median(svc[whole_miss]) * 1e3), 3) if whole_miss.any() else None,
                       "partial_miss_p50": round(float(np.median(svc[part_miss]) * 1e3), 3) if part_miss.any() else None,
                       "partial_miss_blocks_p50": float(np.median(missing[part_miss])) if part_miss.any() else None},
        "misses": int(n_miss), "hit_ratio": round(1 - n_miss / n_req, 4),
        "partial_misses": st["n_partial_miss"] - st0["n_partial_miss"],
        "loads_ahead": st["n_prefetch"] - st0["n_prefetch"],
        "extra_evictions": st["n_extra_evictions"] - st0["n_extra_evictions"],
        "bytes_swapped_in": st["bytes_h2d"] - st0["bytes_h2d"], "trace_seconds": round(float(arr[-1]), 2),
        "wall_seconds": round(wall, 2), "peak_resident_bytes": st["peak_resident_bytes"],
        "decisions_equal_policy_replay": bool(decisions_match),
        "hit_tokens_per_s": round(batch * seq / float(np.median(svc[~miss])), 1) if (~miss).any() else None,
    }
    ctx.close()
    del arena, ws
    return res


# Average end-to-end latencies the paper prints (Tables 1 and 2; 4 x A100, OPT-13B, TP=2 x PP=2,
# unit not printed, seconds by context).  Context only: another machine, the whole model.
PAPER_TABLES = {
    "3 models / 2 resident, max batch 8": {"(1, 1, 1)": (1.262, 0.606, 0.518), "(10, 1, 1)": (1.172, 0.886, 0.550),
                                           "(10, 10, 1)": (1.014, 0.716, 0.374)},
    "6 models / 4 resident, max batch 32": {"(1, 1, 1, 1, 1, 1)": (1.847, 1.282, 0.174),
                                            "(10, 10, 1, 1, 1, 1)": (2.017, 1.413, 0.229),
                                            "(10, 10, 10, 10, 1, 1)": (1.535, 1.470, 0.312)},
}
GRIDS = [
    ("3 models / 2 resident, max batch 8", 3, 2, 8, [(1, 1, 1), (10, 1, 1), (10, 10, 1)]),
    ("6 models / 4 resident, max batch 32", 6, 4, 32, [(1,) * 6, (10, 10, 1, 1, 1, 1), (10, 10, 10, 10, 1, 1)]),
]
CVS = (0.25, 1.0, 4.0)


def run_grid(args):
    """The paper's simulated workloads (Section 5.2) on one worker's shard: Gamma arrivals per model
    over `--duration` seconds, 8 input tokens per request, oldest-first batching, LRU swapping."""
    import torch
    import paper_2306_13835_amd as P
    from paper_2306_13835_amd.serving import serve_engine
    from synth import CONFIGS, fill_shard, token_ids, shard_bytes, param_list
    from synth.arrivals import gamma_rates_trace

    torch.cuda.set_device(0)
    torch.zeros(1, device="cuda")
    desc = CONFIGS["opt13b_tp4"]["desc"]          # one GPU's quarter of OPT-13B, as in the paper's 4-GPU runs
    seq, nbytes = 8, shard_bytes(desc)
    gap = 4096 if args.host_layout == "separate" else 0
    n_t = len(param_list(desc))
    max_models = max(g[1] for g in GRIDS)
    pool = P.HostPool(max_models * (nbytes + n_t * (256 + gap)) + 8192)
    t0 = time.time()
    keep = [fill_shard(desc, 60 + k, alloc=lambda s: pool.take(s, gap=gap), threads=16) for k in range(max_models)]
    log(f"[grid] {max_models} shards ({max_models * nbytes / 1e9:.1f} GB pinned) ready in {time.time() - t0:.1f}s")
    results = {}
    for name, n_models, resident, max_batch, skews in GRIDS:
        budget = resident * nbytes
        arena = torch.empty((resident + 1) * P.arena_bytes(desc), dtype=torch.uint8, device="cuda")
        two_lanes = bool(getattr(args, "two_lane", False))
        ws = torch.empty(P.workspace_bytes(desc, max_batch * seq) * (2 if two_lanes else 1) + 512, dtype=torch.uint8,
                         device="cuda")
        logits = torch.empty(max_batch, seq, desc.vocab // desc.tp, dtype=torch.float32, device="cuda")
        logits2 = torch.empty_like(logits)
        ctx = P.Context(budget, arena, ws, transfer_mode=TRANSFER_MODES[args.transfer], pipeline=True)
        models = [ctx.register_model(desc, keep[k]) for k in range(n_models)]
        eng = P.Engine(ctx, max_batch, seq, two_lanes=two_lanes)
        table = {}
        for skew in skews:
            row = []
            for cv in CVS:
                arr, mod = gamma_rates_trace(skew, cv, args.duration, seed=700 + int(cv * 100))
                ids = [token_ids(2000 + i, 1, seq, desc.vocab) for i in range(len(arr))]
                for k in range(min(resident, n_models)):       # warm-up requests, not recorded (Section 5.2)
                    eng.submit(models[k], ids[0], 0.0)
                    if two_lanes:
                        eng.dispatch(logits, logits2)
                        ctx.sync()
                    else:
                        eng.step(logits)
                ctx.sync()
                st0 = ctx.stats()
                if two_lanes:
                    from paper_2306_13835_amd.serving import serve_engine_async
                    lat, batches = serve_engine_async(ctx, eng, models, arr, mod, lambda i: ids[i], logits, logits2)
                else:
                    lat, batches = serve_engine(ctx, eng, models, arr, mod, lambda i: ids[i], logits)
                ctx.sync()
                st = ctx.stats()
                row.append({"cv": cv, "requests": len(arr), "mean_s": round(float(lat.mean()), 4),
                            "p50_s": round(float(np.percentile(lat, 50)), 4), "p99_s": round(float(np.percentile(lat, 99)), 4),
                            "swaps": st["n_miss"] - st0["n_miss"], "batches": len(batches),
                            "mean_batch": round(float(np.mean([b[0] for b in batches])), 2)})
                log(f"[grid] {name} rates {skew} CV {cv}: mean {row[-1]['mean_s']} s, p99 {row[-1]['p99_s']} s, "
                    f"{row[-1]['swaps']} swaps / {len(arr)} requests")
            table[str(tuple(skew))] = row
        results[name] = table
        eng.close()
        ctx.close()
        del arena, ws, logits
    out = {"metric": "average end-to-end request latency per (rates, CV), the paper's Section 5.2 grids on one worker's shard",
           "unit": "s", "n_gpus": 1, "higher_is_better": False, "data": "synthetic", "dtype": "f16",
           "config": {"workload": f"opt13b_tp4 shard ({nbytes} B) x 3 and x 6 models, {args.duration:.0f} s Gamma arrivals, "
                                  f"{seq} tokens per request, oldest-first batching, LRU, "
                                  + ("two-lane engine" if getattr(args, "two_lane", False) else "serial engine"),
                      "transfer": args.transfer,
                      "host_layout": args.host_layout},
           "results": results, "paper_tables_context": PAPER_TABLES}
    del keep
    pool.close()
    print(json.dumps(out), flush=True)


def run_cyclic(args):
    """Models requested in a fixed order (a structured stream, the paper's closing section): three
    shards, room for two, one request every 0.25 s.  Whole-model LRU misses on every request; the
    engine's load-ahead predictor hides the swap behind the idle time between requests."""
    import torch
    import paper_2306_13835_amd as P
    from paper_2306_13835_amd.serving import serve_engine
    from synth import CONFIGS, fill_shard, token_ids, shard_bytes, param_list, cyclic_trace

    torch.cuda.set_device(0)
    torch.zeros(1, device="cuda")
    desc = CONFIGS["opt6.7b_tp2"]["desc"]
    seq, nbytes, n_models, period = 8, shard_bytes(desc), 3, 0.25
    n_req = args.requests or 60
    gap = 4096 if args.host_layout == "separate" else 0
    n_t = len(param_list(desc))
    pool = P.HostPool(n_models * (nbytes + n_t * (256 + gap)) + 8192)
    keep = [fill_shard(desc, 90 + k, alloc=lambda s: pool.take(s, gap=gap), threads=16) for k in range(n_models)]
    arr, mod = cyclic_trace(n_models, period, n_req, jitter=0.2, seed=900)
    ids = [token_ids(3000 + i, 1, seq, desc.vocab) for i in range(n_req)]
    out = {}
    for label, ahead in (("lru_only", False), ("load_ahead", True)):
        arena = torch.empty(3 * P.arena_bytes(desc), dtype=torch.uint8, device="cuda")
        ws = torch.empty(P.workspace_bytes(desc, seq), dtype=torch.uint8, device="cuda")
        logits = torch.empty(1, seq, desc.vocab // desc.tp, dtype=torch.float32, device="cuda")
        ctx = P.Context(2 * nbytes, arena, ws, transfer_mode=TRANSFER_MODES[args.transfer], pipeline=True)
        models = [ctx.register_model(desc, keep[k]) for k in range(n_models)]
        eng = P.Engine(ctx, 1, seq)
        eng.set_prefetch(ahead)
        lat, batches = serve_engine(ctx, eng, models, arr, mod, lambda i: ids[i], logits)
        ctx.sync()
        st = ctx.stats()
        steady = lat[3 * n_models:]                       # after the predictor has seen the cycle twice
        out[label] = {"mean_s": round(float(lat.mean()), 4), "steady_mean_s": round(float(steady.mean()), 4),
                      "steady_p99_s": round(float(np.percentile(steady, 99)), 4),
                      "misses_at_dispatch": int(sum(b[2] for b in batches)), "loads_ahead": st["n_prefetch"],
                      "bytes_swapped_in": st["bytes_h2d"]}
        log(f"[cyclic] {label}: {out[label]}")
        eng.close()
        ctx.close()
        del arena, ws, logits
    res = {"metric": "request latency on a cyclic stream (3 models in fixed order, 2 resident), LRU alone vs loading ahead",
           "value": out["load_ahead"]["steady_mean_s"], "unit": "s", "n_gpus": 1, "steps": n_req, "warmup": 0,
           "higher_is_better": False, "data": "synthetic", "dtype": "f16", "vs_baseline": None,
           "config": {"workload": f"3 x opt6.7b_tp2 shard ({nbytes} B), budget 2 shards, one request of {seq} tokens "
                                  f"every {period} s in the order 0,1,2,0,...", "transfer": args.transfer,
                      "host_layout": args.host_layout},
           "results": out}
    del keep
    pool.close()
    print(json.dumps(res), flush=True)


def run_mixed(args):
    """Shards of two sizes under one byte budget (the paper's closing section names heterogeneous model
    sizes as open; its own runs use one size): three opt6.7b/TP2 shards and five opt1.3b shards, 20e9 B,
    the serving trace's arrival process.  The residency decisions must be those of the byte-budget LRU
    policy on the same trace; evictions forced by arena fragmentation (none of the policy's) are counted."""
    import torch
    import paper_2306_13835_amd as P
    from paper_2306_13835_amd.serving import serve_trace
    from synth import CONFIGS, fill_shard, token_ids, shard_bytes, param_list, gamma_zipf_trace

    torch.cuda.set_device(0)
    torch.zeros(1, device="cuda")
    big, small = CONFIGS["opt6.7b_tp2"]["desc"], CONFIGS["opt1.3b_tp1"]["desc"]
    c = CONFIGS["serve8x6.7b_tp2"]
    kinds = [big, small, small, big, small, small, big, small]      # by popularity rank: sizes interleaved
    n_models, batch, seq, budget = len(kinds), 1, 64, c["budget"]
    n_req = args.requests or 1000
    sizes = [shard_bytes(d) for d in kinds]
    gap = 4096 if args.host_layout == "separate" else 0
    pool = P.HostPool(sum(sz + len(param_list(d)) * (256 + gap) for sz, d in zip(sizes, kinds)) + 8192)
    # room for the budget's worth of shards plus one large shard in transit
    arena = torch.empty(4 * P.arena_bytes(big), dtype=torch.uint8, device="cuda")
    ws = torch.empty(max(P.workspace_bytes(d, batch * seq) for d in (big, small)) + 512, dtype=torch.uint8, device="cuda")
    logits = torch.empty(batch * seq * max(d.vocab // d.tp for d in (big, small)), dtype=torch.float32, device="cuda")
    ctx = P.Context(budget, arena, ws, transfer_mode=TRANSFER_MODES[args.transfer], pipeline=True)
    t0 = time.time()
    keep = [fill_shard(d, 70 + k, alloc=lambda sh: pool.take(sh, gap=gap), threads=16) for k, d in enumerate(kinds)]
    models = [ctx.register_model(d, t) for d, t in zip(kinds, keep)]
    log(f"[mixed] {n_models} shards ({sum(sizes) / 1e9:.1f} GB pinned) ready in {time.time() - t0:.1f}s")
    arr, mod = gamma_zipf_trace(n_models, c["rate"], c["cv"], c["zipf"], n_req, 510)
    ids = [token_ids(4000 + i, batch, seq, big.vocab) for i in range(n_req)]
    for k in (0, 1, 0, 1):                     # unrecorded warm-up: a hit and a miss of each size
        ctx.infer(models[k], ids[0], out=logits)
    ctx.sync()
    for m in models:
        ctx.swap_out(m)
    ctx.sync()
    ev0, st0 = len(ctx.events()), ctx.stats()
    last = [time.time()]

    def progress(i):
        if time.time() - last[0] > 20:
            last[0] = time.time()
            log(f"[mixed] request {i + 1}/{n_req}")

    t0 = time.perf_counter()
    lat, svc, miss = serve_trace(ctx, models, arr, mod, lambda i: ids[i], logits, progress=progress)
    wall = time.perf_counter() - t0
    ctx.sync()
    st = ctx.stats()
    events = [(e[0], e[1], e[2]) for e in ctx.events()[ev0:]]
    replay = P.residency_replay(budget, sizes, [int(x) for x in mod])
    extra = st["n_extra_evictions"] - st0["n_extra_evictions"]
    is_big = np.array([kinds[int(m)] is big for m in mod])

    def cls(sel, nbytes):
        hit, ms = sel & ~miss, sel & miss
        hit_ms = float(np.median(svc[hit]) * 1e3) if hit.any() else None
        miss_ms = float(np.median(svc[ms]) * 1e3) if ms.any() else None
        return {"requests": int(sel.sum()), "misses": int(ms.sum()),
                "mean_latency_s": round(float(lat[sel].mean()), 4), "p99_latency_s": round(float(np.percentile(lat[sel], 99)), 4),
                "hit_ms_p50": round(hit_ms, 3) if hit_ms is not None else None,
                "miss_ms_p50": round(miss_ms, 3) if miss_ms is not None else None,
                "miss_gbps_p50": round(nbytes / miss_ms / 1e6, 2) if miss_ms else None}

    n_miss = st["n_miss"] - st0["n_miss"]
    res = {"metric": "p99 request latency under swap, shards of two sizes under one byte budget",
           "value": round(float(np.percentile(lat, 99)), 4), "unit": "s", "n_gpus": 1, "steps": n_req, "warmup": 4,
           "ms_per_step": round(wall / n_req * 1e3, 3), "higher_is_better": False, "scaling": "weak",
           "vs_baseline": None, "dtype": "f16", "data": "synthetic",
           "config": {"workload": f"3 x opt6.7b_tp2 ({sizes[0]} B) + 5 x opt1.3b ({sizes[1]} B) shards, budget {budget} B, "
                                  f"{n_req} requests batch {batch} x seq {seq}, Gamma CV=4 / Zipf 1.5 arrivals, "
                                  "serial oldest-first engine, whole-model LRU by bytes",
                      "sizes_by_popularity": ["6.7b/2" if d is big else "1.3b" for d in kinds],
                      "transfer": args.transfer, "host_layout": args.host_layout, "arena_bytes": int(arena.numel())},
           "latency_s": {"mean": round(float(lat.mean()), 4), "p50": round(float(np.percentile(lat, 50)), 4),
                         "p99": round(float(np.percentile(lat, 99)), 4), "max": round(float(lat.max()), 4)},
           "large": cls(is_big, sizes[0]), "small": cls(~is_big, sizes[1]),
           "misses": int(n_miss), "hit_ratio": round(1 - n_miss / n_req, 4),
           "bytes_swapped_in": st["bytes_h2d"] - st0["bytes_h2d"],
           "peak_resident_bytes": st["peak_resident_bytes"], "extra_evictions_for_arena_room": int(extra),
           "decisions_equal_policy_replay": bool(events == replay),
           "hits_and_misses_equal_policy_replay": bool([e[:2] for e in events] == [e[:2] for e in replay]),
           "trace_seconds": round(float(arr[-1]), 2), "wall_seconds": round(wall, 2)}
    ctx.close()
    del keep
    pool.close()
    print(json.dumps(res), flush=True)


SPLITS = [(1, 1), (2, 1), (4, 1), (1, 2), (1, 4), (2, 2)]     # (TP, PP) of the paper's Section 5.1 sweeps


def run_scaling(args):
    """Section 5.1 of the paper on one GPU's share: OPT-13B split TP x PP ways, two models, room for
    one, alternating blocking requests of 2 input tokens; the share of GPU 0 (rank 0, stage 0) is
    what this GPU swaps.  Reports, per split, the swap and request latency next to the link bound
    for that many bytes (the paper's own figures for this experiment are not in its text)."""
    import torch
    import paper_2306_13835_amd as P
    from synth import ShardDesc, fill_shard, token_ids, shard_bytes, param_list

    torch.cuda.set_device(0)
    torch.zeros(1, device="cuda")
    gap = 4096 if args.host_layout == "separate" else 0
    seq, steps, warmup = 2, args.steps, args.warmup
    rows = []
    link = None
    for tp, pp in SPLITS:
        desc = ShardDesc(40, 5120, 20480, 40, tp=tp, rank=0, pp=pp, stage=0)
        nbytes, n_t = shard_bytes(desc), len(param_list(desc))
        arena = torch.empty(2 * P.arena_bytes(desc), dtype=torch.uint8, device="cuda")
        ws = torch.empty(P.workspace_bytes(desc, seq), dtype=torch.uint8, device="cuda")
        out = torch.empty(1, seq, desc.out_features, dtype=torch.float32, device="cuda")
        ctx = P.Context(nbytes, arena, ws, transfer_mode=TRANSFER_MODES[args.transfer], pipeline=True)
        pool = P.HostPool(2 * (nbytes + n_t * (256 + gap)) + 8192)
        t0 = time.time()
        keep = [fill_shard(desc, 200 + 10 * tp + pp + k, alloc=lambda s: pool.take(s, gap=gap), threads=16) for k in range(2)]
        models = [ctx.register_model(desc, t) for t in keep]
        ids = [token_ids(210 + k, 1, seq, desc.vocab) for k in range(2)]
        log(f"[scaling] TP={tp} PP={pp}: shard {nbytes / 1e9:.2f} GB x 2 ready in {time.time() - t0:.1f}s")
        if link is None:                                       # the link peak, once: one 1 GiB DMA copy
            from paper_2306_13835_amd import binding as B
            cal = P.HostPool(1 << 30)
            dev = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
            ts = []
            for _ in range(5):
                ctx.stream_h2d.synchronize()
                t = time.perf_counter()
                B.op_dma(dev, cal.ptr, 1 << 30, ctx.stream_h2d)
                ctx.stream_h2d.synchronize()
                ts.append(time.perf_counter() - t)
            link = (1 << 30) / float(np.median(ts)) / 1e9
            cal.close()
            del dev
        # isolated swap-in / swap-out of one shard
        ins, outs = [], []
        for _ in range(3):
            ctx.swap_in(models[0]); ctx.wait(models[0])
            ctx.swap_out(models[0]); ctx.wait(models[0])
            i_ms, o_ms, _ = ctx.last_swap_ms(models[0])
            ins.append(i_ms); outs.append(o_ms)
        # the paper's workload: alternating blocking requests, every one swaps
        lat = []
        for i in range(warmup + steps):
            t = time.perf_counter()
            ctx.infer(models[i % 2], ids[i % 2], out=out)
            ctx.stream_compute.synchronize()
            if i >= warmup:
                lat.append((time.perf_counter() - t) * 1e3)
        ctx.sync()
        rows.append({"tp": tp, "pp": pp, "ways": tp * pp, "shard_bytes": nbytes, "tensors": n_t,
                     "swap_in_ms": round(float(np.median(ins)), 2), "swap_out_ms": round(float(np.median(outs)), 2),
                     "link_bound_ms": round(nbytes / link / 1e6, 2),
                     "request_latency_ms": round(float(np.median(lat)), 2),
                     "swap_in_gbps": round(nbytes / float(np.median(ins)) / 1e6, 2)})
        log(f"[scaling] {rows[-1]}")
        ctx.close()
        del keep, arena, ws, out
        pool.close()
    base = rows[0]
    for r in rows:
        r["speedup_vs_one_gpu"] = round(base["request_latency_ms"] / r["request_latency_ms"], 3)
    res = {"metric": "swap and request latency of one GPU's share of OPT-13B vs the (TP, PP) split (Section 5.1 workload)",
           "value": rows[-1]["request_latency_ms"], "unit": "ms", "n_gpus": 1, "steps": steps, "warmup": warmup,
           "higher_is_better": False, "data": "synthetic", "dtype": "f16", "vs_baseline": None,
           "config": {"workload": "OPT-13B, 2 models, 1 resident, alternating blocking requests of 2 tokens; GPU 0's share "
                                  "(rank 0, stage 0) per split", "transfer": args.transfer, "host_layout": args.host_layout},
           "link_peak_measured_gbps": round(link, 2),
           "paper_context": "24 GB / 32 GB/s = 0.75 s lower bound on one A100 (Section 5.1); measured figures not in the text",
           "results": rows}
    print(json.dumps(res), flush=True)
