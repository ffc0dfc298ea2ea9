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


def run_serve(args):
    import torch
    import paper_2306_13835_amd as P
    from paper_2306_13835_amd.serving import serve_trace
    from synth import CONFIGS, fill_shard, token_ids, shard_bytes, param_list, gamma_zipf_trace

    torch.cuda.set_device(0)
    torch.zeros(1, device="cuda")
    c = CONFIGS["serve8x6.7b_tp2"]
    desc, batch, seq, n_models = c["desc"], c["batch"], c["seq"], c["n_models"]
    n_req = args.requests or c["n_requests"]
    nbytes = shard_bytes(desc)
    budget = c["budget"]
    gap = 4096 if args.host_layout == "separate" else 0
    # The budget caps the bytes of models *marked resident* (at most two here).  The arena holds one
    # more range so that a victim can still be streaming out of its range while the requested model
    # streams into another one, as the paper's overlapped offload and load do (Sections 3.2, 5.1).
    resident_max = budget // nbytes
    arena = torch.empty((resident_max + 1) * P.arena_bytes(desc), dtype=torch.uint8, device="cuda")
    ws = torch.empty(P.workspace_bytes(desc, batch * seq), dtype=torch.uint8, device="cuda")
    logits = torch.empty(batch, seq, desc.vocab // desc.tp, dtype=torch.float32, device="cuda")
    ctx = P.Context(budget, arena, ws, transfer_mode={"dma": 0, "kernel": 1, "auto": 2}[args.transfer],
                    pipeline=True)
    n_t = len(param_list(desc))
    pool = P.HostPool(n_models * (nbytes + n_t * (256 + gap)) + 8192)
    t0 = time.time()
    models, keep = [], []
    for k in range(n_models):
        t = fill_shard(desc, c["wseed"] + k, alloc=lambda s: pool.take(s, gap=gap), threads=16)
        keep.append(t)
        models.append(ctx.register_model(desc, t))
    log(f"[serve] {n_models} shards ({n_models * nbytes / 1e9:.1f} GB pinned) ready in {time.time() - t0:.1f}s")
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
    st0 = ctx.stats()
    last = [time.time()]

    def progress(i):
        if time.time() - last[0] > 20:
            last[0] = time.time()
            log(f"[serve] request {i + 1}/{n_req}")

    t0 = time.perf_counter()
    lat, svc, miss = serve_trace(ctx, models, arr, mod, lambda i: ids[i], logits, progress=progress)
    wall = time.perf_counter() - t0
    ctx.sync()
    st = ctx.stats()
    events = ctx.events()[ev0:]
    # the decisions taken on the GPU path must be the ones the policy takes on the bare trace
    replay = P.residency_replay(budget, [nbytes] * n_models, [int(x) for x in mod])
    decisions_match = [(e[0], e[1], e[2]) for e in events] == replay
    n_miss = st["n_miss"] - st0["n_miss"]
    res = {
        "metric": "p99 request latency under swap (8 models, 2 resident, Gamma CV=4 / Zipf 1.5 arrivals)",
        "value": round(float(np.percentile(lat, 99)), 4), "unit": "s", "n_gpus": 1, "steps": n_req, "warmup": 3,
        "ms_per_step": round(wall / n_req * 1e3, 3), "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"serve8x6.7b_tp2: {n_models} shards x {nbytes} B, budget {budget} B, {n_req} requests "
                               f"batch {batch} x seq {seq}, serial oldest-first engine, LRU",
                   "transfer": args.transfer, "host_layout": args.host_layout,
                   "arena_bytes": int(arena.numel()), "arena_note": "budget + one transit range"},
        "latency_s": {"mean": round(float(lat.mean()), 4), "p50": round(float(np.percentile(lat, 50)), 4),
                      "p90": round(float(np.percentile(lat, 90)), 4), "p99": round(float(np.percentile(lat, 99)), 4),
                      "max": round(float(lat.max()), 4)},
        "service_ms": {"hit_p50": round(float(np.median(svc[~miss]) * 1e3), 3) if (~miss).any() else None,
                       "miss_p50": round(float(np.median(svc[miss]) * 1e3), 3) if miss.any() else None,
                       "miss_max": round(float(svc[miss].max() * 1e3), 3) if miss.any() else None},
        "misses": int(n_miss), "hit_ratio": round(1 - n_miss / n_req, 4),
        "bytes_swapped_in": st["bytes_h2d"] - st0["bytes_h2d"], "trace_seconds": round(float(arr[-1]), 2),
        "wall_seconds": round(wall, 2), "peak_resident_bytes": st["peak_resident_bytes"],
        "decisions_equal_policy_replay": bool(decisions_match),
        "hit_tokens_per_s": round(batch * seq / float(np.median(svc[~miss])), 1) if (~miss).any() else None,
    }
    ctx.close()
    del keep
    pool.close()
    print(json.dumps(res), flush=True)
