#!/usr/bin/env python3
"""Benchmark of the swap + shard-forward hot path on one MI355X.

Default workload (`--workload swap`): one GPU's share of OPT-6.7B at TP=2
(6,667,665,408 B of fp16 parameters in pinned host memory).  Two models share
an HBM budget that admits one, and requests alternate between them, so every
request is a miss: the least recently used model is swapped out on the d2h
stream while the requested one is swapped in layer by layer on the h2d stream
and its forward pass (batch 4 x seq 256) follows the layers as they land.
This is the paper's worst-case experiment (Section 5.1: alternating blocking
requests to two models with one resident), on one rank.

A step = one request: LRU decision, swap-out of the victim, swap-in, forward,
logits complete.  `value` = parameter bytes swapped in per second of wall time
over the timed steps; the device-timeline swap rates, latencies and the
roofline of the copy kernel are reported next to it.

`--workload serve` replays the multi-model serving trace (8 models, 20 GB
budget, Gamma/Zipf arrivals) and reports request latency percentiles.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
MFMA_F16_PEAK_TFLOPS = 2500.0
PCIE5_X16_NOMINAL_GBPS = 64.0
# HBM traffic of one h2d copy launch (201,404,416 B layer block) from the rocprofv3 --pmc runs
# summarised in profiles/copy_table_kernel_opt6.7b_tp2_pmc.md; None until measured.
COPY_KERNEL_TRAFFIC_BYTES = None


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def median(xs):
    xs = sorted(xs)
    return xs[len(xs) // 2]


def ev_time(torch, stream, fn):
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    fn()
    e1.record(stream)
    stream.synchronize()
    return e0.elapsed_time(e1)


def measure_link_peak(torch, P, B, pool_bytes=1 << 30, reps=10):
    """Best large single DMA copy pinned host -> HBM and back: the roofline denominator."""
    pool = P.HostPool(pool_bytes + 4096)
    h = pool.take((pool_bytes,), np.uint8)
    h[:] = 3
    d = torch.empty(pool_bytes, dtype=torch.uint8, device="cuda")
    s = torch.cuda.Stream()
    out = {}
    for name, (dst, src) in (("h2d", (d, h)), ("d2h", (h, d))):
        ts = [ev_time(torch, s, lambda: B.op_dma(dst, src, pool_bytes, s)) for _ in range(reps + 1)][1:]
        out[name] = pool_bytes / median(ts) / 1e6
    del d
    pool.close()
    return out


MODES = {"dma": 0, "kernel": 1, "auto": 2}


def measure_bidir_peak(torch, P, B, ctx, nbytes=1 << 29, reps=5):
    """Both link directions at once with large DMA copies on the library's two transfer streams."""
    pool = P.HostPool(2 * nbytes + 8192)
    h1, h2 = pool.take((nbytes,), np.uint8), pool.take((nbytes,), np.uint8)
    h1[:] = 1
    d1 = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    d2 = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    sa, sb = ctx.stream_h2d, ctx.stream_d2h
    res = []
    for _ in range(reps):
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        ev[0].record(sa); B.op_dma(d1, h1, nbytes, sa); ev[1].record(sa)
        ev[2].record(sb); B.op_dma(h2, d2, nbytes, sb); ev[3].record(sb)
        sa.synchronize(); sb.synchronize()
        res.append((nbytes / ev[0].elapsed_time(ev[1]) / 1e6, nbytes / ev[2].elapsed_time(ev[3]) / 1e6))
    del d1, d2
    pool.close()
    return {"h2d": median([r[0] for r in res]), "d2h": median([r[1] for r in res])}


def run_swap(args):
    import torch
    import paper_2306_13835_amd as P
    from paper_2306_13835_amd import binding as B
    from synth import CONFIGS, fill_shard, token_ids, shard_bytes, forward_flop, param_list

    torch.cuda.set_device(0)
    torch.zeros(1, device="cuda")            # bring the HIP context up before the library's first call
    cfg = CONFIGS[args.config]
    desc, batch, seq = cfg["desc"], cfg["batch"], cfg["seq"]
    nbytes = shard_bytes(desc)
    M = batch * seq
    log(f"[bench] {args.config}: shard {nbytes/1e9:.3f} GB, {len(param_list(desc))} tensors, M={M}")

    link = measure_link_peak(torch, P, B)
    log(f"[bench] link peak (1 GiB DMA): h2d {link['h2d']:.2f} GB/s, d2h {link['d2h']:.2f} GB/s")

    a_bytes = P.arena_bytes(desc)
    arena = torch.empty(2 * a_bytes, dtype=torch.uint8, device="cuda")
    ws = torch.empty(P.workspace_bytes(desc, M), dtype=torch.uint8, device="cuda")
    logits = torch.empty(batch, seq, desc.vocab // desc.tp, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    # library-owned streams: one hardware queue and a private set of compute units per direction
    ctx = P.Context(nbytes, arena, ws, transfer_mode=P.XFER_KERNEL, pipeline=True,
                    copy_blocks=args.copy_blocks, copy_cus=args.copy_cus)
    s_c = ctx.stream_compute
    pool = P.HostPool(2 * (nbytes + 256 * len(param_list(desc))) + 4096)
    t0 = time.time()
    tensors = [fill_shard(desc, cfg["wseed"] + k, alloc=lambda s: pool.take(s), threads=16) for k in range(2)]
    models = [ctx.register_model(desc, t) for t in tensors]
    ids = [token_ids(cfg["idseed"] + k, batch, seq, desc.vocab) for k in range(2)]
    log(f"[bench] weights generated and registered in {time.time()-t0:.1f}s")

    bidir = measure_bidir_peak(torch, P, B, ctx)
    log(f"[bench] both directions at once (DMA): h2d {bidir['h2d']:.2f} GB/s, d2h {bidir['d2h']:.2f} GB/s")

    def request(k):
        ctx.infer(models[k], ids[k], out=logits)
        s_c.synchronize()

    # ---- side measurements (outside the timed region) ---------------------------
    side = {}
    ctx.sync()
    # pure transfer, no forward, nothing else on the link: kernel path and per-tensor DMA path
    for mode, key in ((P.XFER_KERNEL, "kernel"), (P.XFER_DMA, "dma")):
        ctx.set_mode(mode, True, args.copy_blocks)
        ins, outs = [], []
        for _ in range(3):
            ctx.swap_in(models[0]); ctx.wait(models[0])
            ctx.swap_out(models[0]); ctx.wait(models[0])
            i_ms, o_ms, blocks = ctx.last_swap_ms(models[0])
            ins.append(i_ms); outs.append(o_ms)
        side[f"swap_in_ms_{key}"] = median(ins)
        side[f"swap_out_ms_{key}"] = median(outs)
    ctx.set_mode(P.XFER_KERNEL, True, args.copy_blocks)
    transfer_ms = side["swap_in_ms_kernel"]
    # first-token latency from a swapped-out model, nothing else in flight
    for pipe, key in ((True, "pipelined"), (False, "load_then_run")):
        ctx.set_mode(P.XFER_KERNEL, pipe, args.copy_blocks)
        ts = []
        for _ in range(3):
            ctx.sync()
            t = time.perf_counter()
            request(0)
            ts.append((time.perf_counter() - t) * 1e3)
            ctx.swap_out(models[0]); ctx.wait(models[0])
        side[f"first_token_ms_{key}"] = median(ts)
    ctx.set_mode(MODES[args.transfer], True, args.copy_blocks)
    # resident forward (hit path)
    request(0)
    ts = []
    for _ in range(5):
        t = time.perf_counter(); request(0); ts.append((time.perf_counter() - t) * 1e3)
    side["forward_resident_ms"] = median(ts)
    ctx.swap_out(models[0]); ctx.wait(models[0])
    ctx.sync()

    # ---- timed region -------------------------------------------------------------
    for i in range(args.warmup):
        request(i % 2)
    torch.cuda.synchronize()
    lat, in_ms, out_ms = [], [], []
    t_start = time.perf_counter()
    for i in range(args.steps):
        t = time.perf_counter()
        request((args.warmup + i) % 2)
        lat.append((time.perf_counter() - t) * 1e3)
    ctx.sync()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_start
    # per-launch durations of the h2d copy kernel, from the HIP events the library records on
    # the h2d stream after every transfer block (last step of each model)
    launch_ms, launch_bytes = [], []
    for k in range(2):
        i_ms, o_ms, blocks = ctx.last_swap_ms(models[k])
        in_ms.append(i_ms)
        out_ms.append(o_ms)
        d = np.diff([0.0] + list(blocks))
        launch_ms += list(d)
    # bytes per block: block 0 = embeddings + final LN, then equal layer blocks
    specs = param_list(desc)
    sizes = [2 * int(np.prod(s)) for _, s, _ in specs]
    b0 = sizes[0] + sizes[1] + sizes[-2] + sizes[-1]
    per_layer = sum(sizes[2:18])
    launch_bytes = ([b0] + [per_layer] * desc.layers) * 2
    avg_launch_ms = float(np.mean(launch_ms))
    avg_launch_bytes = float(np.mean(launch_bytes))
    achieved = avg_launch_bytes / avg_launch_ms / 1e6

    value = args.steps * nbytes / wall / 1e9
    flop = forward_flop(desc, batch, seq)
    result = {
        "metric": "host->HBM swap-in GB/s (demand-paged requests, swap-out overlapped, forward pipelined)",
        "value": round(value, 3), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall / args.steps * 1e3, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"{args.config} shard x2 models, budget 1 resident, alternating blocking requests, "
                               f"batch {batch} x seq {seq}", "shard_bytes": nbytes, "tensors": len(specs),
                   "transfer": args.transfer, "pipeline": "per-layer events",
                   "copy_blocks": args.copy_blocks, "copy_cus": args.copy_cus},
        "swap_in_gbps_device_timeline": round(nbytes / median(in_ms) / 1e6, 3),
        "shard_load_latency_s": round(median(in_ms) / 1e3, 5),
        "first_token_latency_ms_p50": round(median(lat), 3),
        "first_token_latency_ms_max": round(max(lat), 3),
        "link_peak_measured_gbps": {k: round(v, 3) for k, v in link.items()},
        "link_peak_both_directions_gbps": {k: round(v, 3) for k, v in bidir.items()},
        "swap_out_gbps_device_timeline": round(nbytes / median(out_ms) / 1e6, 3),
        "swap_in_frac_of_link_peak": round(nbytes / median(in_ms) / 1e6 / link["h2d"], 4),
        "isolated": {
            "swap_in_gbps_kernel": round(nbytes / side["swap_in_ms_kernel"] / 1e6, 3),
            "swap_out_gbps_kernel": round(nbytes / side["swap_out_ms_kernel"] / 1e6, 3),
            "swap_in_gbps_dma_per_tensor": round(nbytes / side["swap_in_ms_dma"] / 1e6, 3),
            "swap_out_gbps_dma_per_tensor": round(nbytes / side["swap_out_ms_dma"] / 1e6, 3),
            "pure_transfer_ms": round(transfer_ms, 3),
            "first_token_ms_pipelined": round(side["first_token_ms_pipelined"], 3),
            "first_token_ms_load_then_run": round(side["first_token_ms_load_then_run"], 3),
            "first_token_over_transfer": round(side["first_token_ms_pipelined"] / transfer_ms, 4),
            "forward_resident_ms": round(side["forward_resident_ms"], 3),
            "forward_resident_tokens_per_s": round(M / side["forward_resident_ms"] * 1e3, 1),
            "forward_resident_tflops": round(flop / side["forward_resident_ms"] / 1e9, 2),
            "forward_frac_of_mfma_f16_peak": round(flop / side["forward_resident_ms"] / 1e9 / MFMA_F16_PEAK_TFLOPS, 4),
        },
        "roofline": {
            "kernel": "copy_table_kernel<0> (host -> HBM, one launch per transfer block)",
            "bound": "host_link", "achieved": round(achieved, 3), "peak": round(link["h2d"], 3), "unit": "GB/s",
            "frac": round(achieved / link["h2d"], 4), "traffic": COPY_KERNEL_TRAFFIC_BYTES,
            "peak_source": "measured: median 1 GiB hipMemcpyAsync pinned->HBM in this run "
                           f"(PCIe Gen5 x16 nominal {PCIE5_X16_NOMINAL_GBPS} GB/s; HBM peak {HBM_PEAK_GBPS} GB/s is not the bound)",
            "bytes_per_launch": avg_launch_bytes, "avg_launch_ms": round(avg_launch_ms, 4),
            "launches_timed": len(launch_ms),
        },
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(tensors[0], ids[0], desc, nbytes)
    ctx.close()
    del tensors
    pool.close()
    print(json.dumps(result), flush=True)


def cpu_baseline(tensors, ids, desc, nbytes):
    """The CPU oracle as it stands, on this machine's host cores, on a bounded sample."""
    from oracle.swap import DeviceImage           # oracle use is confined to this baseline leg
    from oracle import opt_shard as O
    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else os.cpu_count()
    cores = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))
    img = DeviceImage([t.nbytes for t in tensors])
    t = time.perf_counter(); img.swap_in(tensors); t_in = time.perf_counter() - t
    scratch = [np.empty_like(x) for x in tensors[2:18]]
    t = time.perf_counter()
    img2 = DeviceImage([x.nbytes for x in scratch]); img2.swap_in(tensors[2:18]); img2.swap_out(scratch)
    t_layer = (time.perf_counter() - t) / 2
    t_out = t_layer * nbytes / sum(x.nbytes for x in scratch)      # swap-out extrapolated from one layer block
    del img, img2, scratch
    rows = [0]
    t = time.perf_counter()
    O.forward(tensors, ids[rows], layers=desc.layers, heads=desc.heads, tp=desc.tp, rank=desc.rank)
    t_fwd = (time.perf_counter() - t) * ids.shape[0] / len(rows)
    step = t_in + t_fwd + t_out
    return {"value": round(nbytes / step / 1e9, 4), "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": f"full-shard per-tensor memcpy swap-in ({t_in:.2f}s), swap-out extrapolated from one layer "
                      f"block ({t_out:.2f}s), fp32 forward of 1 of {ids.shape[0]} batch rows x{ids.shape[0]} "
                      f"({t_fwd:.1f}s); serial, no overlap",
            "oracle_swap_in_gbps": round(nbytes / t_in / 1e9, 3), "oracle_forward_s": round(t_fwd, 2)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", choices=["swap", "serve"], default="swap")
    ap.add_argument("--config", default="opt6.7b_tp2")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--transfer", choices=["auto", "kernel", "dma"], default="auto",
                    help="transfer mode of the timed region")
    ap.add_argument("--copy-blocks", type=int, default=0, help="workgroups per copy kernel (0: library default)")
    ap.add_argument("--copy-cus", type=int, default=0, help="compute units reserved per transfer direction")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (one rank's shard of the model); "
              "--gpus N with N > 1 is not supported", file=sys.stderr)
        sys.exit(2)
    import paper_2306_13835_amd as P
    P.lib()   # fails loudly when the HIP library is not built
    if args.workload == "serve":
        from paper_2306_13835_amd.serve_bench import run_serve
        run_serve(args)
    else:
        run_swap(args)


if __name__ == "__main__":
    main()
