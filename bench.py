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
# Memory traffic of one h2d copy launch of a 201,404,416 B layer block, from the two rocprofv3 --pmc
# passes summarised in profiles/counters_opt6.7b_tp2_pmc.md: FETCH_SIZE 98,373 KiB x 2.0 (calibration
# factor of that counter) of loads from the host mapping + WRITE_SIZE 196,684 KiB x 1.0 of HBM stores.
COPY_KERNEL_TRAFFIC = {"opt6.7b_tp2": {"fetch_bytes": 98373 * 2 * 1024, "write_bytes": 196684 * 1024}}
# The same for an offload launch of a layer block (HBM -> host), mean of the 8- and the 12-wavefront launches that the
# blocks of an offload beside a load alternate between: FETCH_SIZE 98,350 KiB x 2.0 from HBM, WRITE_SIZE (196,735 +
# 197,551) / 2 KiB towards the host.
COPY_KERNEL_OUT_TRAFFIC = {"opt6.7b_tp2": {"fetch_bytes": 98350 * 2 * 1024, "write_bytes": (196735 + 197551) // 2 * 1024}}
# Same two passes, the fc1 product of that shard inside its 4 x 256 forward (M=1024, N=8192, K=4096,
# 128x128x64 tiles): FETCH_SIZE 65,614 KiB x 2.0 = W once (67.1 MB) + A once per XCD (8 x 8.4 MB);
# WRITE_SIZE 16,488 KiB = the fp16 output once.
# Same passes, LayerNorm of 1024 x 4096: FETCH_SIZE 8,281 KiB x 2.0 (16.96 MB for 16.78 MB of fp32 rows),
# WRITE_SIZE 8,192 KiB (the fp16 rows).
LAYERNORM_TRAFFIC = {"opt6.7b_tp2": (8281 * 2 + 8192) * 1024}
# FETCH_SIZE over one resident forward pass of a small request (profiles/forward_small_requests_...md):
# bytes that left HBM per pass, against 6,667,665,408 B of weights.
SMALL_REQUEST_FETCH = {"opt6.7b_tp2": {8: 6849e6, 64: 7963e6}}
GEMM_FC1_TRAFFIC = {"opt6.7b_tp2": {"fetch_bytes": 65614 * 2 * 1024, "write_bytes": 16488 * 1024}}


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


MODES = {"dma": 0, "kernel": 1, "auto": 2, "dma_in_kernel_out": 3, "kernel_in_dma_out": 4, "dma_runs": 5}
GAP = 4096   # bytes between host tensors in the "separate" layout


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


def fit_alpha_beta(torch, P, B, stream, sizes=(4 << 10, 64 << 10, 1 << 20, 8 << 20, 32 << 20, 64 << 20)):
    """Section 5.1's message cost T(n) = alpha + beta * n, fitted for single host -> device messages of n bytes:
    one hipMemcpyAsync per message (what a per-tensor swap pays for each tensor) and one copy-kernel launch
    per message (what the per-block launch pays once for up to 16 tensors).  Every size is timed with HIP
    events over a run of back-to-back messages on one stream; least squares on relative error."""
    pool = P.HostPool(2 * max(sizes) + 8192)
    h = pool.take((2 * max(sizes),), np.uint8)
    h[:] = 5
    d = torch.empty(2 * max(sizes), dtype=torch.uint8, device="cuda")
    out = {}
    for name, send in (("dma_message", lambda n, off: B.op_dma(d.data_ptr() + off, h.ctypes.data + off, n, stream)),
                       ("kernel_launch", lambda n, off: B.op_copy(d.data_ptr() + off, h.ctypes.data + off, n, 32, stream))):
        ts = []
        for n in sizes:
            k = 40 if n <= (1 << 20) else 6
            offs = [(i % 2) * max(sizes) for i in range(k)]
            send(n, 0)
            stream.synchronize()
            best = min(ev_time(torch, stream, lambda: [send(n, o) for o in offs]) for _ in range(3)) / k   # ms
            ts.append(best * 1e-3)
        n_arr, t_arr = np.array(sizes, dtype=np.float64), np.array(ts)
        A = np.stack([np.ones_like(n_arr), n_arr], axis=1) / t_arr[:, None]      # relative-error weighting
        (alpha, beta), *_ = np.linalg.lstsq(A, np.ones_like(t_arr), rcond=None)
        out[name] = {"alpha_us": round(float(alpha) * 1e6, 2), "beta_ns_per_KiB": round(float(beta) * 1024e9, 3),
                     "asymptotic_gbps": round(1e-9 / float(beta), 2),
                     "per_message_us": {str(n): round(t * 1e6, 2) for n, t in zip(sizes, ts)}}
    del d
    pool.close()
    return out


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
    logits = torch.empty(batch, seq, desc.out_features, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    # library-owned streams: one hardware queue and a private set of compute units per direction
    ctx = P.Context(nbytes, arena, ws, transfer_mode=P.XFER_KERNEL, pipeline=True,
                    copy_blocks=args.copy_blocks, copy_cus=args.copy_cus, copy_waves_out=args.copy_waves_out)
    s_c = ctx.stream_compute
    # Host parameter store.  "separate": every tensor is its own pinned region with a gap before
    # the next one, as individually allocated parameter tensors are (the paper's per-tensor
    # messages, Section 5.1).  "packed": the tensors of a shard lie back to back in one slab.
    n_t = len(param_list(desc))
    pool = P.HostPool(4 * nbytes + 2 * n_t * (256 + GAP) + 2 * n_t * 256 + 8192)
    t0 = time.time()
    sep = [fill_shard(desc, cfg["wseed"] + k, alloc=lambda s: pool.take(s, gap=GAP), threads=16) for k in range(2)]
    packed = []
    for k in range(2):
        packed.append([pool.take(t.shape) for t in sep[k]])
        for dst, src in zip(packed[k], sep[k]):
            dst[...] = src
    primary, other = (sep, packed) if args.host_layout == "separate" else (packed, sep)
    tensors = primary
    models = [ctx.register_model(desc, t) for t in primary]
    models_other = [ctx.register_model(desc, t) for t in other]
    ids = [token_ids(cfg["idseed"] + k, batch, seq, desc.vocab) for k in range(2)]
    log(f"[bench] weights generated and registered in {time.time()-t0:.1f}s")

    bidir = measure_bidir_peak(torch, P, B, ctx)
    log(f"[bench] both directions at once (DMA): h2d {bidir['h2d']:.2f} GB/s, d2h {bidir['d2h']:.2f} GB/s")

    def request(k, pair=None):
        ctx.infer((pair or models)[k], ids[k], out=logits)
        s_c.synchronize()

    def alternate(pair, steps, warmup):
        """Alternating blocking requests to the two models of `pair`; returns wall seconds and latencies."""
        for m in models + models_other:
            ctx.swap_out(m)
        ctx.sync()
        for i in range(warmup):
            request(i % 2, pair)
        torch.cuda.synchronize()
        lat = []
        t_start = time.perf_counter()
        for i in range(steps):
            t = time.perf_counter()
            request((warmup + i) % 2, pair)
            lat.append((time.perf_counter() - t) * 1e3)
        ctx.sync()
        torch.cuda.synchronize()
        return time.perf_counter() - t_start, lat

    # ---- side measurements (outside the timed region) ---------------------------
    side = {}
    if not args.only_timed:
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
                side.setdefault(f"blocks_{key}", []).append(list(blocks))
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
        # the hit path at the request sizes of the paper's workloads (8 tokens; 1 x 64 in the serving trace):
        # every weight byte is read once, so the bound is shard bytes / HBM bandwidth
        if desc.has_embed:
            for tokens in (8, 64):
                if tokens > M or tokens > desc.max_pos:
                    continue
                small_ids = token_ids(cfg["idseed"] + 7, 1, tokens, desc.vocab)
                small_out = torch.empty(1, tokens, desc.out_features, dtype=torch.float32, device="cuda")
                ts = []
                for _ in range(8):
                    t = time.perf_counter()
                    ctx.infer(models[0], small_ids, out=small_out)
                    s_c.synchronize()
                    ts.append((time.perf_counter() - t) * 1e3)
                side[f"forward_resident_1x{tokens}_ms"] = median(ts[3:])
        ctx.swap_out(models[0]); ctx.wait(models[0])
        ctx.sync()

        # the same alternation on the other transfer paths, for the comparison of the copy kernel with the DMA engines:
        # one hipMemcpyAsync per run of adjacent tensors, one per tensor (the paper's per-tensor messages), and the
        # copy kernel at full width in both directions (AUTO narrows the kernel of an offload that runs beside a load: a wide one takes the link from the load)
        side["paths"] = {}
        for alt, mode, waves_out in (("dma_runs", "dma_runs", 0), ("dma_per_tensor", "dma", 0),
                                     ("kernel_both_ways_full_width", "kernel", 0), ("kernel_both_ways_offload_8_waves", "kernel", 8)):
            ctx.set_mode(MODES[mode], True, args.copy_blocks)
            ctx.set_copy_width(args.copy_blocks, waves_out)
            w_alt, lat_alt = alternate(models, 4, 2)
            side["paths"][alt] = {"ms_per_step": round(w_alt / 4 * 1e3, 3), "value_gbps": round(4 * nbytes / w_alt / 1e9, 3),
                                  "step_latencies_ms": [round(x, 1) for x in lat_alt]}
        ctx.set_copy_width(args.copy_blocks, args.copy_waves_out)

        # the same alternation if evictions only freed the device copy (parameters are read-only on the device);
        # an option, off by default: the paper's swap-out is a real copy and so is the timed region's
        ctx.set_mode(MODES[args.transfer], True, args.copy_blocks)
        ctx.set_discard(True)
        w_disc, _ = alternate(models, 4, 2)
        ctx.set_discard(False)
        side["discard_ms_per_step"] = w_disc / 4 * 1e3

        # the same alternation on the other host layout, for the report
        ctx.set_mode(MODES[args.transfer], True, args.copy_blocks)
        w_other, lat_other = alternate(models_other, 4, 2)
        side["other_layout_ms_per_step"] = w_other / 4 * 1e3

    ctx.set_mode(MODES[args.transfer], True, args.copy_blocks)
    ctx.set_copy_width(args.copy_blocks, args.copy_waves_out)
    # ---- timed region -------------------------------------------------------------
    in_ms, out_ms = [], []
    wall, lat = alternate(models, args.steps, args.warmup)
    # per-launch durations of the h2d transfers of the timed region, from the HIP events the
    # library records on the h2d stream after every transfer block (last load of each model)
    specs = param_list(desc)
    sizes = [2 * int(np.prod(sh)) for _, sh, _ in specs]
    n_front = 2 if desc.has_embed else 0                    # block 0: the tensors outside the layers
    per_layer = sum(sizes[n_front:n_front + 16])            # then one equal block per layer
    block_bytes = [sum(sizes) - per_layer * desc.local_layers] + [per_layer] * desc.local_layers
    timed_blocks = []
    for k in range(2):
        i_ms, o_ms, blocks = ctx.last_swap_ms(models[k])
        in_ms.append(i_ms)
        out_ms.append(o_ms)
        timed_blocks.append(list(blocks))
    # AUTO on a host list in separate pieces: a miss that evicts loads its matrices through the DMA engines (one
    # copy each) and gathers the small tensors of a block with one narrow copy-kernel launch, while its victim's
    # offload goes through the copy kernel; a packed list takes DMA copies both ways
    loads_by_kernel = args.transfer in ("kernel", "kernel_in_dma_out")
    offloads_by_kernel = args.transfer in ("kernel", "dma_in_kernel_out") or \
        (args.transfer == "auto" and args.host_layout == "separate")
    roof_blocks = timed_blocks
    roof_where = "timed region: the last load of each of the two models (2 x %d launches)" % len(block_bytes)
    launch_ms = [d for blocks in roof_blocks for d in np.diff([0.0] + blocks)]
    avg_launch_ms = float(np.mean(launch_ms))
    avg_launch_bytes = float(np.mean(block_bytes))
    achieved = avg_launch_bytes / avg_launch_ms / 1e6

    if args.only_timed:
        n_launch = len(block_bytes)
        out_launch_ms = float(np.mean(out_ms)) / n_launch
        result = {"metric": "host->HBM swap-in GB/s (demand-paged requests, swap-out overlapped, forward pipelined)",
                  "value": round(args.steps * nbytes / wall / 1e9, 3), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
                  "warmup": args.warmup, "ms_per_step": round(wall / args.steps * 1e3, 3), "higher_is_better": True,
                  "dtype": "f16", "data": "synthetic",
                  "config": {"workload": f"{args.config} shard x2 models, budget 1 resident, alternating blocking requests, "
                                         f"batch {batch} x seq {seq}; timed region only (for profilers)",
                             "transfer": args.transfer, "host_layout": args.host_layout},
                  "step_latencies_ms": [round(x, 1) for x in lat],
                  "load_avg_block_ms": round(avg_launch_ms, 4), "load_gbps": round(achieved, 3),
                  "offload_avg_launch_ms": round(out_launch_ms, 4),
                  "offload_gbps": round(avg_launch_bytes / out_launch_ms / 1e6, 3), "bytes_per_launch": avg_launch_bytes,
                  "launches_per_swap": n_launch}
        ctx.close()
        del tensors
        pool.close()
        print(json.dumps(result), flush=True)
        return

    # the largest product of a layer (fc1: [M, h] x [f/t, h]^T) alone, for the MFMA roofline
    gM, gN, gK = M, desc.local_ffn, desc.hidden
    ga = torch.randn(gM, gK, device="cuda").half()
    gw = torch.randn(gN, gK, device="cuda").half()
    gb = torch.zeros(gN, device="cuda").half()
    go = torch.empty(gM, gN, device="cuda").half()
    sg = torch.cuda.Stream()
    B.op_gemm(ga, gw, gb, go, gM, gN, gK, P.EPI_BIAS_RELU_F16, sg)
    reps = 20
    gms = ev_time(torch, sg, lambda: [B.op_gemm(ga, gw, gb, go, gM, gN, gK, P.EPI_BIAS_RELU_F16, sg)
                                      for _ in range(reps)]) / reps
    gemm_tflops = 2.0 * gM * gN * gK / gms / 1e9

    # LayerNorm of the forward pass's activations [M, h] alone, for the HBM roofline of the elementwise kernels:
    # 16 input buffers in rotation (more than the last-level cache holds), fp32 in, fp16 out
    lM, lh, lrot = M, desc.hidden, 16
    lx = [torch.randn(lM, lh, device="cuda") for _ in range(lrot)]
    lg, lb = torch.ones(lh, device="cuda").half(), torch.zeros(lh, device="cuda").half()
    lo = torch.empty(lM, lh, device="cuda").half()
    B.op_layernorm(lx[0], lg, lb, lo, lM, lh, sg)
    lreps = 4 * lrot
    lms = ev_time(torch, sg, lambda: [B.op_layernorm(lx[i % lrot], lg, lb, lo, lM, lh, sg) for i in range(lreps)]) / lreps
    ln_bytes = 6 * lM * lh
    del lx

    value = args.steps * nbytes / wall / 1e9
    flop = forward_flop(desc, batch, seq)
    ms_step = wall / args.steps * 1e3
    n_launch = len(block_bytes)
    link_note = ("measured: median 1 GiB hipMemcpyAsync pinned<->HBM in this run, one direction at a time "
                 f"(PCIe Gen5 x16 nominal {PCIE5_X16_NOMINAL_GBPS} GB/s; HBM peak {HBM_PEAK_GBPS} GB/s is not the bound)")
    if loads_by_kernel:
        roofline = {
            "kernel": "copy_table_kernel<0, 256> (host -> HBM, one launch per transfer block)",
            "bound": "host_link", "achieved": round(achieved, 3), "peak": round(link["h2d"], 3), "unit": "GB/s",
            "frac": round(achieved / link["h2d"], 4),
            "traffic": sum(COPY_KERNEL_TRAFFIC[args.config].values()) if args.config in COPY_KERNEL_TRAFFIC else None,
            "traffic_detail": dict(COPY_KERNEL_TRAFFIC.get(args.config, {}),
                                   note="per layer-block launch: bytes loaded over the host link + bytes stored to HBM; "
                                        "algorithmic = 201,404,416 each"),
            "peak_source": link_note,
            "bytes_per_launch": avg_launch_bytes, "avg_launch_ms": round(avg_launch_ms, 4),
            "launches_timed": len(launch_ms), "measured_over": roof_where,
            "note": "every launch of the timed region runs beside an offload on the link's other direction; alone the "
                    "same kernel reaches isolated.swap_in_gbps_kernel",
        }
    else:
        roofline = {
            "kernel": ("hipMemcpyAsync host -> HBM for the matrices (DMA engines, not a kernel of this library) + one "
                       "copy_table_kernel<0, 256> launch per transfer block that gathers its small tensors"
                       if args.transfer == "auto" and args.host_layout == "separate" else
                       "hipMemcpyAsync host -> HBM (DMA engines / the runtime's copy shader), not a kernel of this library"),
            "bound": "host_link", "achieved": round(achieved, 3), "peak": round(link["h2d"], 3), "unit": "GB/s",
            "frac": round(achieved / link["h2d"], 4), "traffic": None, "peak_source": link_note,
            "bytes_per_launch": avg_launch_bytes, "avg_launch_ms": round(avg_launch_ms, 4),
            "launches_timed": len(launch_ms), "measured_over": roof_where + " (per transfer block: its copies together)",
        }
    out_launch_ms = float(np.mean(out_ms)) / n_launch
    roofline_out = {
        "kernel": ("copy_table_kernel<1, 256> (HBM -> host, one launch per transfer block)" if offloads_by_kernel
                   else "hipMemcpyAsync HBM -> host, not a kernel of this library"),
        "bound": "host_link", "achieved": round(avg_launch_bytes / out_launch_ms / 1e6, 3), "peak": round(link["d2h"], 3),
        "unit": "GB/s", "frac": round(avg_launch_bytes / out_launch_ms / 1e6 / link["d2h"], 4),
        "traffic": (sum(COPY_KERNEL_OUT_TRAFFIC[args.config].values())
                    if offloads_by_kernel and args.config in COPY_KERNEL_OUT_TRAFFIC else None),
        "traffic_detail": (dict(COPY_KERNEL_OUT_TRAFFIC[args.config], note="per layer-block launch: bytes fetched from HBM + bytes "
                                "written over the host link; algorithmic = 201,404,416 each")
                           if offloads_by_kernel and args.config in COPY_KERNEL_OUT_TRAFFIC else None),
        "bytes_per_launch": avg_launch_bytes, "avg_launch_ms": round(out_launch_ms, 4), "launches_timed": 2 * n_launch,
        "measured_over": "timed region: the last offload of each of the two models, start event to end event over its "
                         f"{n_launch} back-to-back launches",
        "peak_source": link_note,
        "note": "every launch of the timed region runs beside a load on the link's other direction (both at once the link "
                "carries link_peak_both_directions_gbps); alone the same kernel reaches isolated.swap_out_gbps_kernel",
    }
    # Every step moves the shard once in each direction.  With both directions busy the link carries less
    # per direction than alone (link_peak_both_directions_gbps, large DMA copies): the step cannot be shorter
    # than the slower direction's share of it.
    slow = min(bidir["h2d"], bidir["d2h"])
    two_way = {"bytes_each_way_per_step": nbytes, "slower_direction_gbps_under_two_way_dma": round(slow, 3),
               "bound_ms_per_step": round(nbytes / slow / 1e6, 3), "ms_per_step": round(ms_step, 3),
               "frac": round(nbytes / slow / 1e6 / ms_step, 4)}
    kt = side["paths"]["kernel_both_ways_offload_8_waves"]
    kernel_throughout = {"note": "the timed workload with every load and offload through the copy kernel (loads 128 "
                                 "wavefronts wide, offloads 8), none through the DMA engines",
                         "ms_per_step": kt["ms_per_step"], "value_gbps": kt["value_gbps"],
                         "over_headline_ms": round(kt["ms_per_step"] / ms_step, 4)}
    alpha_beta = fit_alpha_beta(torch, P, B, sg)
    # what the fitted model predicts for this shard's swap-in, against what was measured alone on the link
    ab_d, ab_k = alpha_beta["dma_message"], alpha_beta["kernel_launch"]
    alpha_beta["shard_swap_in_ms"] = {
        "per_tensor_dma_model": round(n_t * ab_d["alpha_us"] * 1e-3 + nbytes / ab_d["asymptotic_gbps"] / 1e6, 2),
        "per_tensor_dma_measured": round(side["swap_in_ms_dma"], 2),
        "per_block_kernel_model": round(n_launch * ab_k["alpha_us"] * 1e-3 + nbytes / ab_k["asymptotic_gbps"] / 1e6, 2),
        "per_block_kernel_measured": round(side["swap_in_ms_kernel"], 2),
        "messages": {"per_tensor_dma": n_t, "per_block_kernel": n_launch}}
    result = {
        "metric": "host->HBM swap-in GB/s (demand-paged requests, swap-out overlapped, forward pipelined)",
        "value": round(value, 3), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"{args.config} shard x2 models, budget 1 resident, alternating blocking requests, "
                               f"batch {batch} x seq {seq}", "shard_bytes": nbytes, "tensors": n_t,
                   "transfer": args.transfer, "host_layout": args.host_layout, "pipeline": "per-layer events",
                   "copy_blocks": args.copy_blocks, "copy_cus": args.copy_cus, "copy_waves_out": args.copy_waves_out},
        "swap_in_gbps_device_timeline": round(nbytes / median(in_ms) / 1e6, 3),
        "shard_load_latency_s": round(median(in_ms) / 1e3, 5),
        "first_token_latency_ms_p50": round(median(lat), 3),
        "first_token_latency_ms_max": round(max(lat), 3),
        "step_latencies_ms": [round(x, 1) for x in lat],
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
            "forward_small_requests": {
                f"1x{t}": {"ms": round(side[f"forward_resident_1x{t}_ms"], 3),
                           "weight_stream_bound_ms": round(nbytes / HBM_PEAK_GBPS / 1e6, 3),
                           "frac_of_hbm_peak": round(nbytes / HBM_PEAK_GBPS / 1e6 / side[f"forward_resident_1x{t}_ms"], 4),
                           "traffic": SMALL_REQUEST_FETCH.get(args.config, {}).get(t)}
                for t in (8, 64) if f"forward_resident_1x{t}_ms" in side},
        },
        "roofline": roofline_out if (offloads_by_kernel and not loads_by_kernel) else roofline,
        "roofline_load": roofline,
        "roofline_offload": roofline_out,
        "link_bound_two_way": two_way,
        "roofline_gemm": {
            "kernel": f"gemm_dma_kernel<1> (128x128x64 tiles) fc1 shape M={gM} N={gN} K={gK}, bias+ReLU epilogue",
            "bound": "mfma", "achieved": round(gemm_tflops, 2), "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": round(gemm_tflops / MFMA_F16_PEAK_TFLOPS, 4),
            "traffic": sum(GEMM_FC1_TRAFFIC[args.config].values()) if args.config in GEMM_FC1_TRAFFIC else None,
            "algorithmic_bytes": 2 * (gM * gK + gN * gK + gM * gN),
            "avg_launch_ms": round(gms, 4), "launches_timed": reps,
        },
        "without_copy_back": {"note": "option discard_on_evict (not the paper's swap-out, not the timed region): "
                                      "evictions free the device copy only", "ms_per_step": round(side["discard_ms_per_step"], 3),
                              "value_gbps": round(nbytes / side["discard_ms_per_step"] / 1e6, 3)},
        "roofline_layernorm": {
            "kernel": f"layernorm_kernel, {lM} rows x {lh} (fp32 in, fp16 out), inputs rotating through {lrot} buffers",
            "bound": "hbm", "achieved": round(ln_bytes / lms / 1e6, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": round(ln_bytes / lms / 1e6 / HBM_PEAK_GBPS, 4),
            "traffic": LAYERNORM_TRAFFIC.get(args.config), "algorithmic_bytes": ln_bytes,
            "avg_launch_ms": round(lms, 5), "launches_timed": lreps,
        },
        "transfer_paths_compared": dict(side["paths"], note="the timed workload, 4 steps each, on the other transfer paths "
                                        "(dma_runs: one hipMemcpyAsync per run of adjacent tensors in both directions; dma_per_tensor: "
                                        "the paper's per-tensor messages; kernel_both_ways: the copy kernel for loads and offloads); "
                                        f"the timed region ran '{args.transfer}'"),
        "kernel_transfers_throughout": kernel_throughout,
        "alpha_beta_fit": alpha_beta,
        "other_host_layout": {
            "layout": "packed" if args.host_layout == "separate" else "separate",
            "ms_per_step": round(side["other_layout_ms_per_step"], 3),
            "value_gbps": round(nbytes / side["other_layout_ms_per_step"] / 1e6, 3),
        },
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(tensors[0], ids[0], desc, nbytes)
    ctx.close()
    del tensors, sep, packed, primary, other, arena, ws, logits
    pool.close()
    torch.cuda.empty_cache()
    if args.serve_requests > 0:
        # (53 GB of pinned host memory: a box that cannot give that much still reports the timed region)
        try:
            result["serving"] = serving_leg(args)
        except (MemoryError, RuntimeError, OSError) as e:
            result["serving"] = {"error": f"{type(e).__name__}: {e}"}
    print(json.dumps(result), flush=True)


def serving_leg(args):
    """The second half of the metric, p99 request latency under swap, on a bounded prefix of the serving
    workload (8 shards of the opt6.7b TP=2 shape, budget 20e9 B, Gamma CV 4 / Zipf 1.5 arrivals at 20
    requests/s, 1 x 64 tokens): the paper's engine as it stands (serial, oldest first, whole-model LRU) and
    this library's asynchronous two-lane engine with residency per transfer block."""
    from paper_2306_13835_amd.serve_bench import serve_setup, serve_once
    c, pool, keep = serve_setup(args.host_layout)
    n_req = min(args.serve_requests, c["n_requests"])
    out = {"workload": f"serve8x6.7b_tp2 reduced to the first {n_req} of {c['n_requests']} requests of the seeded trace "
                       f"(8 shards, budget {c['budget']} B, real-time open-loop replay)", "requests": n_req}
    keys = ("latency_s", "misses", "hit_ratio", "partial_misses", "decisions_equal_policy_replay", "service_ms",
            "bytes_swapped_in", "wall_seconds", "trace_seconds")
    for name, kw in (("serial_engine_whole_models", {}), ("two_lane_engine_block_residency", {"blocks": True, "two_lanes": True})):
        log(f"[bench] serving leg: {name}, {n_req} requests")
        r = serve_once(c, keep, n_req, args.transfer, args.host_layout, **kw)
        out[name] = {k: r[k] for k in keys}
        out[name]["p99_latency_s"] = r["latency_s"]["p99"]
        out[name]["p50_latency_s"] = r["latency_s"]["p50"]
    del keep
    pool.close()
    return out


def run_counters(args):
    """Short run for `rocprofv3 --pmc`: a plain device-to-device copy of known size (calibration of
    FETCH_SIZE / WRITE_SIZE), then one kernel-mode swap-in, one resident forward, one swap-out."""
    import torch
    import paper_2306_13835_amd as P
    from paper_2306_13835_amd import binding as B
    from synth import CONFIGS, fill_shard, token_ids, shard_bytes, param_list
    torch.cuda.set_device(0)
    torch.zeros(1, device="cuda")
    cfg = CONFIGS[args.config]
    desc, batch, seq = cfg["desc"], cfg["batch"], cfg["seq"]
    if args.shape:                                             # e.g. 1x64: the forward pass of a small request instead
        batch, seq = (int(x) for x in args.shape.lower().split("x"))
    nbytes, M = shard_bytes(desc), batch * seq
    arena = torch.empty(P.arena_bytes(desc), dtype=torch.uint8, device="cuda")
    ws = torch.empty(P.workspace_bytes(desc, M), dtype=torch.uint8, device="cuda")
    logits = torch.empty(batch, seq, desc.out_features, dtype=torch.float32, device="cuda")
    ctx = P.Context(nbytes, arena, ws, transfer_mode=P.XFER_KERNEL, pipeline=False)
    pool = P.HostPool(nbytes + len(param_list(desc)) * (256 + GAP) + 8192)
    tensors = fill_shard(desc, cfg["wseed"], alloc=lambda s: pool.take(s, gap=GAP), threads=16)
    m = ctx.register_model(desc, tensors)
    cal = 1 << 30
    a = torch.zeros(cal, dtype=torch.uint8, device="cuda")
    b = torch.empty(cal, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    B.op_copy(b, a, cal, 1024, ctx.stream_compute)           # copy_table_kernel<2>: reads and writes 2^30 B
    ctx.stream_compute.synchronize()
    ctx.swap_in(m); ctx.wait(m)                              # copy_table_kernel<0> x (layers + 1)
    for _ in range(max(1, args.repeat)):
        ctx.infer(m, token_ids(cfg["idseed"], batch, seq, desc.vocab), out=logits)
    ctx.sync()
    ctx.swap_out(m); ctx.wait(m)                             # copy_table_kernel<1, 256> x (layers + 1), 128 wavefronts wide
    for waves in (8, 12):                                    # the two widths of an offload that runs beside a load
        ctx.set_copy_width(0, waves)
        ctx.swap_in(m); ctx.wait(m)
        ctx.swap_out(m); ctx.wait(m)
    ctx.close()
    del tensors
    pool.close()
    print(json.dumps({"workload": "counters", "config": args.config, "calibration_copy_bytes": cal,
                      "shard_bytes": nbytes, "batch": batch, "seq": seq, "forwards": max(1, args.repeat)}), flush=True)


def cpu_baseline(tensors, ids, desc, nbytes):
    """The CPU oracle as it stands, on this machine's host cores, on a bounded sample."""
    from oracle.swap import DeviceImage           # oracle use is confined to this baseline leg
    from oracle import opt_shard as O
    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else os.cpu_count()
    blas_threads = None
    try:                                          # the threads numpy's BLAS really uses for the oracle's matmuls
        from threadpoolctl import threadpool_info
        blas_threads = max([int(p.get("num_threads", 0)) for p in threadpool_info() if p.get("user_api") == "blas"] or [0]) or None
    except Exception:
        pass
    img = DeviceImage([t.nbytes for t in tensors])
    t = time.perf_counter(); img.swap_in(tensors); t_in = time.perf_counter() - t
    back = [np.empty_like(x) for x in tensors]    # the whole shard back into host tensors of the same sizes
    t = time.perf_counter(); img.swap_out(back); t_out = time.perf_counter() - t
    del img, back
    rows = [0]
    t = time.perf_counter()
    O.forward_stage(tensors, ids[rows], layers=desc.layers, heads=desc.heads, tp=desc.tp, rank=desc.rank,
                    pp=desc.pp, stage=desc.stage)
    t_fwd = (time.perf_counter() - t) * ids.shape[0] / len(rows)
    step = t_in + t_fwd + t_out
    return {"value": round(nbytes / step / 1e9, 4), "unit": "GB/s", "cores": blas_threads or cores, "kind": "oracle",
            "sample": f"full-shard per-tensor memcpy swap-in ({t_in:.2f}s) and swap-out ({t_out:.2f}s), one thread; fp32 "
                      f"forward of 1 of {ids.shape[0]} batch rows, extrapolated x{ids.shape[0]} ({t_fwd:.1f}s), "
                      f"{blas_threads or '?'} BLAS threads; serial, no overlap",
            "cores_note": f"threads the oracle's matrix products ran on (numpy BLAS pool); the box offers {cores} to this process",
            "oracle_swap_in_gbps": round(nbytes / t_in / 1e9, 3), "oracle_swap_out_gbps": round(nbytes / t_out / 1e9, 3),
            "oracle_forward_s": round(t_fwd, 2)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", choices=["swap", "serve", "grid", "cyclic", "scaling", "mixed", "counters"], default="swap")
    ap.add_argument("--config", default="opt6.7b_tp2")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only-timed", action="store_true",
                    help="swap workload: warm-up and timed steps only, none of the side measurements (for profiler runs)")
    ap.add_argument("--duration", type=float, default=30.0, help="grid workload: seconds of arrivals per trial")
    ap.add_argument("--requests", type=int, default=0, help="serve workload: number of requests (0: all 2000)")
    ap.add_argument("--transfer", choices=sorted(MODES), default="auto",
                    help="transfer mode of the timed region")
    ap.add_argument("--host-layout", choices=["separate", "packed"], default="separate",
                    help="how the parameter tensors lie in pinned host memory")
    ap.add_argument("--block-residency", action="store_true",
                    help="serve workload: residency per transfer block instead of per model")
    ap.add_argument("--two-lane", action="store_true",
                    help="serve / grid workloads: the asynchronous engine (batches of loaded models go on while another loads)")
    ap.add_argument("--load-ahead", action="store_true",
                    help="serve workload with --two-lane: let the idle engine load the predicted next model")
    ap.add_argument("--shape", default="", help="counters workload: BATCHxSEQ of the forward pass (default: the config's)")
    ap.add_argument("--repeat", type=int, default=1, help="counters workload: number of resident forward passes")
    ap.add_argument("--copy-blocks", type=int, default=0, help="workgroups per copy kernel (0: library default)")
    ap.add_argument("--copy-cus", type=int, default=0, help="compute units reserved per transfer direction")
    ap.add_argument("--copy-waves-out", type=int, default=0, help="wavefronts of an offload's copy kernel (0: library's choice)")
    ap.add_argument("--serve-requests", type=int, default=400,
                    help="swap workload: requests of the serving trace replayed after the timed region for the latency "
                         "percentiles (0: skip that leg)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (one rank's shard of the model); "
              "--gpus N with N > 1 is not supported", file=sys.stderr)
        sys.exit(2)
    import paper_2306_13835_amd as P
    P.lib()   # fails loudly when the HIP library is not built
    if args.workload == "counters":
        run_counters(args)
    elif args.workload == "grid":
        from paper_2306_13835_amd.serve_bench import run_grid
        run_grid(args)
    elif args.workload == "serve":
        from paper_2306_13835_amd.serve_bench import run_serve
        run_serve(args)
    elif args.workload == "cyclic":
        from paper_2306_13835_amd.serve_bench import run_cyclic
        run_cyclic(args)
    elif args.workload == "scaling":
        from paper_2306_13835_amd.serve_bench import run_scaling
        run_scaling(args)
    elif args.workload == "mixed":
        from paper_2306_13835_amd.serve_bench import run_mixed
        run_mixed(args)
    else:
        run_swap(args)


if __name__ == "__main__":
    main()
