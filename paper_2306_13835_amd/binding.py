"""ctypes binding with the same names as include/computron.h."""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libcomputron_mi355.so")

XFER_DMA, XFER_KERNEL, XFER_AUTO, XFER_DMA_IN_KERNEL_OUT, XFER_KERNEL_IN_DMA_OUT, XFER_DMA_RUNS = 0, 1, 2, 3, 4, 5
EPI_BIAS_F16, EPI_BIAS_RELU_F16, EPI_BIAS_RESID_F32, EPI_F32 = 0, 1, 2, 3

DECLARED_SYMBOLS = [
    "ctn_create", "ctn_destroy", "ctn_host_alloc", "ctn_host_free", "ctn_register_model",
    "ctn_swap_in", "ctn_swap_out", "ctn_wait", "ctn_sync", "ctn_infer", "ctn_workspace_bytes",
    "ctn_arena_bytes", "ctn_is_resident", "ctn_get_stats", "ctn_get_events", "ctn_last_swap_ms",
    "ctn_debug_read_param", "ctn_get_streams", "ctn_set_graphs", "ctn_set_mode", "ctn_last_hip_error", "ctn_strerror",
    "ctn_residency_replay", "ctn_op_copy", "ctn_op_dma", "ctn_op_embed", "ctn_op_layernorm",
    "ctn_op_gemm", "ctn_op_gemm_ws", "ctn_op_attention", "ctn_debug_gemm_tile", "ctn_engine_create", "ctn_engine_destroy",
    "ctn_engine_submit", "ctn_engine_step", "ctn_engine_pending", "ctn_engine_replay",
    "ctn_slot_bytes", "ctn_resident_blocks", "ctn_get_block_events", "ctn_block_residency_replay",
    "ctn_engine_set_prefetch", "ctn_engine_idle", "ctn_predictor_replay", "ctn_infer_stage",
    "ctn_engine_create_async", "ctn_engine_dispatch", "ctn_engine_lanes", "ctn_engine_replay_async",
    "ctn_set_discard", "ctn_op_gemm_static", "ctn_static_scratch_bytes", "ctn_set_copy_width", "ctn_test_op_gemm",
]


class ModelDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("layers", "hidden", "ffn", "heads", "vocab", "max_pos", "tp", "rank",
                                         "pp", "stage")]


class Param(C.Structure):
    _fields_ = [("host_ptr", C.c_void_p), ("nbytes", C.c_uint64), ("ndim", C.c_int32),
                ("shape", C.c_int64 * 2)]


class Config(C.Structure):
    _fields_ = [("hbm_budget_bytes", C.c_uint64), ("arena_dev", C.c_void_p), ("arena_bytes", C.c_uint64),
                ("workspace_dev", C.c_void_p), ("workspace_bytes", C.c_uint64),
                ("stream_compute", C.c_void_p), ("stream_h2d", C.c_void_p), ("stream_d2h", C.c_void_p),
                ("transfer_mode", C.c_int32), ("pipeline", C.c_int32), ("copy_blocks", C.c_int32),
                ("copy_cus", C.c_int32), ("block_residency", C.c_int32), ("discard_on_evict", C.c_int32),
                ("copy_waves_out", C.c_int32)]


class Stats(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("bytes_h2d", "bytes_d2h", "n_swap_in", "n_swap_out", "n_hit",
                                          "n_miss", "n_infer", "resident_bytes", "peak_resident_bytes",
                                          "budget_bytes", "n_partial_miss", "n_extra_evictions", "n_prefetch")]


class Event(C.Structure):
    _fields_ = [("kind", C.c_int32), ("model", C.c_int32), ("n_victims", C.c_int32),
                ("victims", C.c_int32 * 13)]


class BlockEvent(C.Structure):
    _fields_ = [("kind", C.c_int32), ("model", C.c_int32), ("first_block", C.c_int32), ("end_block", C.c_int32),
                ("use", C.c_uint64)]


class BatchRecord(C.Structure):
    _fields_ = [("start", C.c_double), ("finish", C.c_double), ("model", C.c_int32), ("count", C.c_int32),
                ("miss", C.c_int32), ("reserved", C.c_int32), ("offset", C.c_uint64)]


class CtnError(RuntimeError):
    def __init__(self, code: int, what: str, hip: int = 0):
        self.code, self.hip = code, hip
        msg = lib().ctn_strerror(code).decode()
        super().__init__(f"{what}: {msg} ({code})" + (f", hip error {hip}" if hip else ""))


_lib = None


def lib() -> C.CDLL:
    """Loads the built library; raises if it is missing (no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is not built: run `python -m paper_2306_13835_amd.build`")
    # The streams and device buffers handed to the library come from PyTorch, so both must use
    # one HIP runtime instance: PyTorch's copy has to be in the process before the library binds
    # to libamdhip64 (loading in the other order yields a second runtime that sees no device).
    import torch  # noqa: F401
    L = C.CDLL(LIB_PATH)
    vp, u64, i32, i64 = C.c_void_p, C.c_uint64, C.c_int32, C.c_int64
    P = C.POINTER
    sig = {
        "ctn_create": (C.c_int, [P(Config), P(vp)]),
        "ctn_destroy": (C.c_int, [vp]),
        "ctn_host_alloc": (C.c_int, [u64, P(vp)]),
        "ctn_host_free": (C.c_int, [vp]),
        "ctn_register_model": (C.c_int, [vp, P(ModelDesc), P(Param), C.c_size_t, u64, P(i32)]),
        "ctn_swap_in": (C.c_int, [vp, i32]),
        "ctn_swap_out": (C.c_int, [vp, i32]),
        "ctn_wait": (C.c_int, [vp, i32]),
        "ctn_sync": (C.c_int, [vp]),
        "ctn_infer": (C.c_int, [vp, i32, vp, i32, i32, vp, i32]),
        "ctn_infer_stage": (C.c_int, [vp, i32, vp, vp, i32, i32, i32, vp, i32]),
        "ctn_workspace_bytes": (u64, [P(ModelDesc), i64, i32]),
        "ctn_arena_bytes": (u64, [P(ModelDesc)]),
        "ctn_is_resident": (C.c_int, [vp, i32, P(i32)]),
        "ctn_slot_bytes": (u64, [P(ModelDesc)]),
        "ctn_resident_blocks": (C.c_int, [vp, i32, P(i32), P(i32)]),
        "ctn_get_block_events": (C.c_int, [vp, u64, P(BlockEvent), u64, P(u64), P(u64)]),
        "ctn_block_residency_replay": (C.c_int, [u64, P(i32), P(u64), i32, P(i32), u64, P(Event), P(BlockEvent), u64,
                                                 P(u64)]),
        "ctn_get_stats": (C.c_int, [vp, P(Stats)]),
        "ctn_get_events": (C.c_int, [vp, u64, P(Event), u64, P(u64), P(u64)]),
        "ctn_last_swap_ms": (C.c_int, [vp, i32, P(C.c_float), P(C.c_float), P(C.c_float), i32, P(i32)]),
        "ctn_debug_read_param": (C.c_int, [vp, i32, i32, vp, u64]),
        "ctn_get_streams": (C.c_int, [vp, P(vp), P(vp), P(vp)]),
        "ctn_set_graphs": (C.c_int, [vp, i32]),
        "ctn_set_mode": (C.c_int, [vp, i32, i32, i32]),
        "ctn_set_discard": (C.c_int, [vp, i32]),
        "ctn_set_copy_width": (C.c_int, [vp, i32, i32]),
        "ctn_last_hip_error": (C.c_int, [vp]),
        "ctn_strerror": (C.c_char_p, [C.c_int]),
        "ctn_residency_replay": (C.c_int, [u64, P(u64), i32, P(i32), u64, P(Event)]),
        "ctn_op_copy": (C.c_int, [vp, vp, u64, i32, vp]),
        "ctn_op_dma": (C.c_int, [vp, vp, u64, vp]),
        "ctn_op_embed": (C.c_int, [vp, vp, vp, vp, i32, i32, i32, i32, i32, vp]),
        "ctn_op_layernorm": (C.c_int, [vp, vp, vp, vp, i32, i32, vp]),
        "ctn_op_gemm": (C.c_int, [vp, vp, vp, vp, i32, i32, i32, i32, vp]),
        "ctn_op_gemm_ws": (C.c_int, [vp, vp, vp, vp, i32, i32, i32, i32, vp, u64, vp]),
        "ctn_op_attention": (C.c_int, [vp, vp, i32, i32, i32, i32, vp]),
        "ctn_op_gemm_static": (C.c_int, [vp, vp, vp, vp, i32, i32, i32, i32, vp]),
        "ctn_static_scratch_bytes": (u64, []),
        "ctn_debug_gemm_tile": (C.c_int, [vp, i32]),
        "ctn_test_op_gemm": (C.c_int, [vp, vp, vp, vp, i32, i32, i32, i32, vp, u64, P(i32), i32, vp]),
        "ctn_engine_create": (C.c_int, [vp, i32, i32, P(vp)]),
        "ctn_engine_destroy": (C.c_int, [vp]),
        "ctn_engine_submit": (C.c_int, [vp, i32, vp, C.c_double, P(i64)]),
        "ctn_engine_step": (C.c_int, [vp, vp, P(i64), i32, P(i32), P(i32), P(i32)]),
        "ctn_engine_pending": (C.c_int, [vp, P(i64)]),
        "ctn_engine_set_prefetch": (C.c_int, [vp, i32, i32, i32]),
        "ctn_engine_idle": (C.c_int, [vp, P(i32)]),
        "ctn_predictor_replay": (C.c_int, [i32, i32, i32, P(i32), u64, P(i32)]),
        "ctn_engine_replay": (C.c_int, [i32, i32, u64, P(u64), P(C.c_double), P(i32), u64, C.c_double, C.c_double,
                                        C.c_double, P(BatchRecord), u64, P(u64), P(u64)]),
        "ctn_engine_replay_async": (C.c_int, [i32, i32, u64, P(u64), P(C.c_double), P(i32), u64, C.c_double,
                                              C.c_double, C.c_double, P(BatchRecord), u64, P(u64), P(u64)]),
        "ctn_engine_create_async": (C.c_int, [vp, i32, i32, P(vp)]),
        "ctn_engine_dispatch": (C.c_int, [vp, P(vp), P(i64), i32, P(i32), P(i32), P(i32), P(i32)]),
        "ctn_engine_lanes": (C.c_int, [vp, P(i32)]),
    }
    for name, (res, args) in sig.items():
        f = getattr(L, name)
        f.restype, f.argtypes = res, args
    _lib = L
    return L


def _desc(d) -> ModelDesc:
    return ModelDesc(d.layers, d.hidden, d.ffn, d.heads, d.vocab, d.max_pos, d.tp, d.rank,
                     getattr(d, "pp", 1), getattr(d, "stage", 0))


def workspace_bytes(desc, max_tokens: int, n_models: int = 1) -> int:
    return int(lib().ctn_workspace_bytes(C.byref(_desc(desc)), max_tokens, n_models))


def arena_bytes(desc) -> int:
    return int(lib().ctn_arena_bytes(C.byref(_desc(desc))))


def slot_bytes(desc) -> int:
    return int(lib().ctn_slot_bytes(C.byref(_desc(desc))))


def _block_events_to_list(evs, n) -> List[Tuple[str, int, int, int, int]]:
    kinds = ("load", "evict")
    return [(kinds[e.kind], e.model, e.first_block, e.end_block, int(e.use)) for e in evs[:n]]


def block_residency_replay(budget: int, block_bytes: Sequence[Sequence[int]], trace: Sequence[int]):
    """Host-only replay of the block-granular policy: (events, block events)."""
    n = len(trace)
    nb = (C.c_int32 * len(block_bytes))(*[len(b) for b in block_bytes])
    flat = [int(x) for b in block_bytes for x in b]
    bb = (C.c_uint64 * len(flat))(*flat)
    tr = (C.c_int32 * max(n, 1))(*[int(t) for t in trace])
    out = (Event * max(n, 1))()
    cap = max(n * (len(block_bytes) + 1), 1)
    blocks = (BlockEvent * cap)()
    n_out = C.c_uint64()
    rc = lib().ctn_block_residency_replay(int(budget), nb, bb, len(block_bytes), tr, n, out, blocks, cap,
                                          C.byref(n_out))
    if rc:
        raise CtnError(rc, "ctn_block_residency_replay")
    return _events_to_list(out, n), _block_events_to_list(blocks, int(n_out.value))


def _events_to_list(evs, n) -> List[Tuple[str, int, Tuple[int, ...]]]:
    kinds = ("hit", "miss", "out")
    return [(kinds[e.kind], e.model, tuple(e.victims[i] for i in range(min(e.n_victims, 13))))
            for e in evs[:n]]


def residency_replay(budget: int, sizes: Sequence[int], trace: Sequence[int]):
    n = len(trace)
    sz = (C.c_uint64 * len(sizes))(*[int(s) for s in sizes])
    tr = (C.c_int32 * max(n, 1))(*[int(t) for t in trace])
    out = (Event * max(n, 1))()
    rc = lib().ctn_residency_replay(int(budget), sz, len(sizes), tr, n, out)
    if rc:
        raise CtnError(rc, "ctn_residency_replay")
    return _events_to_list(out, n)


def predictor_replay(n_models: int, dispatches: Sequence[int], min_count: int = 2, min_share_percent: int = 50):
    """Host-only replay of the load-ahead predictor: prediction (or None) after each dispatch."""
    n = len(dispatches)
    d = (C.c_int32 * max(n, 1))(*[int(x) for x in dispatches])
    out = (C.c_int32 * max(n, 1))()
    rc = lib().ctn_predictor_replay(n_models, min_count, min_share_percent, d, n, out)
    if rc:
        raise CtnError(rc, "ctn_predictor_replay")
    return [None if out[i] < 0 else int(out[i]) for i in range(n)]


def engine_replay(n_models: int, max_batch: int, budget: int, sizes: Sequence[int], arrival, model_of,
                  t_base: float, t_per_request: float, t_miss: float, two_lanes: bool = False):
    """Host-only replay of the scheduler; returns [(start, finish, model, request indices, miss)],
    with the lane appended to every tuple for the two-lane engine."""
    n = len(arrival)
    sz = (C.c_uint64 * len(sizes))(*[int(x) for x in sizes])
    arr = (C.c_double * max(n, 1))(*[float(x) for x in arrival])
    mod = (C.c_int32 * max(n, 1))(*[int(x) for x in model_of])
    rec = (BatchRecord * max(n, 1))()
    req = (C.c_uint64 * max(n, 1))()
    nb = C.c_uint64()
    fn = lib().ctn_engine_replay_async if two_lanes else lib().ctn_engine_replay
    rc = fn(n_models, max_batch, int(budget), sz, arr, mod, n, t_base, t_per_request, t_miss, rec, n, C.byref(nb), req)
    if rc:
        raise CtnError(rc, "ctn_engine_replay")
    out = [(r.start, r.finish, r.model, tuple(int(req[r.offset + k]) for k in range(r.count)), bool(r.miss))
           for r in rec[:nb.value]]
    if two_lanes:
        out = [b + (int(r.reserved),) for b, r in zip(out, rec[:nb.value])]
    return out


class Engine:
    """ctn_engine: per-model FIFO queues over a Context, oldest-first batches of at most max_batch."""

    def __init__(self, ctx: "Context", max_batch: int, seq: int, two_lanes: bool = False):
        """two_lanes: the asynchronous engine (hits go on while another model loads); it is driven
        with dispatch() / lanes_busy() instead of step() and needs twice the workspace."""
        self.ctx, self.max_batch, self.seq, self.two_lanes = ctx, max_batch, seq, two_lanes
        h = C.c_void_p()
        create = lib().ctn_engine_create_async if two_lanes else lib().ctn_engine_create
        rc = create(ctx.h, max_batch, seq, C.byref(h))
        if rc:
            raise CtnError(rc, "ctn_engine_create_async" if two_lanes else "ctn_engine_create")
        self.h = h
        self._served = (C.c_int64 * max_batch)()

    def submit(self, model: int, ids: np.ndarray, timestamp: float) -> int:
        ids = np.ascontiguousarray(ids, dtype=np.int32).reshape(-1)
        if ids.size != self.seq:
            raise ValueError("request length differs from the engine's")
        rid = C.c_int64()
        rc = lib().ctn_engine_submit(self.h, model, ids.ctypes.data, float(timestamp), C.byref(rid))
        if rc:
            raise CtnError(rc, "ctn_engine_submit")
        return rid.value

    def step(self, logits_out):
        """Dispatches one batch; returns (request ids, model, was_miss) or None when idle."""
        n, m, miss = C.c_int32(), C.c_int32(), C.c_int32()
        rc = lib().ctn_engine_step(self.h, _addr(logits_out), self._served, self.max_batch, C.byref(n),
                                   C.byref(m), C.byref(miss))
        if rc:
            raise CtnError(rc, "ctn_engine_step", lib().ctn_last_hip_error(self.ctx.h) if rc == -5 else 0)
        if n.value == 0:
            return None
        return [int(self._served[i]) for i in range(n.value)], m.value, bool(miss.value)

    def dispatch(self, logits_hit, logits_load):
        """Two-lane engine: dispatches at most one batch; returns (request ids, model, was_miss, lane)
        or None when nothing can go right now.  The batch's logits land in the buffer of its lane."""
        n, m, miss, lane = C.c_int32(), C.c_int32(), C.c_int32(), C.c_int32()
        bufs = (C.c_void_p * 2)(_addr(logits_hit), _addr(logits_load))
        rc = lib().ctn_engine_dispatch(self.h, bufs, self._served, self.max_batch, C.byref(n), C.byref(m),
                                       C.byref(miss), C.byref(lane))
        if rc:
            raise CtnError(rc, "ctn_engine_dispatch", lib().ctn_last_hip_error(self.ctx.h) if rc == -5 else 0)
        if n.value == 0:
            return None
        return [int(self._served[i]) for i in range(n.value)], m.value, bool(miss.value), lane.value

    def lanes_busy(self) -> Tuple[bool, bool]:
        busy = (C.c_int32 * 2)()
        rc = lib().ctn_engine_lanes(self.h, busy)
        if rc:
            raise CtnError(rc, "ctn_engine_lanes")
        return bool(busy[0]), bool(busy[1])

    def set_prefetch(self, enable: bool, min_count: int = 2, min_share_percent: int = 50):
        rc = lib().ctn_engine_set_prefetch(self.h, int(bool(enable)), min_count, min_share_percent)
        if rc:
            raise CtnError(rc, "ctn_engine_set_prefetch")

    def idle(self) -> Optional[int]:
        """Nothing to submit right now: lets the engine load the predicted next model ahead.
        Returns that model's handle, or None when nothing was started."""
        m = C.c_int32(-1)
        rc = lib().ctn_engine_idle(self.h, C.byref(m))
        if rc:
            raise CtnError(rc, "ctn_engine_idle", lib().ctn_last_hip_error(self.ctx.h) if rc == -5 else 0)
        return None if m.value < 0 else m.value

    def pending(self) -> int:
        n = C.c_int64()
        lib().ctn_engine_pending(self.h, C.byref(n))
        return n.value

    def close(self):
        if self.h:
            lib().ctn_engine_destroy(self.h)
            self.h = None


class HostPool:
    """Pinned, device-mapped host memory from ctn_host_alloc, handed out as numpy arrays."""

    def __init__(self, nbytes: int):
        self.nbytes = int(nbytes)
        p = C.c_void_p()
        rc = lib().ctn_host_alloc(self.nbytes, C.byref(p))
        if rc:
            raise CtnError(rc, f"ctn_host_alloc({nbytes})", lib().ctn_last_hip_error(None))
        self.ptr = p.value
        self._buf = (C.c_uint8 * self.nbytes).from_address(self.ptr)
        self.bytes = np.frombuffer(self._buf, dtype=np.uint8)
        self._cur = 0

    def take(self, shape, dtype=np.float16, align: int = 256, gap: int = 0) -> np.ndarray:
        """Next `align`-aligned array; `gap` bytes are skipped first, so that consecutive arrays
        are not adjacent (as separately allocated tensors would not be)."""
        n = int(np.prod(shape)) * np.dtype(dtype).itemsize
        lo = (self._cur + gap + align - 1) // align * align
        if lo + n > self.nbytes:
            raise MemoryError("HostPool exhausted")
        self._cur = lo + n
        return self.bytes[lo:lo + n].view(dtype).reshape(shape)

    def close(self):
        if self.ptr:
            self.bytes = None
            self._buf = None
            lib().ctn_host_free(self.ptr)
            self.ptr = None


def _addr(a) -> int:
    if a is None:
        return 0
    if isinstance(a, int):
        return a
    if isinstance(a, np.ndarray):
        return a.ctypes.data
    return int(a.data_ptr())      # torch tensor


class Context:
    """One ctn_ctx.  `arena`/`workspace` are torch CUDA tensors (uint8), streams are
    torch.cuda.Stream objects; torch only provides the memory and the streams."""

    def __init__(self, budget: int, arena, workspace, stream_compute=None, stream_h2d=None, stream_d2h=None,
                 transfer_mode: int = XFER_KERNEL, pipeline: bool = True, copy_blocks: int = 0,
                 copy_cus: int = 0, block_residency: bool = False, discard_on_evict: bool = False,
                 copy_waves_out: int = 0):
        """With no streams given the library creates its own three (CU-partitioned); they are
        exposed as `stream_compute`, `stream_h2d`, `stream_d2h` (torch ExternalStream)."""
        import torch
        self._keep = (arena, workspace, stream_compute, stream_h2d, stream_d2h)
        sp = [s.cuda_stream if s is not None else None for s in (stream_compute, stream_h2d, stream_d2h)]
        cfg = Config(int(budget), arena.data_ptr(), arena.numel() * arena.element_size(),
                     workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                     sp[0], sp[1], sp[2], transfer_mode, int(bool(pipeline)), copy_blocks, copy_cus,
                     int(bool(block_residency)), int(bool(discard_on_evict)), copy_waves_out)
        h = C.c_void_p()
        rc = lib().ctn_create(C.byref(cfg), C.byref(h))
        if rc:
            raise CtnError(rc, "ctn_create", lib().ctn_last_hip_error(None))
        a, b, c = C.c_void_p(), C.c_void_p(), C.c_void_p()
        lib().ctn_get_streams(h, C.byref(a), C.byref(b), C.byref(c))
        self.stream_compute, self.stream_h2d, self.stream_d2h = (
            torch.cuda.ExternalStream(p.value) for p in (a, b, c))
        self.h = h
        self._params = []
        self._out_features = []

    def _check(self, rc: int, what: str):
        if rc:
            raise CtnError(rc, what, lib().ctn_last_hip_error(self.h) if rc == -5 else 0)

    def close(self):
        if self.h:
            rc = lib().ctn_destroy(self.h)
            self.h = None
            if rc:
                raise CtnError(rc, "ctn_destroy")

    def _register(self, desc, tensors: Sequence[np.ndarray], budget: int = 0) -> int:
        arr = (Param * len(tensors))()
        for i, t in enumerate(tensors):
            arr[i].host_ptr = t.ctypes.data
            arr[i].nbytes = t.nbytes
            arr[i].ndim = t.ndim
            arr[i].shape[0] = t.shape[0]
            arr[i].shape[1] = t.shape[1] if t.ndim > 1 else 0
        out = C.c_int32(-1)
        self._check(lib().ctn_register_model(self.h, C.byref(_desc(desc)), arr, len(tensors), int(budget),
                                             C.byref(out)), "ctn_register_model")
        self._params.append(list(tensors))
        return out.value

    def swap_in(self, m: int):
        self._check(lib().ctn_swap_in(self.h, m), "ctn_swap_in")

    def swap_out(self, m: int):
        self._check(lib().ctn_swap_out(self.h, m), "ctn_swap_out")

    def wait(self, m: int):
        self._check(lib().ctn_wait(self.h, m), "ctn_wait")

    def sync(self):
        self._check(lib().ctn_sync(self.h), "ctn_sync")

    def register_model(self, desc, tensors: Sequence[np.ndarray], budget: int = 0) -> int:
        m = self._register(desc, tensors, budget)
        pp = getattr(desc, "pp", 1)
        last = getattr(desc, "stage", 0) == pp - 1
        self._out_features.append(desc.vocab // desc.tp if last else desc.hidden)
        return m

    def infer(self, m: int, ids: np.ndarray, out=None):
        """ids int32 [batch, seq] (host).  `out`: None -> new numpy fp32 array (blocking);
        a numpy array -> filled (blocking); a torch CUDA tensor -> enqueued only."""
        ids = np.ascontiguousarray(ids, dtype=np.int32)
        b, s = ids.shape
        is_dev = out is not None and not isinstance(out, np.ndarray)
        if out is None:
            out = np.empty((b, s, self._out_features[m]), dtype=np.float32)
        self._check(lib().ctn_infer(self.h, m, ids.ctypes.data, b, s, _addr(out), int(is_dev)), "ctn_infer")
        return out

    def infer_stage(self, m: int, hidden, out=None):
        """A pipeline stage after the first: `hidden` fp32 [batch, seq, hidden], a numpy array (host)
        or a torch CUDA tensor; `out` as for infer()."""
        in_dev = not isinstance(hidden, np.ndarray)
        if not in_dev:
            hidden = np.ascontiguousarray(hidden, dtype=np.float32)
        b, s = int(hidden.shape[0]), int(hidden.shape[1])
        is_dev = out is not None and not isinstance(out, np.ndarray)
        if out is None:
            out = np.empty((b, s, self._out_features[m]), dtype=np.float32)
        self._check(lib().ctn_infer_stage(self.h, m, None, _addr(hidden), int(in_dev), b, s, _addr(out), int(is_dev)),
                    "ctn_infer_stage")
        return out

    def is_resident(self, m: int) -> bool:
        o = C.c_int32()
        self._check(lib().ctn_is_resident(self.h, m, C.byref(o)), "ctn_is_resident")
        return bool(o.value)

    def resident_blocks(self, m: int) -> Tuple[int, int]:
        k, n = C.c_int32(), C.c_int32()
        self._check(lib().ctn_resident_blocks(self.h, m, C.byref(k), C.byref(n)), "ctn_resident_blocks")
        return k.value, n.value

    def block_events(self, first: int = 0):
        n, total = C.c_uint64(), C.c_uint64()
        self._check(lib().ctn_get_block_events(self.h, 0, None, 0, C.byref(n), C.byref(total)), "ctn_get_block_events")
        cap = max(int(total.value) - first, 0)
        buf = (BlockEvent * max(cap, 1))()
        self._check(lib().ctn_get_block_events(self.h, first, buf, cap, C.byref(n), C.byref(total)),
                    "ctn_get_block_events")
        return _block_events_to_list(buf, int(n.value))

    def stats(self) -> dict:
        s = Stats()
        self._check(lib().ctn_get_stats(self.h, C.byref(s)), "ctn_get_stats")
        return {n: int(getattr(s, n)) for n, _ in Stats._fields_}

    def events(self, first: int = 0):
        n, total = C.c_uint64(), C.c_uint64()
        self._check(lib().ctn_get_events(self.h, 0, None, 0, C.byref(n), C.byref(total)), "ctn_get_events")
        cap = max(int(total.value) - first, 0)
        buf = (Event * max(cap, 1))()
        self._check(lib().ctn_get_events(self.h, first, buf, cap, C.byref(n), C.byref(total)), "ctn_get_events")
        return _events_to_list(buf, int(n.value))

    def last_swap_ms(self, m: int):
        nb = C.c_int32()
        self._check(lib().ctn_last_swap_ms(self.h, m, None, None, None, 0, C.byref(nb)), "ctn_last_swap_ms")
        blocks = (C.c_float * nb.value)()
        i, o = C.c_float(), C.c_float()
        self._check(lib().ctn_last_swap_ms(self.h, m, C.byref(i), C.byref(o), blocks, nb.value, C.byref(nb)),
                    "ctn_last_swap_ms")
        return i.value, o.value, list(blocks)

    def debug_read_param(self, m: int, index: int) -> np.ndarray:
        t = self._params[m][index]
        dst = np.empty(t.shape, dtype=t.dtype)
        self._check(lib().ctn_debug_read_param(self.h, m, index, dst.ctypes.data, dst.nbytes),
                    "ctn_debug_read_param")
        return dst

    def debug_gemm_tile(self, cfg: int):
        """Test / tuning switch for this context's products (ctn_debug_gemm_tile)."""
        self._check(lib().ctn_debug_gemm_tile(self.h, cfg), "ctn_debug_gemm_tile")

    def set_graphs(self, enable: bool):
        self._check(lib().ctn_set_graphs(self.h, int(bool(enable))), "ctn_set_graphs")

    def set_discard(self, enable: bool):
        """Eviction without the copy back (the host tensors stay the single source)."""
        self._check(lib().ctn_set_discard(self.h, int(bool(enable))), "ctn_set_discard")

    def set_copy_width(self, blocks_in: int, waves_out: int = 0):
        """Copy-kernel width: workgroups of 256 threads for loads, wavefronts for offloads."""
        self._check(lib().ctn_set_copy_width(self.h, blocks_in, waves_out), "ctn_set_copy_width")

    def set_mode(self, transfer_mode: int, pipeline: bool, copy_blocks: int = 0):
        self._check(lib().ctn_set_mode(self.h, transfer_mode, int(bool(pipeline)), copy_blocks), "ctn_set_mode")


# ---- single operations (device pointers / torch tensors) ----------------------

def _op(rc, what):
    if rc:
        raise CtnError(rc, what)


def op_copy(dst, src, nbytes, blocks, stream):
    _op(lib().ctn_op_copy(_addr(dst), _addr(src), nbytes, blocks, stream.cuda_stream), "ctn_op_copy")


def op_dma(dst, src, nbytes, stream):
    _op(lib().ctn_op_dma(_addr(dst), _addr(src), nbytes, stream.cuda_stream), "ctn_op_dma")


def op_embed(ids, tok, pos, x, M, seq, hidden, vocab_local, rank, stream):
    _op(lib().ctn_op_embed(_addr(ids), _addr(tok), _addr(pos), _addr(x), M, seq, hidden, vocab_local, rank,
                           stream.cuda_stream), "ctn_op_embed")


def op_layernorm(x, g, b, out, rows, hidden, stream):
    _op(lib().ctn_op_layernorm(_addr(x), _addr(g), _addr(b), _addr(out), rows, hidden, stream.cuda_stream),
        "ctn_op_layernorm")


def op_gemm(A, W, bias, out, M, N, K, epilogue, stream):
    _op(lib().ctn_op_gemm(_addr(A), _addr(W), _addr(bias), _addr(out), M, N, K, epilogue, stream.cuda_stream),
        "ctn_op_gemm")


def op_gemm_ws(A, W, bias, out, M, N, K, epilogue, workspace, stream):
    nbytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _op(lib().ctn_op_gemm_ws(_addr(A), _addr(W), _addr(bias), _addr(out), M, N, K, epilogue, _addr(workspace), nbytes,
                             stream.cuda_stream), "ctn_op_gemm_ws")


def op_gemm_static(A, W, bias, out, M, N, K, epilogue, stream):
    """ctn_op_gemm_ws with the library's static scratch array: allocates nothing."""
    _op(lib().ctn_op_gemm_static(_addr(A), _addr(W), _addr(bias), _addr(out), M, N, K, epilogue, stream.cuda_stream),
        "ctn_op_gemm_static")


def static_scratch_bytes() -> int:
    return int(lib().ctn_static_scratch_bytes())


def op_attention(qkv, out, batch, seq, heads, head_dim, stream):
    _op(lib().ctn_op_attention(_addr(qkv), _addr(out), batch, seq, heads, head_dim, stream.cuda_stream),
        "ctn_op_attention")


def test_op_gemm(A, W, bias, out, M, N, K, epilogue, workspace, hooks, stream):
    """ctn_op_gemm_ws under an explicit list of test switches (see ctn_debug_gemm_tile); workspace may be None."""
    nbytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    hooks = [int(h) for h in hooks]
    arr = (C.c_int32 * max(len(hooks), 1))(*hooks)
    _op(lib().ctn_test_op_gemm(_addr(A), _addr(W), _addr(bias), _addr(out), M, N, K, epilogue, _addr(workspace), nbytes,
                               arr, len(hooks), stream.cuda_stream), "ctn_test_op_gemm")


test_op_gemm.__test__ = False      # (not a pytest test, whatever module imports it)
