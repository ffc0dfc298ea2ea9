"""Seeded fp16 parameter fills and token ids.

Every tensor is i.i.d. N(0, 0.02^2) rounded to fp16, except LayerNorm gains,
which are 1 + N(0, 0.02^2).  Tensor `i` of a shard draws from its own
counter-based Philox stream keyed by (seed, i), so tensors can be generated
in any order, in parallel and directly into caller-provided (e.g. pinned)
memory, and always hold the same bits.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from typing import Callable, List, Optional

import numpy as np

from .shapes import ShardDesc, param_list

SIGMA = 0.02
_CHUNK = 1 << 22  # elements drawn per call; the stream is the same for any chunking


def _fill_one(dst: np.ndarray, seed: int, index: int, kind: str) -> None:
    rng = np.random.Generator(np.random.Philox(key=[seed, index]))
    flat = dst.reshape(-1)
    n = flat.size
    for lo in range(0, n, _CHUNK):
        hi = min(n, lo + _CHUNK)
        z = rng.standard_normal(hi - lo, dtype=np.float32)
        z *= np.float32(SIGMA)
        if kind == "gain":
            z += np.float32(1.0)
        flat[lo:hi] = z  # float32 -> float16, round to nearest even


def fill_shard(desc: ShardDesc, seed: int,
               alloc: Optional[Callable[[tuple], np.ndarray]] = None,
               threads: int = 8) -> List[np.ndarray]:
    """Return the shard's tensors (canonical order) filled from `seed`.

    `alloc(shape)` must return a writable C-contiguous float16 array; by
    default ordinary numpy memory is used.
    """
    specs = param_list(desc)
    if alloc is None:
        alloc = lambda shape: np.empty(shape, dtype=np.float16)
    tensors = [alloc(shape) for _, shape, _ in specs]
    for t, (_, shape, _) in zip(tensors, specs):
        if t.dtype != np.float16 or tuple(t.shape) != tuple(shape) or not t.flags.c_contiguous:
            raise ValueError("alloc() must return C-contiguous float16 arrays of the requested shape")
    jobs = [(t, seed, i, kind) for i, (t, (_, _, kind)) in enumerate(zip(tensors, specs))]
    if threads <= 1:
        for j in jobs:
            _fill_one(*j)
    else:
        # biggest tensors first so the pool drains evenly
        jobs.sort(key=lambda j: -j[0].size)
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(lambda j: _fill_one(*j), jobs))
    return tensors


def token_ids(seed: int, batch: int, seq: int, vocab: int) -> np.ndarray:
    """Uniform ids over the *full* vocabulary, int32 [batch, seq]."""
    rng = np.random.Generator(np.random.Philox(key=[seed, 0x1D5]))
    return rng.integers(0, vocab, size=(batch, seq), dtype=np.int32)
