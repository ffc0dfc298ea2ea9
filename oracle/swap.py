"""CPU oracle: what a swap-in / swap-out must leave behind, byte for byte.

TEST INFRASTRUCTURE ONLY (never imported by the product path).

Section 3.2 of the paper: a load entry copies every parameter tensor of a
worker's shard from page-locked host memory into device memory, an offload
entry copies them back into the same page-locked buffers.  Section 5.1 notes
the tensors travel as separate messages.  A transfer performs no arithmetic,
so the definition is plain byte identity and the oracle is one `memcpy`
(numpy slice assignment on uint8 views) per tensor.

Parity status: fully pinned (round-trip identity, overwrite-then-restore,
poison pattern, odd tensor sizes).
"""
from __future__ import annotations

from typing import List, Sequence

import numpy as np


def as_bytes(t: np.ndarray) -> np.ndarray:
    if not t.flags.c_contiguous:
        raise ValueError("tensors must be C-contiguous")
    return t.reshape(-1).view(np.uint8)


class DeviceImage:
    """Host-side stand-in for the device copy of one shard: one byte array per tensor.

    Where tensors sit in device memory is not observable through the library
    boundary, so the image keeps them separate; only contents are compared.
    """

    def __init__(self, nbytes: Sequence[int], poison: int = 0x7E):
        self.tensors: List[np.ndarray] = [np.full(n, poison, dtype=np.uint8) for n in nbytes]
        self.resident = False

    def swap_in(self, host: Sequence[np.ndarray]) -> None:
        if len(host) != len(self.tensors):
            raise ValueError("tensor count mismatch")
        for dst, src in zip(self.tensors, host):
            b = as_bytes(src)
            if b.size != dst.size:
                raise ValueError("tensor size mismatch")
            dst[:] = b
        self.resident = True

    def swap_out(self, host: Sequence[np.ndarray]) -> None:
        if not self.resident:
            raise RuntimeError("swap_out of a shard that is not resident")
        for src, dst in zip(self.tensors, host):
            as_bytes(dst)[:] = src
        self.resident = False
