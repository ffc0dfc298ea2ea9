"""Shared plumbing for the GPU tests: torch provides device memory and streams only."""
import numpy as np
import torch

import paper_2306_13835_amd as P
from paper_2306_13835_amd import binding as B
from synth import fill_shard, param_list, shard_bytes


class Rig:
    """A context with its arena, workspace, streams and pinned host pool."""

    def __init__(self, descs, budget=None, max_tokens=64, arena_bytes=None, mode=P.XFER_KERNEL,
                 pipeline=True, host_bytes=None, torch_streams=False, gap=0, block_residency=False, two_lanes=False):
        self.dev = torch.device("cuda:0")
        torch.cuda.set_device(0)
        streams = [torch.cuda.Stream() for _ in range(3)] if torch_streams else [None] * 3
        need = [P.slot_bytes(d) * (d.local_layers + 1) if block_residency else P.arena_bytes(d) for d in descs]
        arena_bytes = arena_bytes or sum(need)
        budget = budget or sum(shard_bytes(d) for d in descs)
        ws = max(P.workspace_bytes(d, max_tokens) for d in descs) * (2 if two_lanes else 1) + 512
        self.arena = torch.empty(arena_bytes, dtype=torch.uint8, device=self.dev)
        self.workspace = torch.empty(ws, dtype=torch.uint8, device=self.dev)
        torch.cuda.synchronize()
        self.ctx = P.Context(budget, self.arena, self.workspace, *streams, transfer_mode=mode, pipeline=pipeline,
                             block_residency=block_residency)
        self.gap = gap     # bytes skipped between host tensors: > 0 makes every tensor its own region
        host_bytes = host_bytes or sum(shard_bytes(d) + (256 + gap) * len(param_list(d)) for d in descs) + 4096
        self.pool = P.HostPool(host_bytes)
        if gap:
            self.pool.bytes[:] = 0     # so that tests can see a stray write between tensors
        self.descs = list(descs)
        self.models, self.tensors = [], []

    def add(self, desc, seed):
        t = fill_shard(desc, seed, alloc=lambda shape: self.pool.take(shape, gap=self.gap))
        m = self.ctx.register_model(desc, t)
        self.models.append(m)
        self.tensors.append(t)
        return m

    def close(self):
        self.ctx.close()
        self.tensors = []
        self.pool.close()


def block_bytes(desc):
    """Parameter bytes of each transfer block: embeddings with the final LayerNorm, then each layer."""
    n = [2 * int(np.prod(shape)) for _, shape, _ in param_list(desc)]
    return [n[0] + n[1] + n[-2] + n[-1]] + [sum(n[2 + 16 * l:18 + 16 * l]) for l in range(desc.layers)]


def block_of_tensor(desc, i):
    n = 16 * desc.layers + 4
    return 0 if i < 2 or i >= n - 2 else 1 + (i - 2) // 16


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def errors(got: np.ndarray, want: np.ndarray):
    diff = np.abs(got.astype(np.float64) - want.astype(np.float64))
    return diff.max(), diff.mean() / np.abs(want).mean()
