"""Cuts one rank's whole-model parameter list into the list of one pipeline stage (test helper).

Stage p of `pp` gets layers [p*L/pp, (p+1)*L/pp); the embeddings go to stage 0, the final
LayerNorm to the last stage together with a copy of the token matrix as its head.
"""
import numpy as np


def stage_params(shard, layers, pp, stage):
    assert len(shard) == 16 * layers + 4 and layers % pp == 0
    local = layers // pp
    out = []
    if stage == 0:
        out += [shard[0], shard[1]]
    lo = 2 + 16 * local * stage
    out += list(shard[lo:lo + 16 * local])
    if stage == pp - 1:
        out += [shard[-2], shard[-1]]
        if pp > 1:
            out.append(np.array(shard[0], copy=True))
    return out
