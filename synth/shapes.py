"""Shapes of one tensor-parallel rank's share of an OPT decoder.

The paper evaluates OPT-13B in fp16 (Section 5.1) and shards every tensor
across the TP group so that each rank keeps the same *number* of tensors at
1/TP of the size (Section 5.1, alpha-beta discussion).  This module lists the
tensors one rank holds, in the order the forward pass touches them, which is
also the order they are swapped in.

Sharding convention (Megatron style): q/k/v/fc1 are split along the output
dimension (column parallel), out-proj/fc2 along the input dimension (row
parallel) with their bias replicated, the token embedding is split along the
vocabulary, positions and LayerNorms are replicated.
"""
from __future__ import annotations

from dataclasses import dataclass, asdict
from typing import Dict, List, Tuple

POS_OFFSET = 2  # OPT stores position rows shifted by two


@dataclass(frozen=True)
class ShardDesc:
    layers: int
    hidden: int
    ffn: int
    heads: int
    vocab: int = 50272
    max_pos: int = 2048
    tp: int = 1
    rank: int = 0
    pp: int = 1      # pipeline stages the model is cut into (Section 5.1 evaluates TP x PP splits)
    stage: int = 0   # this shard's stage: layers [stage*L/pp, (stage+1)*L/pp)

    def __post_init__(self):
        if self.hidden % self.heads or self.heads % self.tp or self.ffn % self.tp \
                or self.vocab % self.tp or not (0 <= self.rank < self.tp) \
                or self.pp < 1 or self.layers % self.pp or not (0 <= self.stage < self.pp):
            raise ValueError(f"inconsistent shard description {self}")

    @property
    def local_layers(self) -> int:
        return self.layers // self.pp

    @property
    def first_layer(self) -> int:
        return self.stage * self.local_layers

    @property
    def has_embed(self) -> bool:
        return self.stage == 0

    @property
    def has_head(self) -> bool:
        return self.stage == self.pp - 1

    @property
    def out_features(self) -> int:
        """Width of what one inference emits: a vocabulary slice of logits, or the residual stream."""
        return self.local_vocab if self.has_head else self.hidden

    @property
    def head_dim(self) -> int:
        return self.hidden // self.heads

    @property
    def local_heads(self) -> int:
        return self.heads // self.tp

    @property
    def local_hidden(self) -> int:
        return self.hidden // self.tp

    @property
    def local_ffn(self) -> int:
        return self.ffn // self.tp

    @property
    def local_vocab(self) -> int:
        return self.vocab // self.tp

    @property
    def pos_rows(self) -> int:
        return self.max_pos + POS_OFFSET

    def asdict(self) -> Dict[str, int]:
        return asdict(self)


# kind: "normal" -> N(0, sigma^2); "gain" -> 1 + N(0, sigma^2) (LayerNorm weight)
ParamSpec = Tuple[str, Tuple[int, ...], str]

LAYER_TENSORS = 16
EXTRA_TENSORS = 4


def param_list(d: ShardDesc) -> List[ParamSpec]:
    """Canonical tensor list of one rank (and pipeline stage), forward order.

    Whole model on the rank (pp == 1): `16*L + 4` tensors.  With pipeline
    stages: the embeddings only on stage 0, the stage's own layers, the final
    LayerNorm only on the last stage, followed there by that stage's copy of
    the tied head matrix (`lm_head`).
    """
    h, hl, fl = d.hidden, d.local_hidden, d.local_ffn
    out: List[ParamSpec] = []
    if d.has_embed:
        out += [("embed_tokens", (d.local_vocab, h), "normal"),
                ("embed_positions", (d.pos_rows, h), "normal")]
    for i in range(d.first_layer, d.first_layer + d.local_layers):
        p = f"layers.{i}."
        out += [
            (p + "ln1.w", (h,), "gain"), (p + "ln1.b", (h,), "normal"),
            (p + "q.w", (hl, h), "normal"), (p + "q.b", (hl,), "normal"),
            (p + "k.w", (hl, h), "normal"), (p + "k.b", (hl,), "normal"),
            (p + "v.w", (hl, h), "normal"), (p + "v.b", (hl,), "normal"),
            (p + "o.w", (h, hl), "normal"), (p + "o.b", (h,), "normal"),
            (p + "ln2.w", (h,), "gain"), (p + "ln2.b", (h,), "normal"),
            (p + "fc1.w", (fl, h), "normal"), (p + "fc1.b", (fl,), "normal"),
            (p + "fc2.w", (h, fl), "normal"), (p + "fc2.b", (h,), "normal"),
        ]
    if d.has_head:
        out += [("final_ln.w", (h,), "gain"), ("final_ln.b", (h,), "normal")]
        if d.pp > 1:
            out += [("lm_head", (d.local_vocab, h), "normal")]
    if d.pp == 1:
        assert len(out) == LAYER_TENSORS * d.layers + EXTRA_TENSORS
    return out


def _numel(shape: Tuple[int, ...]) -> int:
    n = 1
    for s in shape:
        n *= s
    return n


def shard_params(d: ShardDesc) -> int:
    return sum(_numel(s) for _, s, _ in param_list(d))


def shard_bytes(d: ShardDesc) -> int:
    return 2 * shard_params(d)


def forward_flop(d: ShardDesc, batch: int, seq: int) -> int:
    """Multiply-add FLOP (2 per MAC) of the dense contractions of one forward."""
    m = batch * seq
    h, hl, fl = d.hidden, d.local_hidden, d.local_ffn
    per_layer = 2 * m * (3 * hl * h + h * hl + 2 * fl * h)
    attn = 4 * batch * d.local_heads * seq * seq * d.head_dim
    head = 2 * m * h * d.local_vocab if d.has_head else 0
    return d.local_layers * (per_layer + attn) + head


# The five workloads.  `batch`/`seq` are the forward shapes; seeds follow the
# recipe: weights seed = config number (50+k for the serving models), ids 100+n.
CONFIGS: Dict[str, dict] = {
    "opt125m_tp1": dict(desc=ShardDesc(12, 768, 3072, 12), batch=1, seq=8, wseed=1, idseed=101),
    "opt1.3b_tp1": dict(desc=ShardDesc(24, 2048, 8192, 32), batch=8, seq=128, wseed=2, idseed=102),
    "opt6.7b_tp2": dict(desc=ShardDesc(32, 4096, 16384, 32, tp=2, rank=0), batch=4, seq=256, wseed=3, idseed=103),
    "opt13b_tp4": dict(desc=ShardDesc(40, 5120, 20480, 40, tp=4, rank=0), batch=16, seq=128, wseed=4, idseed=104),
    # the paper's hybrid split of OPT-13B (Section 5.1: TP = 2 x PP = 2 on four GPUs): one GPU's share
    "opt13b_tp2_pp2": dict(desc=ShardDesc(40, 5120, 20480, 40, tp=2, rank=0, pp=2, stage=0), batch=16, seq=128,
                           wseed=6, idseed=106),
    # beyond the paper's sizes: one GPU's share of the 66B member of the family split eight ways (16.5 GB)
    "opt66b_tp8": dict(desc=ShardDesc(64, 9216, 36864, 72, tp=8, rank=0), batch=4, seq=256, wseed=7, idseed=107),
    "serve8x6.7b_tp2": dict(desc=ShardDesc(32, 4096, 16384, 32, tp=2, rank=0), batch=1, seq=64,
                            n_models=8, wseed=50, budget=20_000_000_000, n_requests=2000,
                            rate=20.0, cv=4.0, zipf=1.5, trace_seed=500, idseed=1000),
}
