"""CPU oracle: forward pass of one tensor-parallel rank of a pre-LN OPT decoder.

TEST INFRASTRUCTURE ONLY.  Nothing on the product path may import this file;
it shares no code with the HIP library and is deliberately plain and slow.

The paper names the model (OPT, Section 5.1) and says tensor-parallel workers
exchange data through collectives (Section 3.1) but never spells the network
out; what is computed here is the public OPT decoder at the given dimensions,
split Megatron-style, evaluated for ONE rank with the cross-rank all-reduce
("hook") replaced by the identity, so the rank carries its own partial sums:

  x      = tok_r[id - lo] (zero row if id outside [lo, lo + V/t)) + pos[p + 2]
  per layer:
    a    = LN(x; g1, b1)                         biased variance, eps 1e-5
    q,k,v= a Wq^T + bq, ...                      each [M, h/t], heads of size d
    S    = (q d^-1/2) k^T, causal; P = softmax(S); o = P v
    x    = x + hook(o Wo^T) + bo
    u    = relu(LN(x; g2, b2) W1^T + b1)
    x    = x + hook(u W2^T) + b2
  logits = LN(x; gf, bf) tok_r^T                 [b, s, V/t]

All arithmetic is done in `dtype` (float32 by default: the precision the
acceptance tolerance is stated against; float64 is used by the pins) on
parameters up-converted exactly from fp16.  Parity status: the definition is
pinned (index-by-index float64 brute force, the TP-sum and vocabulary-slice
identities, PyTorch CPU ops and an independent OPT implementation used as a
black box, causality / batch-independence invariants).  Agreement with the
*released* OPT checkpoints is "parity unpinned": no checkpoint is available.
"""
from __future__ import annotations

from typing import Callable, Dict, List, Optional, Sequence

import numpy as np

LN_EPS = 1e-5
POS_OFFSET = 2
TENSORS_PER_LAYER = 16
_LAYER_KEYS = ("ln1.w", "ln1.b", "q.w", "q.b", "k.w", "k.b", "v.w", "v.b",
               "o.w", "o.b", "ln2.w", "ln2.b", "fc1.w", "fc1.b", "fc2.w", "fc2.b")


def layer_norm(x: np.ndarray, g: np.ndarray, b: np.ndarray) -> np.ndarray:
    mu = x.mean(axis=-1, keepdims=True)
    xc = x - mu
    var = (xc * xc).mean(axis=-1, keepdims=True)
    return xc / np.sqrt(var + x.dtype.type(LN_EPS)) * g + b


def causal_softmax(scores: np.ndarray) -> np.ndarray:
    """scores [..., s, s]; entries with key index > query index are masked out."""
    s = scores.shape[-1]
    mask = np.triu(np.ones((s, s), dtype=bool), k=1)
    sc = np.where(mask, -np.inf, scores)
    sc = sc - sc.max(axis=-1, keepdims=True)
    e = np.exp(sc)
    return (e / e.sum(axis=-1, keepdims=True)).astype(scores.dtype)


def embed_tokens_only(ids: np.ndarray, tok: np.ndarray, rank: int, dtype) -> np.ndarray:
    """Vocabulary-parallel token lookup (the part the hook would all-reduce).

    ids int [b, s] over the full vocabulary; tok is this rank's [V/t, h] slice.
    """
    b, s = ids.shape
    vl = tok.shape[0]
    local = ids.astype(np.int64) - rank * vl
    inside = (local >= 0) & (local < vl)
    x = np.zeros((b, s, tok.shape[1]), dtype=dtype)
    x[inside] = np.asarray(tok)[local[inside]].astype(dtype)
    return x


def embed(ids: np.ndarray, tok: np.ndarray, pos: np.ndarray, rank: int, dtype,
          hook: Callable[[np.ndarray], np.ndarray] = lambda z: z) -> np.ndarray:
    """Residual stream entering layer 0: hooked token rows plus position rows."""
    s = ids.shape[1]
    x = hook(embed_tokens_only(ids, tok, rank, dtype))
    return x + np.asarray(pos)[POS_OFFSET:POS_OFFSET + s].astype(dtype)[None, :, :]


def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, heads: int) -> np.ndarray:
    """q, k, v [b, s, heads*d] -> [b, s, heads*d]."""
    b, s, hl = q.shape
    d = hl // heads
    split = lambda z: z.reshape(b, s, heads, d).transpose(0, 2, 1, 3)
    qh, kh, vh = split(q) * q.dtype.type(d ** -0.5), split(k), split(v)
    p = causal_softmax(qh @ kh.transpose(0, 1, 3, 2))
    return (p @ vh).transpose(0, 2, 1, 3).reshape(b, s, hl)


def attn_partial(x: np.ndarray, w: Dict[str, np.ndarray], heads: int) -> np.ndarray:
    """This rank's contribution o Wo^T of the attention block (no bias, no residual)."""
    a = layer_norm(x, w["ln1.w"], w["ln1.b"])
    q = a @ w["q.w"].T + w["q.b"]
    k = a @ w["k.w"].T + w["k.b"]
    v = a @ w["v.w"].T + w["v.b"]
    return attention(q, k, v, heads) @ w["o.w"].T


def mlp_partial(x: np.ndarray, w: Dict[str, np.ndarray]) -> np.ndarray:
    """This rank's contribution u W2^T of the feed-forward block (no bias, no residual)."""
    a = layer_norm(x, w["ln2.w"], w["ln2.b"])
    u = np.maximum(a @ w["fc1.w"].T + w["fc1.b"], x.dtype.type(0))
    return u @ w["fc2.w"].T


def decoder_layer(x: np.ndarray, w: Dict[str, np.ndarray], heads: int,
                  hook: Callable[[np.ndarray], np.ndarray]) -> np.ndarray:
    x = x + hook(attn_partial(x, w, heads)) + w["o.b"]
    x = x + hook(mlp_partial(x, w)) + w["fc2.b"]
    return x


def layer_weights(params: Sequence[np.ndarray], layer: int, dtype, first: int = 2) -> Dict[str, np.ndarray]:
    """The 16 tensors of the `layer`-th layer held in `params`, whose layer tensors start at index `first`."""
    base = first + TENSORS_PER_LAYER * layer
    return {k: np.asarray(params[base + i]).astype(dtype) for i, k in enumerate(_LAYER_KEYS)}


def forward(params: Sequence[np.ndarray], ids: np.ndarray, *, layers: int, heads: int,
            tp: int = 1, rank: int = 0, dtype=np.float32,
            hook: Optional[Callable[[np.ndarray], np.ndarray]] = None,
            taps: Optional[List[np.ndarray]] = None) -> np.ndarray:
    """Logits [b, s, V/t] of one rank.  `params` is the canonical 16L+4 list.

    `heads` is the full model's head count; the rank owns heads/tp of them.
    `taps`, if given, receives the residual stream after the embedding and
    after every layer (for per-stage comparisons in tests).
    """
    if len(params) != TENSORS_PER_LAYER * layers + 4:
        raise ValueError("parameter list has the wrong length")
    hook = hook or (lambda z: z)
    local_heads = heads // tp
    x = embed(ids, params[0], params[1], rank, dtype, hook)
    if taps is not None:
        taps.append(x.copy())
    for l in range(layers):
        w = layer_weights(params, l, dtype)   # one layer up-converted at a time
        x = decoder_layer(x, w, local_heads, hook)
        if taps is not None:
            taps.append(x.copy())
    y = layer_norm(x, np.asarray(params[-2]).astype(dtype), np.asarray(params[-1]).astype(dtype))
    return y @ np.asarray(params[0]).astype(dtype).T


def forward_stage(params: Sequence[np.ndarray], inp: np.ndarray, *, layers: int, heads: int,
                  tp: int = 1, rank: int = 0, pp: int = 1, stage: int = 0, dtype=np.float32,
                  hook: Optional[Callable[[np.ndarray], np.ndarray]] = None) -> np.ndarray:
    """One pipeline stage of one rank.

    The paper splits models by tensor *and* pipeline parallelism (Section 5.1:
    swapping gets faster with either).  A pipeline stage owns a contiguous
    range of decoder layers: stage p of `pp` holds layers [p*L/pp, (p+1)*L/pp).
    Stage 0 also holds the embeddings and starts from token ids; the last
    stage also holds the final LayerNorm and its own copy of the (tied) head
    matrix and ends in logits; every other boundary carries the residual
    stream [b, s, h].  `layers` is the whole model's layer count and `params`
    the stage's list: [embed_tokens, embed_positions] if stage 0, 16 tensors
    per local layer, [final_ln.w, final_ln.b] if last, then lm_head if last
    and pp > 1 (with pp == 1 the head is embed_tokens, as in `forward`).
    """
    if layers % pp or not 0 <= stage < pp:
        raise ValueError("layers must divide evenly into stages")
    local = layers // pp
    is_first, is_last = stage == 0, stage == pp - 1
    n_front = 2 if is_first else 0
    n_back = (3 if pp > 1 else 2) if is_last else 0
    if len(params) != n_front + TENSORS_PER_LAYER * local + n_back:
        raise ValueError("parameter list has the wrong length for this stage")
    hook = hook or (lambda z: z)
    if is_first:
        x = embed(inp, params[0], params[1], rank, dtype, hook)
    else:
        x = np.asarray(inp).astype(dtype)
    for l in range(local):
        x = decoder_layer(x, layer_weights(params, l, dtype, first=n_front), heads // tp, hook)
    if not is_last:
        return x
    at = n_front + TENSORS_PER_LAYER * local
    y = layer_norm(x, np.asarray(params[at]).astype(dtype), np.asarray(params[at + 1]).astype(dtype))
    head = params[at + 2] if pp > 1 else params[0]
    return y @ np.asarray(head).astype(dtype).T
