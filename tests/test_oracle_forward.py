"""Pins for oracle/opt_shard.py: none of them re-uses the oracle's own formulae."""
import numpy as np
import pytest

from oracle import opt_shard as O
from synth import ShardDesc, fill_shard, token_ids

from bruteforce_opt import forward as brute_forward
from tp_split import split

TINY = dict(layers=2, hidden=16, ffn=64, heads=4, vocab=32, max_pos=16)


def tiny_full(seed=7, sigma_boost=8.0):
    d = ShardDesc(**TINY)
    p = fill_shard(d, seed, threads=1)
    # widen the distribution so softmax / relu / LN are far from degenerate
    out = []
    for i, a in enumerate(p):
        a32 = a.astype(np.float32)
        if a.ndim == 1 and abs(float(a32.mean()) - 1.0) < 0.2:      # a LayerNorm gain
            a32 = 1.0 + (a32 - 1.0) * sigma_boost
        else:
            a32 = a32 * sigma_boost
        out.append(a32.astype(np.float16))
    return d, out


def tolist(params):
    return [p.astype(np.float64).tolist() for p in params]


@pytest.mark.parametrize("t", [1, 2, 4])
def test_bruteforce_every_rank(t):
    d, full = tiny_full()
    ids = token_ids(11, 2, 5, d.vocab)
    for r in range(t):
        shard = split(full, d.layers, t, r)
        want = np.array(brute_forward(tolist(shard), ids.tolist(), d.layers, d.heads, t, r))
        got64 = O.forward(shard, ids, layers=d.layers, heads=d.heads, tp=t, rank=r, dtype=np.float64)
        got32 = O.forward(shard, ids, layers=d.layers, heads=d.heads, tp=t, rank=r, dtype=np.float32)
        assert got64.shape == (2, 5, d.vocab // t)
        assert np.abs(got64 - want).max() < 1e-11
        assert got32.dtype == np.float32
        assert np.abs(got32 - want).max() < 1e-5 * max(1.0, np.abs(want).max())


def test_tp_sum_identity_layer_blocks():
    """Sum over ranks of the partial products + bias equals the unsharded block."""
    d, full = tiny_full(seed=9)
    rng = np.random.default_rng(0)
    x = rng.standard_normal((2, 5, d.hidden))
    for t in (2, 4):
        for l in range(d.layers):
            wf = O.layer_weights(full, l, np.float64)
            attn_full = O.attn_partial(x, wf, d.heads)
            mlp_full = O.mlp_partial(x, wf)
            attn_sum = np.zeros_like(x)
            mlp_sum = np.zeros_like(x)
            for r in range(t):
                ws = O.layer_weights(split(full, d.layers, t, r), l, np.float64)
                attn_sum += O.attn_partial(x, ws, d.heads // t)
                mlp_sum += O.mlp_partial(x, ws)
            assert np.abs(attn_sum - attn_full).max() < 1e-12
            assert np.abs(mlp_sum - mlp_full).max() < 1e-12


def _true_tp_forward(full, ids, d, t):
    """All t ranks in lock step with a real sum at every hook (built from the
    oracle's per-rank blocks); must equal the unsharded model."""
    shards = [split(full, d.layers, t, r) for r in range(t)]
    x = sum(O.embed_tokens_only(ids, shards[r][0], r, np.float64) for r in range(t))
    x = x + full[1][2:2 + ids.shape[1]].astype(np.float64)[None]
    for l in range(d.layers):
        ws = [O.layer_weights(shards[r], l, np.float64) for r in range(t)]
        x = x + sum(O.attn_partial(x, ws[r], d.heads // t) for r in range(t)) + ws[0]["o.b"]
        x = x + sum(O.mlp_partial(x, ws[r]) for r in range(t)) + ws[0]["fc2.b"]
    y = O.layer_norm(x, full[-2].astype(np.float64), full[-1].astype(np.float64))
    return np.concatenate([y @ shards[r][0].astype(np.float64).T for r in range(t)], axis=-1)


@pytest.mark.parametrize("t", [2, 4])
def test_all_ranks_with_real_allreduce_equal_unsharded_model(t):
    d, full = tiny_full(seed=21)
    ids = token_ids(5, 3, 6, d.vocab)
    want = O.forward(full, ids, layers=d.layers, heads=d.heads, dtype=np.float64)
    got = _true_tp_forward(full, ids, d, t)
    assert np.abs(got - want).max() < 1e-11


def test_vocab_slice_identity():
    d, full = tiny_full(seed=3)
    ids = token_ids(8, 2, 7, d.vocab)
    whole = O.embed_tokens_only(ids, full[0], 0, np.float64)
    for t in (2, 4):
        parts = [O.embed_tokens_only(ids, split(full, d.layers, t, r)[0], r, np.float64) for r in range(t)]
        assert np.array_equal(sum(parts), whole)
        # exactly one rank contributes each token row
        nz = sum((np.abs(p).sum(-1) > 0).astype(int) for p in parts)
        assert nz.max() <= 1


def test_against_torch_cpu_ops():
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    d, full = tiny_full(seed=5)
    rng = np.random.default_rng(1)
    x = rng.standard_normal((2, 6, d.hidden))
    w = O.layer_weights(full, 1, np.float64)
    tx = torch.from_numpy(x)
    tw = {k: torch.from_numpy(v) for k, v in w.items()}
    # LayerNorm
    want = F.layer_norm(tx, (d.hidden,), tw["ln1.w"], tw["ln1.b"], eps=1e-5).numpy()
    assert np.abs(O.layer_norm(x, w["ln1.w"], w["ln1.b"]) - want).max() < 1e-12
    # causal softmax
    sc = rng.standard_normal((2, 4, 6, 6))
    mask = torch.triu(torch.full((6, 6), float("-inf"), dtype=torch.float64), diagonal=1)
    want = torch.softmax(torch.from_numpy(sc) + mask, dim=-1).numpy()
    assert np.abs(O.causal_softmax(sc) - want).max() < 1e-14
    # attention block through torch's fused SDPA (default scale = d^-1/2)
    a = F.layer_norm(tx, (d.hidden,), tw["ln1.w"], tw["ln1.b"], eps=1e-5)
    heads = lambda z: z.view(2, 6, d.heads, d.head_dim).transpose(1, 2)
    q, k, v = (heads(F.linear(a, tw[n + ".w"], tw[n + ".b"])) for n in "qkv")
    o = F.scaled_dot_product_attention(q, k, v, is_causal=True).transpose(1, 2).reshape(2, 6, d.hidden)
    want = F.linear(o, tw["o.w"]).numpy()
    assert np.abs(O.attn_partial(x, w, d.heads) - want).max() < 1e-12
    # MLP block
    a2 = F.layer_norm(tx, (d.hidden,), tw["ln2.w"], tw["ln2.b"], eps=1e-5)
    want = F.linear(F.relu(F.linear(a2, tw["fc1.w"], tw["fc1.b"])), tw["fc2.w"]).numpy()
    assert np.abs(O.mlp_partial(x, w) - want).max() < 1e-12


def test_against_independent_opt_implementation_black_box():
    """t = 1: an independent OPT implementation (library class built from a
    config, random weights replaced by ours) must give the same logits."""
    torch = pytest.importorskip("torch")
    tr = pytest.importorskip("transformers")
    d, full = tiny_full(seed=13)
    cfg = tr.OPTConfig(vocab_size=d.vocab, hidden_size=d.hidden, ffn_dim=d.ffn,
                       num_hidden_layers=d.layers, num_attention_heads=d.heads,
                       max_position_embeddings=d.max_pos, word_embed_proj_dim=d.hidden,
                       do_layer_norm_before=True, dropout=0.0, attention_dropout=0.0,
                       activation_function="relu", pad_token_id=None)
    try:
        cfg._attn_implementation = "eager"
    except Exception:
        pass
    m = tr.OPTForCausalLM(cfg).double().eval()
    dec = m.model.decoder
    T = lambda a: torch.from_numpy(a.astype(np.float64))
    with torch.no_grad():
        dec.embed_tokens.weight.copy_(T(full[0]))
        dec.embed_positions.weight.copy_(T(full[1]))
        dec.final_layer_norm.weight.copy_(T(full[-2]))
        dec.final_layer_norm.bias.copy_(T(full[-1]))
        for l, layer in enumerate(dec.layers):
            w = O.layer_weights(full, l, np.float64)
            at = layer.self_attn
            for mod, n in ((at.q_proj, "q"), (at.k_proj, "k"), (at.v_proj, "v"), (at.out_proj, "o"),
                           (layer.fc1, "fc1"), (layer.fc2, "fc2")):
                mod.weight.copy_(T(w[n + ".w"]))
                mod.bias.copy_(T(w[n + ".b"]))
            layer.self_attn_layer_norm.weight.copy_(T(w["ln1.w"]))
            layer.self_attn_layer_norm.bias.copy_(T(w["ln1.b"]))
            layer.final_layer_norm.weight.copy_(T(w["ln2.w"]))
            layer.final_layer_norm.bias.copy_(T(w["ln2.b"]))
    assert m.lm_head.weight.data_ptr() == dec.embed_tokens.weight.data_ptr()  # tied head
    ids = token_ids(17, 3, 9, d.vocab)
    with torch.no_grad():
        want = m(torch.from_numpy(ids.astype(np.int64))).logits.numpy()
    got = O.forward(full, ids, layers=d.layers, heads=d.heads, dtype=np.float64)
    # the library evaluates its softmax in float32 whatever the module dtype,
    # which limits agreement to ~1e-7; a wrong term or index is off by >1e-2
    assert np.abs(got - want).max() < 2e-6


def test_invariants_causality_batch_independence_softmax_ln():
    d, full = tiny_full(seed=2)
    ids = token_ids(4, 3, 8, d.vocab)
    base = O.forward(full, ids, layers=d.layers, heads=d.heads)
    # causality: changing token j leaves earlier positions bit-identical
    ids2 = ids.copy()
    ids2[:, 5] = (ids2[:, 5] + 1) % d.vocab
    alt = O.forward(full, ids2, layers=d.layers, heads=d.heads)
    assert np.array_equal(alt[:, :5], base[:, :5])
    assert not np.array_equal(alt[:, 5:], base[:, 5:])
    # batch rows do not interact
    solo = O.forward(full, ids[1:2], layers=d.layers, heads=d.heads)
    assert np.abs(solo[0] - base[1]).max() < 1e-5
    # softmax rows sum to one, masked entries are zero
    rng = np.random.default_rng(0)
    p = O.causal_softmax(rng.standard_normal((2, 3, 7, 7)))
    assert np.abs(p.sum(-1) - 1).max() < 1e-14
    assert np.all(np.triu(p, k=1) == 0)
    # LayerNorm with unit gain, zero bias: zero mean, unit variance
    x = rng.standard_normal((5, 64)) * 3 + 2
    y = O.layer_norm(x, np.ones(64), np.zeros(64))
    assert np.abs(y.mean(-1)).max() < 1e-12
    assert np.abs(y.var(-1) - 1).max() < 1e-4


def test_out_of_range_ids_use_zero_token_row():
    d, full = tiny_full(seed=6)
    shard = split(full, d.layers, 2, 1)      # owns ids [16, 32)
    ids = np.array([[3, 20, 15, 16]], dtype=np.int32)
    x = O.embed(ids, shard[0], shard[1], 1, np.float64)
    pos = shard[1].astype(np.float64)
    assert np.array_equal(x[0, 0], pos[2])
    assert np.array_equal(x[0, 2], pos[4])
    assert np.array_equal(x[0, 1], full[0][20].astype(np.float64) + pos[3])
    assert np.array_equal(x[0, 3], full[0][16].astype(np.float64) + pos[5])


def _tiny4(seed=13):
    d = ShardDesc(layers=4, hidden=16, ffn=64, heads=4, vocab=32, max_pos=16)
    p = fill_shard(d, seed, threads=1)
    return d, [(a.astype(np.float32) * 8.0 if not (a.ndim == 1 and abs(float(a.astype(np.float32).mean()) - 1.0) < 0.2)
                else 1.0 + (a.astype(np.float32) - 1.0) * 8.0).astype(np.float16) for a in p]


@pytest.mark.parametrize("t", [1, 2])
@pytest.mark.parametrize("pp", [1, 2, 4])
def test_pipeline_stages_chain_to_the_brute_force_model(pp, t):
    """Stage after stage, fed with the previous stage's residual stream, must end in the logits the
    index-by-index brute force computes for the whole rank; every boundary equals the residual
    stream the whole-model oracle records after that layer."""
    from pp_split import stage_params
    d, full = _tiny4()
    ids = token_ids(17, 2, 5, d.vocab)
    for r in range(t):
        shard = split(full, d.layers, t, r)
        want = np.array(brute_forward(tolist(shard), ids.tolist(), d.layers, d.heads, t, r))
        taps = []
        O.forward(shard, ids, layers=d.layers, heads=d.heads, tp=t, rank=r, dtype=np.float64, taps=taps)
        x = ids
        for stage in range(pp):
            sp = stage_params(shard, d.layers, pp, stage)
            x = O.forward_stage(sp, x, layers=d.layers, heads=d.heads, tp=t, rank=r, pp=pp, stage=stage,
                                dtype=np.float64)
            if stage < pp - 1:
                assert x.shape == (2, 5, d.hidden)
                assert np.array_equal(x, taps[(stage + 1) * d.layers // pp])
        assert x.shape == (2, 5, d.vocab // t)
        assert np.abs(x - want).max() < 1e-11


def test_pipeline_stage_argument_checks():
    from pp_split import stage_params
    d, full = _tiny4()
    ids = token_ids(17, 1, 3, d.vocab)
    with pytest.raises(ValueError):
        O.forward_stage(full, ids, layers=4, heads=4, pp=3, stage=0)                 # 4 layers, 3 stages
    with pytest.raises(ValueError):
        O.forward_stage(stage_params(full, 4, 2, 0), ids, layers=4, heads=4, pp=2, stage=1)   # wrong list
    # a wrong head matrix or a skipped embedding must show: the last stage uses its own copy
    sp = stage_params(full, 4, 2, 1)
    x = np.random.default_rng(1).standard_normal((1, 3, d.hidden))
    a = O.forward_stage(sp, x, layers=4, heads=4, pp=2, stage=1, dtype=np.float64)
    sp[-1] = sp[-1] * 2
    b = O.forward_stage(sp, x, layers=4, heads=4, pp=2, stage=1, dtype=np.float64)
    assert np.allclose(b, 2 * a)
