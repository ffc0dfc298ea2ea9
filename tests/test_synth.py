"""Shapes, byte counts and generators of the synthetic workloads."""
import numpy as np
import pytest

from synth import CONFIGS, ShardDesc, fill_shard, param_list, shard_bytes, shard_params, token_ids, forward_flop
from synth.arrivals import gamma_rates_trace, gamma_zipf_trace, zipf_popularity
from golden_values import load as golden


def test_opt13b_footprint_matches_paper():
    g = golden()
    full = ShardDesc(40, 5120, 20480, 40)
    gib = shard_bytes(full) / 2**30
    assert abs(gib - g["opt13b_fp16_footprint_gb"]) < 0.5          # "about 24 GB"
    assert abs(gib / g["link_bandwidth_gbps"] - g["swap_lower_bound_s"]) < 0.02


@pytest.mark.parametrize("name,params,tensors", [
    ("opt125m_tp1", 125_239_296, 196),
    ("opt1.3b_tp1", 1_315_758_080, 388),
    ("opt6.7b_tp2", 3_333_832_704, 516),
    ("opt13b_tp4", 3_222_169_600, 644),
])
def test_shard_sizes(name, params, tensors):
    d = CONFIGS[name]["desc"]
    assert shard_params(d) == params
    assert len(param_list(d)) == tensors
    # closed form: L[(4h^2+2hf+3h+f)/t + 6h] + (V/t)h + P h + 2h
    L, h, f, t = d.layers, d.hidden, d.ffn, d.tp
    assert params == L * ((4 * h * h + 2 * h * f + 3 * h + f) // t + 6 * h) + d.vocab // t * h + 2050 * h + 2 * h


def test_ranks_of_a_model_partition_the_sharded_tensors():
    d1 = ShardDesc(4, 64, 256, 8)
    for t in (2, 4):
        dt = ShardDesc(4, 64, 256, 8, tp=t, rank=1)
        for (n1, s1, _), (nt, st, _) in zip(param_list(d1), param_list(dt)):
            assert n1 == nt
            ratio = np.prod(s1) / np.prod(st)
            assert ratio in (1, t)


def test_budget_admits_two_serving_models_not_three():
    c = CONFIGS["serve8x6.7b_tp2"]
    b = shard_bytes(c["desc"])
    assert b == 6_667_665_408
    assert 2 * b <= c["budget"] < 3 * b


def test_fill_is_deterministic_order_free_and_distributed_as_stated():
    d = ShardDesc(2, 64, 256, 8, vocab=512, max_pos=30)
    a = fill_shard(d, 42, threads=1)
    b = fill_shard(d, 42, threads=4)
    c = fill_shard(d, 43, threads=4)
    assert all(np.array_equal(x.view(np.uint16), y.view(np.uint16)) for x, y in zip(a, b))
    assert not np.array_equal(a[0], c[0])
    specs = param_list(d)
    big = a[0].astype(np.float64)
    assert abs(big.mean()) < 1e-3 and abs(big.std() - 0.02) < 1e-3
    for t, (_, shape, kind) in zip(a, specs):
        assert t.dtype == np.float16 and t.shape == shape
        if kind == "gain":
            assert abs(float(t.astype(np.float64).mean()) - 1.0) < 0.02
    # caller-provided memory is filled in place
    pool = np.zeros(shard_params(d), dtype=np.float16)
    off = [0]

    def alloc(shape):
        n = int(np.prod(shape))
        v = pool[off[0]:off[0] + n].reshape(shape)
        off[0] += n
        return v

    e = fill_shard(d, 42, alloc=alloc)
    assert np.array_equal(np.concatenate([x.reshape(-1) for x in a]).view(np.uint16), pool.view(np.uint16))
    assert e[0].base is not None


def test_token_ids_cover_full_vocab():
    ids = token_ids(103, 4, 256, 50272)
    assert ids.shape == (4, 256) and ids.dtype == np.int32
    assert ids.min() >= 0 and ids.max() < 50272 and ids.max() > 25136
    assert np.array_equal(ids, token_ids(103, 4, 256, 50272))


def test_forward_flop_matches_closed_form_figures():
    assert abs(forward_flop(CONFIGS["opt6.7b_tp2"]["desc"], 4, 256) / 6.88e12 - 1) < 0.02
    assert abs(forward_flop(CONFIGS["opt13b_tp4"]["desc"], 16, 128) / 13.2e12 - 1) < 0.02
    assert abs(forward_flop(CONFIGS["opt1.3b_tp1"]["desc"], 8, 128) / 2.71e12 - 1) < 0.02


def test_gamma_traces_have_requested_rate_and_burstiness():
    t, m = gamma_rates_trace([10, 1, 1], cv=1.0, duration=2000.0, seed=3)
    assert np.all(np.diff(t) >= 0)
    counts = np.bincount(m, minlength=3) / 2000.0
    assert abs(counts[0] - 10) < 0.5 and abs(counts[1] - 1) < 0.15
    for cv in (0.25, 4.0):
        t, m = gamma_rates_trace([5.0], cv=cv, duration=20000.0, seed=4)
        gaps = np.diff(t)
        assert abs(gaps.std() / gaps.mean() / cv - 1) < 0.15
    p = zipf_popularity(8, 1.5)
    assert abs(p[0] - 0.519) < 2e-3 and abs(p[7] - 0.023) < 1e-3
    t, m = gamma_zipf_trace(8, 20.0, 4.0, 1.5, 2000, seed=500)
    assert t.size == 2000 and m.size == 2000 and m.max() < 8
    t2, m2 = gamma_zipf_trace(8, 20.0, 4.0, 1.5, 2000, seed=500)
    assert np.array_equal(t, t2) and np.array_equal(m, m2)
