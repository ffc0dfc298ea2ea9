"""The two-lane engine through the C ABI: batches of loaded models go on while another model loads
(Section 3.2 of the paper).  Every request is answered once and correctly, order within a model is
kept, the residency decisions equal the LRU oracle's on the order of dispatch."""
import time

import numpy as np
import pytest

torch = pytest.importorskip("torch")
import paper_2306_13835_amd as P
from oracle import opt_shard as O
from oracle.lru import LruResidency
from oracle.swap import as_bytes
from synth import ShardDesc, shard_bytes, token_ids, gamma_rates_trace
from gpu_util import Rig

pytestmark = pytest.mark.gpu

DESC = ShardDesc(4, 1024, 4096, 8, vocab=8192, max_pos=64)      # ~118 MB: a load takes milliseconds
SEQ, MAXB = 8, 4


def make(n_models, resident, extra_bytes=7, **kw):
    size = shard_bytes(DESC)
    arena = None if kw.get("block_residency") else (resident + 1) * P.arena_bytes(DESC)
    rig = Rig([DESC] * n_models, budget=resident * size + extra_bytes, arena_bytes=arena,
              max_tokens=MAXB * SEQ, mode=P.XFER_AUTO, two_lanes=True, **kw)
    eng = P.Engine(rig.ctx, MAXB, SEQ, two_lanes=True)
    ms = [rig.add(DESC, seed=160 + i) for i in range(n_models)]
    bufs = [torch.empty(MAXB, SEQ, DESC.vocab, dtype=torch.float32, device="cuda") for _ in range(2)]
    return rig, eng, ms, bufs


def check_rows(rig, m, ids_list, got):
    for row, ids in enumerate(ids_list):
        want = O.forward(rig.tensors[m], ids, layers=DESC.layers, heads=DESC.heads)
        assert np.abs(got[row] - want[0]).max() <= 2e-2
        assert np.abs(got[row] - want[0]).mean() / np.abs(want).mean() <= 1e-3


def test_hit_is_dispatched_while_a_miss_is_in_flight():
    rig, eng, ms, bufs = make(3, 2)
    try:
        ids = [token_ids(500 + i, 1, SEQ, DESC.vocab) for i in range(6)]
        # load model 0 through its first request
        eng.submit(ms[0], ids[0], 0.0)
        served, m, miss, lane = eng.dispatch(*bufs)
        assert (served, m, miss, lane) == ([0], 0, True, 1)
        assert eng.dispatch(*bufs) is None                     # nothing else queued
        rig.ctx.sync()
        assert eng.lanes_busy() == (False, False)
        check_rows(rig, 0, [ids[0]], bufs[1].cpu().numpy())
        # a miss on model 1, then a hit on model 0
        eng.submit(ms[1], ids[1], 1.0)
        eng.submit(ms[0], ids[2], 2.0)
        a = eng.dispatch(*bufs)
        b = eng.dispatch(*bufs)
        assert a == ([1], 1, True, 1)                          # oldest head: model 1, not resident -> load lane
        assert b == ([2], 0, False, 0)                         # the hit goes on the other lane at once
        # a second request for model 1: not dispatched while model 1's miss is in flight
        eng.submit(ms[1], ids[3], 3.0)
        c = eng.dispatch(*bufs)
        if c is None:
            assert eng.pending() == 1
            rig.ctx.sync()
            check_rows(rig, 1, [ids[1]], bufs[1].cpu().numpy())
            check_rows(rig, 0, [ids[2]], bufs[0].cpu().numpy())
            c = eng.dispatch(*bufs)
        assert c == ([3], 1, False, 0)                         # model 1 is loaded: its second request is a hit
        rig.ctx.sync()
        check_rows(rig, 1, [ids[3]], bufs[0].cpu().numpy())
        assert eng.pending() == 0
        with pytest.raises(P.CtnError):
            eng.step(bufs[0])                                  # the serial entry point is not for this engine
    finally:
        eng.close()
        rig.close()


@pytest.mark.parametrize("block_residency,ahead", [(False, False), (True, False), (True, True)])
def test_trace_every_request_once_in_order_and_right(block_residency, ahead):
    from paper_2306_13835_amd.serving import serve_engine_async
    from oracle.partial_lru import PartialLruResidency
    from gpu_util import block_bytes
    extra = shard_bytes(DESC) // 2 if block_residency else 7       # per-block residency gets slack to keep prefixes in
    rig, eng, ms, bufs = make(4, 2, extra_bytes=extra, block_residency=block_residency)
    try:
        eng.set_prefetch(ahead, min_count=2, min_share_percent=40)
        orig = [[t.copy() for t in rig.tensors[m]] for m in ms]
        arr, mod = gamma_rates_trace((60, 30, 30, 10), 4.0, 1.5, seed=77)
        n = len(arr)
        assert 60 < n < 600
        ids = [token_ids(600 + i % 5, 1, SEQ, DESC.vocab) for i in range(n)]
        order, checked = [], [0]

        def on_batch(served, m, miss, lane, intact):
            order.append((tuple(served), m, miss, lane))
            if intact and checked[0] < 12:                             # spot-check some batches against the oracle
                rig.ctx.sync()
                check_rows(rig, m, [ids[r] for r in served], bufs[lane].cpu().numpy())
                checked[0] += 1
        lat, batches = serve_engine_async(rig.ctx, eng, ms, arr, mod, lambda i: ids[i], bufs[0], bufs[1], on_batch)
        rig.ctx.sync()
        served = [r for b in order for r in b[0]]
        assert sorted(served) == list(range(n))
        for m in range(4):
            mine = [r for b in order for r in b[0] if b[1] == m]
            assert mine == sorted(mine)
        assert all(1 <= len(b[0]) <= MAXB and all(mod[r] == b[1] for r in b[0]) for b in order)
        assert all(b[3] == 1 for b in order if b[2])            # misses run on the load lane
        if not ahead:
            assert all(b[3] == (1 if b[2] else 0) for b in order)
        assert (lat > 0).all()
        # decisions = LRU on the order in which batches were dispatched (completion order may differ)
        events = rig.ctx.events()
        budget = 2 * shard_bytes(DESC) + extra
        if block_residency:
            ref = PartialLruResidency(budget, [block_bytes(DESC)] * 4)
            for kind, m, victims in events:
                k, mm, _, ev = ref.touch(m)
                assert (k, mm, tuple(v for v, _, _ in ev)) == (kind, m, victims)
            assert rig.ctx.stats()["n_extra_evictions"] == 0
        else:
            ref = LruResidency(budget, [shard_bytes(DESC)] * 4)
            for kind, m, victims in events:
                assert ref.touch(m) == (kind, m, victims)
        if not ahead:          # a load started ahead is a use (and a miss) without a batch
            assert sum(e[0] == "miss" for e in events) == sum(b[2] for b in order)
        assert rig.ctx.stats()["resident_bytes"] <= budget
        for m in ms:
            for t, o in zip(rig.tensors[m], orig[m]):
                assert np.array_equal(as_bytes(t), as_bytes(o))
    finally:
        eng.close()
        rig.close()


def test_needs_library_streams_and_the_right_entry_points():
    size = shard_bytes(DESC)
    rig = Rig([DESC], budget=size, max_tokens=MAXB * SEQ, torch_streams=True, two_lanes=True)
    try:
        with pytest.raises(P.CtnError):
            P.Engine(rig.ctx, MAXB, SEQ, two_lanes=True)       # caller-supplied streams have no second lane
        eng = P.Engine(rig.ctx, MAXB, SEQ)
        with pytest.raises(P.CtnError):
            eng.dispatch(rig.arena, rig.arena)
        eng.close()
    finally:
        rig.close()


def test_model_that_is_loading_ahead_takes_the_load_lane():
    """A model whose load was started ahead of its request and is still arriving must not make the
    batches of loaded models wait: its batch goes to the load lane, and is no miss."""
    rig, eng, ms, bufs = make(3, 2)
    try:
        eng.set_prefetch(True, min_count=1, min_share_percent=50)
        ids = [token_ids(700 + i, 1, SEQ, DESC.vocab) for i in range(8)]

        def serve(model, k):
            eng.submit(ms[model], ids[k], float(k))
            r = eng.dispatch(*bufs)
            assert r is not None and r[1] == model
            rig.ctx.sync()
            check_rows(rig, model, [ids[k]], bufs[r[3]].cpu().numpy())
            return r
        serve(0, 0); serve(1, 1); serve(0, 2)        # teaches 0 -> 1 and 1 -> 0; resident {0, 1}
        serve(2, 3)                                  # evicts 1; resident {0, 2}
        r = serve(0, 4)
        assert r[2] is False and r[3] == 0           # a plain hit
        ahead = eng.idle()                           # nothing queued: model 1 is predicted and starts loading
        assert ahead == ms[1] and rig.ctx.is_resident(ms[1])
        eng.submit(ms[1], ids[5], 5.0)
        eng.submit(ms[0], ids[6], 6.0)
        a = eng.dispatch(*bufs)
        b = eng.dispatch(*bufs)
        assert a[1] == 1 and a[2] is False           # not a miss: the load was already under way
        if a[3] == 1:                                # still arriving: load lane, and model 0 goes ahead on the hit lane
            assert b == ([6], 0, False, 0)
            rig.ctx.sync()
            check_rows(rig, 1, [ids[5]], bufs[1].cpu().numpy())
            check_rows(rig, 0, [ids[6]], bufs[0].cpu().numpy())
        else:                                        # it had landed already: both are hits, one after the other
            rig.ctx.sync()
            check_rows(rig, 1, [ids[5]], bufs[0].cpu().numpy())
            b = b or eng.dispatch(*bufs)
            assert b == ([6], 0, False, 0)
            rig.ctx.sync()
            check_rows(rig, 0, [ids[6]], bufs[0].cpu().numpy())
        print("model loading ahead ran on lane", a[3], flush=True)
        assert rig.ctx.stats()["n_prefetch"] == 1
    finally:
        eng.close()
        rig.close()


def test_many_hits_complete_while_one_miss_is_loading():
    """A batch that waits for its model's load keeps everything it was given (its token ids among them) for the
    whole load; the batches of loaded models that are dispatched meanwhile must not wait for it.  One large model
    (2.6 GB: tens of milliseconds of load) misses on the load lane; twenty hits on a small resident model are then
    dispatched one after the other, each awaited, and all of them must be done while the load lane is still busy."""
    from synth import CONFIGS
    big = CONFIGS["opt1.3b_tp1"]["desc"]
    small = DESC
    rig = Rig([small, big], max_tokens=MAXB * SEQ, mode=P.XFER_KERNEL, two_lanes=True, gap=4096)
    eng = None
    try:
        eng = P.Engine(rig.ctx, MAXB, SEQ, two_lanes=True)
        m_small = rig.add(small, seed=300)
        m_big = rig.add(big, seed=301)
        bufs = [torch.empty(MAXB, SEQ, max(small.vocab, big.vocab), dtype=torch.float32, device="cuda") for _ in range(2)]
        ids = token_ids(700, 1, SEQ, small.vocab)
        eng.submit(m_small, ids, 0.0)
        assert eng.dispatch(*bufs)[1:] == (m_small, True, 1)
        rig.ctx.sync()
        eng.submit(m_big, ids, 1.0)
        t0 = time.perf_counter()
        assert eng.dispatch(*bufs)[1:] == (m_big, True, 1)     # the load lane is busy from here on
        done = 0
        for i in range(20):
            eng.submit(m_small, ids, 2.0 + i)
            r = eng.dispatch(*bufs)
            assert r is not None and r[1:] == (m_small, False, 0), (i, r)
            while eng.lanes_busy()[0]:
                pass
            done += 1
        t_hits = time.perf_counter() - t0
        still_loading = eng.lanes_busy()[1]
        rig.ctx.sync()
        t_all = time.perf_counter() - t0
        print(f"20 hits in {t_hits * 1e3:.1f} ms, the miss took {t_all * 1e3:.1f} ms", flush=True)
        assert done == 20 and still_loading, (t_hits, t_all)
    finally:
        if eng is not None:
            eng.close()
        rig.close()
