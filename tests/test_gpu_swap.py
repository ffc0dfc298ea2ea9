"""Swap-in / swap-out through the C ABI: byte identity, residency policy, error paths."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
import paper_2306_13835_amd as P
from oracle.lru import LruResidency
from oracle.swap import DeviceImage, as_bytes
from synth import ShardDesc, shard_bytes, param_list, CONFIGS
from gpu_util import Rig

pytestmark = pytest.mark.gpu

SMALL = ShardDesc(3, 256, 1024, 4, vocab=1000, max_pos=62)            # ~5.6 MB, biases of 512 B
SMALL_TP = ShardDesc(2, 640, 2560, 10, vocab=1000, max_pos=30, tp=2, rank=1)   # odd sizes: 640 B, 2560 B biases


def check_device_copy(rig, m, desc):
    """Every tensor read back from the arena equals the oracle's device image."""
    img = DeviceImage([t.nbytes for t in rig.tensors[m]])
    img.swap_in(rig.tensors[m])
    for i in range(len(rig.tensors[m])):
        got = rig.ctx.debug_read_param(m, i)
        assert np.array_equal(as_bytes(got), img.tensors[i]), f"tensor {i}"


@pytest.mark.parametrize("gap", [0, 48, 4096])      # packed slab / tensors 48 B apart / separate regions
@pytest.mark.parametrize("mode", [P.XFER_KERNEL, P.XFER_DMA, P.XFER_AUTO])
@pytest.mark.parametrize("desc", [SMALL, SMALL_TP])
def test_round_trip_scribble_and_poison(mode, desc, gap):
    rig = Rig([desc], mode=mode, gap=gap)
    try:
        m = rig.add(desc, seed=5)
        orig = [t.copy() for t in rig.tensors[m]]
        rig.arena.fill_(0x7E)                         # fp16 NaN pattern everywhere
        torch.cuda.synchronize()
        rig.ctx.swap_in(m)
        rig.ctx.wait(m)
        assert rig.ctx.is_resident(m)
        check_device_copy(rig, m, desc)
        for t in rig.tensors[m]:                      # scribble: swap-out must really copy back
            as_bytes(t)[:] = 0xA5
        rig.ctx.swap_out(m)
        rig.ctx.wait(m)
        assert not rig.ctx.is_resident(m)
        for t, o in zip(rig.tensors[m], orig):
            assert np.array_equal(as_bytes(t), as_bytes(o))
        if gap:   # nothing may be written between the tensors
            used = np.zeros(rig.pool.nbytes, dtype=bool)
            for t in rig.tensors[m]:
                off = t.ctypes.data - rig.pool.ptr
                used[off:off + t.nbytes] = True
            assert not rig.pool.bytes[~used].any()
        st = rig.ctx.stats()
        assert st["bytes_h2d"] == st["bytes_d2h"] == shard_bytes(desc)
        assert st["resident_bytes"] == 0 and st["peak_resident_bytes"] == shard_bytes(desc)
        in_ms, out_ms, blocks = rig.ctx.last_swap_ms(m)
        assert in_ms > 0 and out_ms > 0 and len(blocks) == desc.layers + 1
        assert all(b2 >= b1 for b1, b2 in zip(blocks, blocks[1:]))
    finally:
        rig.close()


@pytest.mark.parametrize("waves_out", [0, 1, 6, 10, 12])       # workgroups of 256, 64, 128, 128 and 256 threads
@pytest.mark.parametrize("mode", [P.XFER_KERNEL, P.XFER_DMA_IN_KERNEL_OUT, P.XFER_KERNEL_IN_DMA_OUT, P.XFER_DMA_RUNS])
def test_round_trip_every_path_and_offload_width(mode, waves_out):
    """The copy kernel in one direction and the DMA engines in the other, and every workgroup size the
    offload's kernel comes in: device copy equal to the oracle's image, host bytes restored after an overwrite,
    nothing written between the tensors."""
    desc = SMALL_TP
    rig = Rig([desc], mode=mode, gap=48)
    try:
        rig.ctx.set_copy_width(0, waves_out)
        m = rig.add(desc, seed=6)
        orig = [t.copy() for t in rig.tensors[m]]
        for cycle in range(2):
            rig.arena.fill_(0x7E)
            torch.cuda.synchronize()
            rig.ctx.swap_in(m)
            rig.ctx.wait(m)
            check_device_copy(rig, m, desc)
            for t in rig.tensors[m]:
                as_bytes(t)[:] = 0x5A
            rig.ctx.swap_out(m)
            rig.ctx.wait(m)
            for t, o in zip(rig.tensors[m], orig):
                assert np.array_equal(as_bytes(t), as_bytes(o))
        used = np.zeros(rig.pool.nbytes, dtype=bool)
        for t in rig.tensors[m]:
            off = t.ctypes.data - rig.pool.ptr
            used[off:off + t.nbytes] = True
        assert not rig.pool.bytes[~used].any()
    finally:
        rig.close()


def test_auto_offloads_beside_a_load_restore_every_byte():
    """Transfer mode AUTO with a host list in separate pieces: a miss that evicts loads through the DMA engines
    while the victim's offload goes through the copy kernel, its blocks alternating between two widths.  Two
    models, room for one, requests alternating: after every swap the evicted model's host bytes (overwritten
    while it was on the device) are back and the loaded model's device copy equals the oracle's image."""
    desc = SMALL
    size = shard_bytes(desc)
    rig = Rig([desc] * 2, budget=size, arena_bytes=2 * P.arena_bytes(desc), mode=P.XFER_AUTO, gap=4096)
    try:
        ms = [rig.add(desc, seed=70 + i) for i in range(2)]
        orig = [[t.copy() for t in rig.tensors[m]] for m in ms]
        rig.ctx.swap_in(ms[0]); rig.ctx.wait(ms[0])
        for step in range(6):
            cur, nxt = ms[step % 2], ms[(step + 1) % 2]
            for t in rig.tensors[cur]:
                as_bytes(t)[:] = 0xC3                      # the copy on the device is the only good one now
            rig.ctx.swap_in(nxt)                           # evicts cur
            rig.ctx.wait(nxt); rig.ctx.wait(cur)
            assert rig.ctx.is_resident(nxt) and not rig.ctx.is_resident(cur)
            for t, o in zip(rig.tensors[cur], orig[cur]):
                assert np.array_equal(as_bytes(t), as_bytes(o))
            check_device_copy(rig, nxt, desc)
        assert rig.ctx.stats()["n_swap_out"] == 6
    finally:
        rig.close()


def test_dma_and_kernel_paths_leave_identical_arenas():
    rig = Rig([SMALL])
    try:
        m = rig.add(SMALL, seed=9)
        images = []
        for mode in (P.XFER_KERNEL, P.XFER_DMA):
            rig.ctx.set_mode(mode, True)
            rig.arena.zero_()
            torch.cuda.synchronize()
            rig.ctx.swap_in(m)
            rig.ctx.wait(m)
            images.append(rig.arena.cpu().numpy().copy())
            rig.ctx.swap_out(m)
            rig.ctx.wait(m)
        assert np.array_equal(images[0], images[1])
    finally:
        rig.close()


@pytest.mark.parametrize("gap", [0, 4096])
def test_many_cycles_any_order_keeps_host_bits(gap):
    descs = [SMALL, SMALL_TP, SMALL]
    rig = Rig(descs, budget=shard_bytes(SMALL) + shard_bytes(SMALL_TP) + 100, gap=gap)
    try:
        ms = [rig.add(d, seed=20 + i) for i, d in enumerate(descs)]
        orig = [[t.copy() for t in rig.tensors[m]] for m in ms]
        rng = np.random.default_rng(0)
        for step in range(40):
            m = int(rng.integers(0, 3))
            if rng.random() < 0.3:
                rig.ctx.swap_out(m)
            else:
                rig.ctx.set_mode(int(rng.integers(0, 6)), True)          # any of the six transfer modes
                rig.ctx.swap_in(m)
                if rng.random() < 0.5:
                    rig.ctx.wait(m)
                    check_device_copy(rig, m, descs[m])
            st = rig.ctx.stats()
            assert st["resident_bytes"] <= st["budget_bytes"]
        rig.ctx.sync()
        for m in ms:
            for t, o in zip(rig.tensors[m], orig[m]):
                assert np.array_equal(as_bytes(t), as_bytes(o))
        assert rig.ctx.stats()["peak_resident_bytes"] <= rig.ctx.stats()["budget_bytes"]
    finally:
        rig.close()


def test_event_log_equals_oracle_lru():
    descs = [SMALL] * 5
    size = shard_bytes(SMALL)
    rig = Rig(descs, budget=2 * size + 10, arena_bytes=2 * P.arena_bytes(SMALL))
    try:
        ms = [rig.add(d, seed=30 + i) for i, d in enumerate(descs)]
        ref = LruResidency(2 * size + 10, [size] * 5)
        rng = np.random.default_rng(3)
        for step in range(60):
            m = int(rng.integers(0, 5))
            if rng.random() < 0.15:
                rig.ctx.swap_out(m)
                ref.swap_out(m)
            else:
                rig.ctx.swap_in(m)
                ref.touch(m)
            assert [rig.ctx.is_resident(k) for k in ms] == [ref.is_resident(k) for k in ms]
        rig.ctx.sync()
        assert rig.ctx.events() == ref.events
        st = rig.ctx.stats()
        assert st["n_hit"] == sum(e[0] == "hit" for e in ref.events)
        assert st["n_miss"] == sum(e[0] == "miss" for e in ref.events)
        assert st["peak_resident_bytes"] == ref.peak_resident
    finally:
        rig.close()


def test_register_errors_and_idempotence():
    rig = Rig([SMALL], budget=shard_bytes(SMALL))
    try:
        m = rig.add(SMALL, seed=1)
        t = rig.tensors[m]
        # pageable memory is not device accessible
        with pytest.raises(P.CtnError) as e:
            rig.ctx.register_model(SMALL, [np.array(x) for x in t])
        assert e.value.code == -1
        # wrong tensor count / wrong shape / wrong budget
        with pytest.raises(P.CtnError):
            rig.ctx.register_model(SMALL, t[:-1])
        bad = list(t)
        bad[4], bad[5] = t[5], t[4]
        with pytest.raises(P.CtnError):
            rig.ctx.register_model(SMALL, bad)
        with pytest.raises(P.CtnError):
            rig.ctx.register_model(SMALL, t, budget=123)
        # a shard larger than the budget
        big = ShardDesc(4, 256, 1024, 4, vocab=1000, max_pos=62)
        with pytest.raises(P.CtnError) as e:
            rig.ctx.register_model(big, t[:-2] + t[2:18] + t[-2:])
        assert e.value.code == -2
        # unknown handle; idempotent swaps
        with pytest.raises(P.CtnError) as e:
            rig.ctx.swap_in(7)
        assert e.value.code == -3
        rig.ctx.swap_out(m)                                   # not resident: no-op
        rig.ctx.swap_in(m); rig.ctx.swap_in(m)
        rig.ctx.wait(m)
        assert rig.ctx.stats()["n_swap_in"] == 1 and rig.ctx.stats()["n_hit"] == 1
    finally:
        rig.close()


def test_serving_loop_decisions_equal_oracle_and_results_are_deterministic():
    """The serving loop on small shards: the residency decisions taken on the GPU path equal the
    oracle's on the same request order; repeating a (model, ids) pair gives identical logits."""
    from paper_2306_13835_amd.serving import serve_trace
    from synth import gamma_zipf_trace, token_ids
    desc = ShardDesc(2, 256, 1024, 4, vocab=1000, max_pos=64)
    size, n = shard_bytes(desc), 6
    rig = Rig([desc] * n, budget=2 * size + 5, arena_bytes=3 * P.arena_bytes(desc), max_tokens=16, mode=P.XFER_AUTO)
    try:
        ms = [rig.add(desc, seed=70 + i) for i in range(n)]
        arr, mod = gamma_zipf_trace(n, 400.0, 4.0, 1.5, 150, seed=9)
        ids = [token_ids(1000 + (i % 7), 1, 16, desc.vocab) for i in range(150)]
        out = torch.empty(1, 16, desc.vocab, dtype=torch.float32, device="cuda")
        seen = {}
        def check(i):
            key = (int(mod[i]), i % 7)
            got = out.cpu().numpy().copy()
            if key in seen:
                assert np.array_equal(seen[key], got)
            seen[key] = got
        lat, svc, miss = serve_trace(rig.ctx, ms, arr, mod, lambda i: ids[i], out, progress=check)
        rig.ctx.sync()
        ref = LruResidency(2 * size + 5, [size] * n)
        for m in mod:
            ref.touch(int(m))
        assert rig.ctx.events() == ref.events
        assert [bool(x) for x in miss] == [e[0] == "miss" for e in ref.events]
        assert (lat >= svc - 1e-6).all() and rig.ctx.stats()["peak_resident_bytes"] <= 2 * size + 5
    finally:
        rig.close()


def test_engine_batches_rows_match_oracle_forward():
    """Requests queued for three models, batches of up to 4: every request's logits row equals the
    oracle's forward of that request alone; batches are single-model, oldest head first."""
    from oracle import opt_shard as O
    from synth import token_ids
    desc = ShardDesc(2, 256, 1024, 4, vocab=1000, max_pos=64)
    size = shard_bytes(desc)
    rig = Rig([desc] * 3, budget=2 * size, arena_bytes=3 * P.arena_bytes(desc), max_tokens=4 * 8, mode=P.XFER_AUTO)
    eng = P.Engine(rig.ctx, max_batch=4, seq=8)
    try:
        ms = [rig.add(desc, seed=80 + i) for i in range(3)]
        which = [0, 1, 0, 0, 2, 0, 0, 1, 0, 2, 2]
        ids = [token_ids(300 + i, 1, 8, desc.vocab) for i in range(len(which))]
        for i, w in enumerate(which):
            assert eng.submit(ms[w], ids[i], timestamp=float(i)) == i
        assert eng.pending() == len(which)
        out = torch.empty(4, 8, desc.vocab, dtype=torch.float32, device="cuda")
        order = []
        while True:
            r = eng.step(out)
            if r is None:
                break
            rig.ctx.stream_compute.synchronize()
            served, m, miss = r
            order.append((tuple(served), m))
            got = out.cpu().numpy()
            for row, rid in enumerate(served):
                want = O.forward(rig.tensors[m], ids[rid], layers=desc.layers, heads=desc.heads)
                assert np.abs(got[row] - want[0]).max() <= 2e-2
                assert np.abs(got[row] - want[0]).mean() / np.abs(want).mean() <= 1e-3
        assert order == [((0, 2, 3, 5), 0), ((1, 7), 1), ((4, 9, 10), 2), ((6, 8), 0)]
        assert eng.pending() == 0
        with pytest.raises(P.CtnError):
            eng.submit(9, ids[0], 0.0)
    finally:
        eng.close()
        rig.close()


def test_engine_loads_ahead_on_a_cyclic_stream():
    """Three models requested in a fixed order with room for two: LRU alone misses every time; with
    loading ahead the engine, once it has seen the cycle twice, has the next model on its way in
    before the request comes.  Predictions equal the oracle's, logits stay right, bytes survive."""
    from oracle import opt_shard as O
    from oracle.prefetch import TransitionPredictor
    from synth import token_ids
    desc = ShardDesc(2, 256, 1024, 4, vocab=1000, max_pos=64)
    size = shard_bytes(desc)
    rig = Rig([desc] * 3, budget=2 * size, arena_bytes=3 * P.arena_bytes(desc), max_tokens=8, mode=P.XFER_AUTO)
    eng = P.Engine(rig.ctx, max_batch=1, seq=8)
    try:
        ms = [rig.add(desc, seed=110 + i) for i in range(3)]
        orig = [[t.copy() for t in rig.tensors[m]] for m in ms]
        ids = [token_ids(400 + i, 1, 8, desc.vocab) for i in range(3)]
        want = [O.forward(rig.tensors[m], ids[m], layers=desc.layers, heads=desc.heads) for m in ms]
        out = torch.empty(1, 8, desc.vocab, dtype=torch.float32, device="cuda")
        assert eng.idle() is None                       # off by default
        eng.set_prefetch(True, min_count=2, min_share_percent=50)
        ref = TransitionPredictor(3, 2, 50)
        misses, loaded_ahead = [], []
        for i in range(15):
            m = i % 3
            eng.submit(ms[m], ids[m], float(i))
            served, model, miss = eng.step(out)
            rig.ctx.stream_compute.synchronize()
            assert model == m and served == [i]
            got = out.cpu().numpy()
            assert np.abs(got - want[m]).max() <= 2e-2
            ref.observe(m)
            misses.append(miss)
            p = eng.idle()                              # nothing queued: the prediction may be loaded
            expect = ref.predict()
            if expect is not None and not rig.ctx.is_resident(expect) and p is None:
                raise AssertionError("a confident prediction of a non-resident model was not loaded")
            if p is not None:
                assert p == expect
                rig.ctx.wait(p)
            loaded_ahead.append(p)
        # the cycle's three transitions have each been seen twice after 7 dispatches
        assert misses[:7] == [True] * 7 and misses[7:] == [False] * 8
        assert loaded_ahead[6:14] == [(i + 1) % 3 for i in range(6, 14)]
        assert rig.ctx.stats()["n_prefetch"] == sum(p is not None for p in loaded_ahead)
        eng.submit(ms[0], ids[0], 99.0)
        assert eng.idle() is None                       # a request is queued: no speculation
        eng.step(out)
        rig.ctx.sync()
        for m in ms:
            for t, o in zip(rig.tensors[m], orig[m]):
                assert np.array_equal(as_bytes(t), as_bytes(o))
    finally:
        eng.close()
        rig.close()


def test_eviction_without_the_copy_back_is_opt_in_and_moves_nothing():
    """discard_on_evict: eviction frees the device copy only.  The host tensors are neither written nor
    needed to be; the default (off) is pinned by the overwrite tests above."""
    from oracle import opt_shard as O
    from synth import token_ids
    desc = ShardDesc(2, 256, 1024, 4, vocab=1000, max_pos=64)
    size = shard_bytes(desc)
    rig = Rig([desc] * 3, budget=2 * size, arena_bytes=3 * P.arena_bytes(desc), max_tokens=16, mode=P.XFER_AUTO)
    try:
        ms = [rig.add(desc, seed=180 + i) for i in range(3)]
        orig = [[t.copy() for t in rig.tensors[m]] for m in ms]
        rig.ctx.set_discard(True)
        rig.ctx.swap_in(ms[0]); rig.ctx.wait(ms[0])
        marker = rig.tensors[ms[0]][4].copy()
        rig.tensors[ms[0]][4][...] = 0                  # what the host holds now is what a reload must bring
        rig.ctx.swap_out(ms[0]); rig.ctx.wait(ms[0])
        assert not rig.tensors[ms[0]][4].any()          # nothing was copied back
        assert rig.ctx.stats()["bytes_d2h"] == 0 and not rig.ctx.is_resident(ms[0])
        rig.ctx.swap_in(ms[0]); rig.ctx.wait(ms[0])
        assert not rig.ctx.debug_read_param(ms[0], 4).any()
        rig.tensors[ms[0]][4][...] = marker
        rig.ctx.swap_out(ms[0]); rig.ctx.sync()
        ids = [token_ids(185 + i, 2, 8, desc.vocab) for i in range(3)]
        want = [O.forward(rig.tensors[m], ids[m], layers=desc.layers, heads=desc.heads) for m in ms]
        for m in (0, 1, 2, 0, 2, 1, 1, 0, 2):
            got = rig.ctx.infer(ms[m], ids[m])
            assert np.abs(got - want[m]).max() <= 2e-2
        rig.ctx.sync()
        st = rig.ctx.stats()
        assert st["bytes_d2h"] == 0 and st["n_miss"] >= 7
        rig.ctx.set_discard(False)                      # back to the paper's behaviour: a real copy
        rig.tensors[ms[2]][5][...] = 0
        rig.ctx.swap_out(ms[2]); rig.ctx.wait(ms[2])
        assert rig.ctx.stats()["bytes_d2h"] == size
        for m in ms:
            for t, o in zip(rig.tensors[m], orig[m]):
                assert np.array_equal(as_bytes(t), as_bytes(o))
    finally:
        rig.close()
