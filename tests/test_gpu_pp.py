"""Pipeline-stage shards (a contiguous layer range of one rank) through the C ABI: stage after stage
reproduces the whole rank's logits, every boundary equals the oracle's stage output, swaps stay exact."""
import time

import numpy as np
import pytest

torch = pytest.importorskip("torch")
import paper_2306_13835_amd as P
from oracle import opt_shard as O
from oracle.swap import as_bytes
from synth import CONFIGS, ShardDesc, fill_shard, token_ids, shard_bytes, param_list
from gpu_util import Rig, errors
from pp_split import stage_params

pytestmark = pytest.mark.gpu

MAX_ABS, MEAN_REL = 2e-2, 1e-3


def assert_close(got, want, what="", residual_stream=False):
    """The acceptance bar is stated for logits, whose spread is about one.  A stage boundary carries
    the residual stream, whose spread grows with depth: there the absolute bound scales with the
    standard deviation of the expected values; the relative bound is the same."""
    mx, rel = errors(got, want)
    bound = MAX_ABS * max(1.0, float(np.std(want))) if residual_stream else MAX_ABS
    print(f"{what} max-abs {mx:.3e} (bound {bound:.3e}) mean-rel {rel:.3e}", flush=True)
    assert np.isfinite(got).all()
    assert mx <= bound and rel <= MEAN_REL, (what, mx, rel)


def add_stage(rig, desc, arrays):
    """Registers a stage whose tensors are copies of `arrays` in the rig's pinned pool."""
    t = []
    for a, (_, shape, _) in zip(arrays, param_list(desc)):
        assert tuple(a.shape) == tuple(shape)
        dst = rig.pool.take(shape, gap=rig.gap)
        dst[...] = a
        t.append(dst)
    m = rig.ctx.register_model(desc, t)
    rig.models.append(m)
    rig.tensors.append(t)
    return m


@pytest.mark.parametrize("device_handoff", [False, True])
@pytest.mark.parametrize("pp,tp,rank", [(2, 1, 0), (4, 2, 1), (2, 4, 3)])
def test_stages_chain_to_the_whole_rank(pp, tp, rank, device_handoff):
    full_desc = ShardDesc(4, 512, 2048, 4, vocab=1024, max_pos=64, tp=tp, rank=rank)
    whole = fill_shard(full_desc, 120 + pp, threads=4)
    stages = [ShardDesc(4, 512, 2048, 4, vocab=1024, max_pos=64, tp=tp, rank=rank, pp=pp, stage=s) for s in range(pp)]
    # room for all stages but one: running the chain also swaps
    budget = sum(shard_bytes(d) for d in stages) - min(shard_bytes(d) for d in stages)
    rig = Rig(stages, budget=budget, max_tokens=2 * 37, mode=P.XFER_AUTO, gap=4096)
    try:
        ms = [add_stage(rig, d, stage_params(whole, 4, pp, d.stage)) for d in stages]
        orig = [[t.copy() for t in rig.tensors[m]] for m in ms]
        ids = token_ids(130, 2, 37, full_desc.vocab)
        want_logits = O.forward(whole, ids, layers=4, heads=4, tp=tp, rank=rank, dtype=np.float32)
        for check_boundaries in (True, False):           # second pass: stages back to back, no host sync between
            x, x_ref = ids, ids
            for d, m in zip(stages, ms):
                out = torch.empty(2, 37, d.out_features, dtype=torch.float32, device="cuda") if device_handoff else None
                x = rig.ctx.infer(m, ids, out=out) if d.stage == 0 else rig.ctx.infer_stage(m, x, out=out)
                assert tuple(x.shape) == (2, 37, d.out_features)
                if check_boundaries:
                    x_ref = O.forward_stage(rig.tensors[m], x_ref, layers=4, heads=4, tp=tp, rank=rank, pp=pp,
                                            stage=d.stage, dtype=np.float32)
                    rig.ctx.sync()
                    assert_close(x.cpu().numpy() if device_handoff else x, x_ref, f"pp={pp} stage {d.stage}",
                                 residual_stream=not d.has_head)
            rig.ctx.sync()
            assert_close(x.cpu().numpy() if device_handoff else x, want_logits, f"pp={pp} chain")
        rig.ctx.sync()
        assert rig.ctx.stats()["n_swap_out"] > 0
        for m in ms:
            for t, o in zip(rig.tensors[m], orig[m]):
                assert np.array_equal(as_bytes(t), as_bytes(o))
    finally:
        rig.close()


@pytest.mark.parametrize("block_residency", [False, True])
@pytest.mark.parametrize("mode", [P.XFER_KERNEL, P.XFER_DMA, P.XFER_AUTO])
def test_stage_shards_round_trip(mode, block_residency):
    """First, middle (no tensors outside the layers) and last stage: device copy equals host, a real copy back."""
    descs = [ShardDesc(6, 256, 1024, 4, vocab=1000, max_pos=30, tp=2, rank=1, pp=3, stage=s) for s in range(3)]
    rig = Rig(descs, mode=mode, block_residency=block_residency, gap=48)
    try:
        for d in descs:
            m = rig.add(d, seed=140 + d.stage)
            assert len(rig.tensors[m]) == {0: 34, 1: 32, 2: 35}[d.stage]
            orig = [t.copy() for t in rig.tensors[m]]
            rig.arena.fill_(0x7E)
            torch.cuda.synchronize()
            rig.ctx.swap_in(m)
            rig.ctx.wait(m)
            assert rig.ctx.resident_blocks(m) == (3, 3)
            for i, o in enumerate(orig):
                assert np.array_equal(as_bytes(rig.ctx.debug_read_param(m, i)), as_bytes(o)), f"tensor {i}"
            for t in rig.tensors[m]:
                t[...] = 0
            rig.ctx.swap_out(m)
            rig.ctx.wait(m)
            for t, o in zip(rig.tensors[m], orig):
                assert np.array_equal(as_bytes(t), as_bytes(o))
        st = rig.ctx.stats()
        assert st["bytes_h2d"] == st["bytes_d2h"] == sum(shard_bytes(d) for d in descs)
    finally:
        rig.close()


def test_stage_argument_errors():
    d0 = ShardDesc(2, 256, 1024, 4, vocab=1000, max_pos=30, pp=2, stage=0)
    d1 = ShardDesc(2, 256, 1024, 4, vocab=1000, max_pos=30, pp=2, stage=1)
    rig = Rig([d0, d1], max_tokens=8)
    eng = None
    try:
        m0, m1 = rig.add(d0, 150), rig.add(d1, 151)
        ids = token_ids(1, 1, 8, d0.vocab)
        hidden = np.zeros((1, 8, 256), dtype=np.float32)
        with pytest.raises(P.CtnError) as e:
            rig.ctx.infer(m1, ids)                      # a later stage needs the residual stream
        assert e.value.code == -1
        out = np.zeros((1, 8, 256), dtype=np.float32)
        rc = P.lib().ctn_infer_stage(rig.ctx.h, m0, ids.ctypes.data, hidden.ctypes.data, 0, 1, 8, out.ctypes.data, 0)
        assert rc == -1                                  # stage 0 takes ids only
        with pytest.raises(P.CtnError):
            rig.ctx.register_model(d1, rig.tensors[m0])  # the first stage's list is not the last stage's
        eng = P.Engine(rig.ctx, 1, 8)
        with pytest.raises(P.CtnError) as e:
            eng.submit(m1, ids, 0.0)                     # the engine's queues hold token ids
        assert e.value.code == -1
        assert eng.submit(m0, ids, 0.0) == 0
    finally:
        if eng:
            eng.close()
        rig.close()


def test_full_size_stage_sampled_batch_rows():
    """One GPU's share of OPT-13B split TP=2 x PP=2 (the paper's hybrid), demand-paged and pipelined as
    bench.py runs it; the oracle evaluates one batch row of the stage."""
    c = CONFIGS["opt13b_tp2_pp2"]
    desc, batch, seq = c["desc"], c["batch"], c["seq"]
    rig = Rig([desc], max_tokens=batch * seq)
    try:
        t0 = time.time()
        m = rig.add(desc, seed=c["wseed"])
        print(f"weights in {time.time() - t0:.1f}s", flush=True)
        ids = token_ids(c["idseed"], batch, seq, desc.vocab)
        out = torch.empty(batch, seq, desc.out_features, dtype=torch.float32, device="cuda")
        rig.ctx.infer(m, ids, out=out)
        rig.ctx.sync()
        got = out.cpu().numpy()
        rows = [5]
        t0 = time.time()
        want = O.forward_stage(rig.tensors[m], ids[rows], layers=desc.layers, heads=desc.heads, tp=desc.tp,
                               rank=desc.rank, pp=desc.pp, stage=desc.stage, dtype=np.float32)
        print(f"oracle row in {time.time() - t0:.1f}s", flush=True)
        assert_close(got[rows], want, "opt13b tp2 pp2 stage 0", residual_stream=True)
        assert np.isfinite(got).all()
        keep = rig.tensors[m][4].copy()
        rig.tensors[m][4][:] = 0
        rig.ctx.swap_out(m); rig.ctx.wait(m)
        assert np.array_equal(rig.tensors[m][4], keep)
    finally:
        rig.close()
