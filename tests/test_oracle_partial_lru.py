"""Pins of the block-granular residency oracle (oracle/partial_lru.py)."""
import numpy as np
import pytest

from oracle.lru import LruResidency
from oracle.partial_lru import PartialLruResidency


def random_case(rng, n_models, max_blocks, equal=False):
    if equal:
        shape = [int(rng.integers(1, 9)) for _ in range(int(rng.integers(1, max_blocks + 1)))]
        blocks = [list(shape) for _ in range(n_models)]
    else:
        blocks = [[int(rng.integers(1, 9)) for _ in range(int(rng.integers(1, max_blocks + 1)))]
                  for _ in range(n_models)]
    biggest = max(sum(b) for b in blocks)
    budget = int(rng.integers(biggest, sum(sum(b) for b in blocks) + 2))
    trace = [int(x) for x in rng.integers(0, n_models, size=60)]
    return blocks, budget, trace


def test_single_block_models_reduce_to_whole_model_lru():
    rng = np.random.default_rng(0)
    for _ in range(200):
        n = int(rng.integers(2, 7))
        sizes = [int(rng.integers(1, 20)) for _ in range(n)]
        budget = int(rng.integers(max(sizes), sum(sizes) + 2))
        part = PartialLruResidency(budget, [[s] for s in sizes])
        whole = LruResidency(budget, sizes)
        for step in range(80):
            m = int(rng.integers(0, n))
            if rng.random() < 0.1:
                a, b = part.swap_out(m), whole.swap_out(m)
                assert tuple(v for v, _, _ in a[3]) == b[2]
            else:
                a, b = part.touch(m), whole.touch(m)
                assert (a[0], a[1]) == (b[0], b[1])
                assert tuple(v for v, _, _ in a[3]) == b[2]
            assert part.resident_bytes == whole.resident_bytes
            assert [part.is_resident(i) for i in range(n)] == [whole.is_resident(i) for i in range(n)]
        assert part.peak_resident == whole.peak_resident


def test_invariants_budget_prefix_minimality_and_single_partial_model():
    rng = np.random.default_rng(1)
    for case in range(300):
        blocks, budget, trace = random_case(rng, int(rng.integers(2, 6)), 6)
        r = PartialLruResidency(budget, blocks)
        for m in trace:
            before = r.resident_bytes
            k_before = list(r.k)
            ev = r.touch(m)
            assert r.resident_bytes <= budget
            assert r.resident_bytes == sum(sum(b[:k]) for b, k in zip(blocks, r.k))
            assert r.is_resident(m)
            if ev[0] == "hit":
                assert r.k == k_before and ev[3] == ()
                continue
            need = sum(blocks[m][ev[2]:])
            assert ev[2] == k_before[m]
            freed = 0
            for v, lo, hi in ev[3]:
                assert v != m and 0 <= lo < hi == k_before[v] and r.k[v] == lo      # tails only
                freed += sum(blocks[v][lo:hi])
            assert r.resident_bytes == before - freed + need
            if ev[3]:
                # minimal: putting the last dropped block back would break the budget
                v, lo, hi = ev[3][-1]
                assert r.resident_bytes + blocks[v][lo] > budget
                # victims fall in recency order; all but the last lose everything they had
                for v2, lo2, _ in ev[3][:-1]:
                    assert lo2 == 0
            # at most one model is partially resident, and it is the least recently used resident one
            partial = [i for i in range(len(blocks)) if 0 < r.k[i] < len(blocks[i])]
            assert len(partial) <= 1
            if partial:
                assert r.last_use[partial[0]] == min(r.last_use.values())
            assert set(r.last_use) == {i for i in range(len(blocks)) if r.k[i] > 0}


def flat_priority_simulation(budget, blocks, trace):
    """Independent restatement: all resident (model, block) pairs form one list; what leaves first is the
    pair with the oldest model stamp and, within a model, the highest block index."""
    stamp = {}
    resident = set()
    clock = 0
    log = []
    for m in trace:
        clock += 1
        missing = [(m, b) for b in range(len(blocks[m])) if (m, b) not in resident]
        stamp[m] = clock
        used = sum(blocks[i][b] for i, b in resident)
        need = sum(blocks[i][b] for i, b in missing)
        order = sorted((p for p in resident if p[0] != m), key=lambda p: (stamp[p[0]], -p[1]))
        gone = []
        while missing and used + need > budget:
            p = order.pop(0)
            resident.remove(p)
            used -= blocks[p[0]][p[1]]
            gone.append(p)
        resident.update(missing)
        log.append((bool(missing), sorted(missing), gone))
    return log


def test_equals_flat_priority_list_simulation():
    rng = np.random.default_rng(2)
    for case in range(200):
        blocks, budget, trace = random_case(rng, int(rng.integers(2, 6)), 5)
        r = PartialLruResidency(budget, blocks)
        ref = flat_priority_simulation(budget, blocks, trace)
        for m, (miss, missing, gone) in zip(trace, ref):
            ev = r.touch(m)
            assert (ev[0] == "miss") == miss
            if miss:
                assert missing == [(m, b) for b in range(ev[2], len(blocks[m]))]
                mine = [(v, b) for v, lo, hi in ev[3] for b in range(hi - 1, lo - 1, -1)]
                assert mine == gone


@pytest.mark.parametrize("equal", [True, False])
def test_never_worse_than_whole_model_lru(equal):
    """Resident content is always a superset of the whole-model policy's: no fewer hits, no more bytes loaded."""
    rng = np.random.default_rng(3)
    for case in range(300):
        blocks, budget, trace = random_case(rng, int(rng.integers(2, 7)), 6, equal=equal)
        sizes = [sum(b) for b in blocks]
        part = PartialLruResidency(budget, blocks)
        whole = LruResidency(budget, sizes)
        loaded_whole = 0
        for m in trace:
            a, b = part.touch(m), whole.touch(m)
            if b[0] == "hit":
                assert a[0] == "hit"
            else:
                loaded_whole += sizes[m]
            for i in range(len(blocks)):
                if whole.is_resident(i):
                    assert part.is_resident(i)
        assert part.bytes_loaded <= loaded_whole


def test_worked_example_slack_below_one_model():
    """Three equal models of 4 blocks x 10 bytes under a budget of 110: the third model fits except for one
    block, so every later miss moves exactly one block (hand-derived)."""
    r = PartialLruResidency(110, [[10] * 4] * 3)
    assert r.touch(0) == ("miss", 0, 0, ())
    assert r.touch(1) == ("miss", 1, 0, ())
    assert r.touch(2) == ("miss", 2, 0, ((0, 3, 4),))          # 120 > 110: model 0 loses its last block
    assert r.touch(0) == ("miss", 0, 3, ((1, 3, 4),))          # reload 10 bytes, model 1 (now oldest) pays
    assert r.touch(0) == ("hit", 0, 4, ())
    assert r.touch(1) == ("miss", 1, 3, ((2, 3, 4),))
    assert r.bytes_loaded == 120 + 20
    assert r.swap_out(1) == ("out", 1, 0, ((1, 0, 4),))
    assert r.touch(2) == ("miss", 2, 3, ())                    # room again: nobody is evicted
    assert r.resident_bytes == 80
