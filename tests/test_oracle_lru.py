"""Pins for oracle/lru.py."""
import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from oracle.lru import LruResidency, replay
from synth.arrivals import gamma_rates_trace
from golden_values import load as golden


def stack_distance_hits(trace, capacity):
    """Textbook characterisation: a reference hits iff fewer than `capacity`
    distinct other models were referenced since the previous reference to it."""
    hits = []
    for i, m in enumerate(trace):
        prev = None
        for j in range(i - 1, -1, -1):
            if trace[j] == m:
                prev = j
                break
        if prev is None:
            hits.append(False)
        else:
            hits.append(len(set(trace[prev + 1:i])) < capacity)
    return hits


def naive_lru(trace, capacity):
    """Brute force with an explicit recency list (most recent last)."""
    order, out = [], []
    for m in trace:
        if m in order:
            order.remove(m)
            order.append(m)
            out.append(("hit", m, ()))
        else:
            victims = ()
            if len(order) == capacity:
                victims = (order.pop(0),)
            order.append(m)
            out.append(("miss", m, victims))
    return out


@given(st.lists(st.integers(0, 5), min_size=1, max_size=60), st.integers(1, 4))
@settings(max_examples=200, deadline=None)
def test_equal_sizes_is_textbook_lru(trace, cap):
    size = 1000
    ev = replay(cap * size + size - 1, [size] * 6, trace)
    assert [e[0] == "hit" for e in ev] == stack_distance_hits(trace, cap)
    assert ev == naive_lru(trace, cap)


@given(st.lists(st.integers(0, 4), min_size=1, max_size=80),
       st.lists(st.integers(1, 50), min_size=5, max_size=5), st.integers(50, 120))
@settings(max_examples=200, deadline=None)
def test_budget_invariant_unequal_sizes(trace, sizes, budget):
    r = LruResidency(budget, sizes)
    for m in trace:
        before = dict(r.last_use)
        ev = r.touch(m)
        assert r.resident_bytes == sum(sizes[k] for k in r.last_use) <= budget
        assert r.is_resident(m)
        if ev[0] == "miss":
            # victims are exactly the least recently used ones, oldest first, and minimal
            by_age = sorted(before, key=before.get)
            assert list(ev[2]) == by_age[:len(ev[2])]
            if ev[2]:
                freed_without_last = sum(sizes[v] for v in ev[2][:-1])
                assert sum(sizes[k] for k in before) - freed_without_last + sizes[m] > budget
    assert r.peak_resident <= budget


def test_too_big_and_explicit_swap_out():
    r = LruResidency(10, [4, 4, 4, 11])
    with pytest.raises(ValueError):
        r.touch(3)
    r.touch(0); r.touch(1)
    assert r.swap_out(1) == ("out", 1, (1,))       # evicting the most recent one is allowed
    assert r.swap_out(1) == ("out", 1, ())         # idempotent
    assert r.touch(2) == ("miss", 2, ())
    assert r.touch(1) == ("miss", 1, (0,))


def test_paper_cap_as_bytes():
    g = golden()
    size = 6_667_665_408
    r = LruResidency(int(g["sim3_resident"]) * size + 1, [size] * 3)
    for m in (0, 1, 2, 0):
        r.touch(m)
    assert len(r.last_use) == int(g["sim3_resident"])


def test_burstier_traces_swap_less():
    """Section 5.2's observation, as a property of the policy on seeded traces."""
    size = 10
    misses = {}
    for cv in (0.25, 4.0):
        tot = 0
        for seed in range(5):
            _, m = gamma_rates_trace([1, 1, 1], cv=cv, duration=400.0, seed=seed)
            tot += sum(e[0] == "miss" for e in replay(2 * size, [size] * 3, m)) / max(1, len(m))
        misses[cv] = tot / 5
    assert misses[4.0] < 0.6 * misses[0.25]
