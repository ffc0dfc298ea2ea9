"""Pins for oracle/engine.py (request scheduling on a simulated clock)."""
import numpy as np
from hypothesis import given, settings, strategies as st

from oracle.engine import latencies, simulate
from golden_values import load as golden


def tick_simulation(arrival, model_of, n_models, max_batch, capacity, t_hit, t_miss):
    """Independent brute force on integer times: advance one tick at a time; when the server is
    free, serve the queue whose oldest waiting request arrived first (lower model on ties)."""
    n = len(arrival)
    done = [None] * n
    resident, t, busy_until, order = [], 0, 0, []
    while any(d is None for d in done):
        if t >= busy_until:
            waiting = [i for i in range(n) if done[i] is None and arrival[i] <= t]
            if waiting:
                first = min(waiting, key=lambda i: (arrival[i], model_of[i], i))
                m = model_of[first]
                batch = [i for i in waiting if model_of[i] == m][:max_batch]
                miss = m not in resident
                if miss:
                    if len(resident) == capacity:
                        resident.pop(0)
                else:
                    resident.remove(m)
                resident.append(m)
                busy_until = t + (t_miss if miss else t_hit)
                for i in batch:
                    done[i] = busy_until
                order.append((t, busy_until, m, tuple(batch), miss))
        t += 1
    return order


trace = st.lists(st.tuples(st.integers(0, 40), st.integers(0, 3)), min_size=1, max_size=25)


@given(trace, st.integers(1, 4), st.integers(1, 3), st.integers(1, 3), st.integers(3, 7))
@settings(max_examples=300, deadline=None)
def test_equals_tick_by_tick_brute_force(reqs, max_batch, capacity, t_hit, t_miss):
    reqs = sorted(reqs, key=lambda r: r[0])
    arrival = [float(a) for a, _ in reqs]
    model_of = [m for _, m in reqs]
    got, lru = simulate(arrival, model_of, 4, max_batch, capacity * 10, [10] * 4,
                        lambda m, b, miss: float(t_miss if miss else t_hit))
    want = tick_simulation([int(a) for a in arrival], model_of, 4, max_batch, capacity, t_hit, t_miss)
    assert [(int(a), int(b), m, r, x) for a, b, m, r, x in got] == want
    assert lru.peak_resident <= capacity * 10


@given(trace, st.integers(1, 5))
@settings(max_examples=200, deadline=None)
def test_invariants(reqs, max_batch):
    reqs = sorted(reqs, key=lambda r: r[0])
    arrival = [float(a) for a, _ in reqs]
    model_of = [m for _, m in reqs]
    batches, _ = simulate(arrival, model_of, 4, max_batch, 20, [10] * 4, lambda m, b, miss: 1.0 + b + 3 * miss)
    served = [r for b in batches for r in b[3]]
    assert sorted(served) == list(range(len(reqs)))                  # everyone exactly once
    t_prev = 0.0
    for start, finish, m, rs, _ in batches:
        assert 1 <= len(rs) <= max_batch and all(model_of[r] == m for r in rs)
        assert start >= t_prev and all(arrival[r] <= start for r in rs) and finish > start
        t_prev = finish
        waiting = [r for r in range(len(reqs)) if arrival[r] <= start and r not in
                   [x for b in batches if b[0] < start for x in b[3]]]
        assert min(arrival[r] for r in waiting) == arrival[rs[0]]    # the oldest head was chosen
    for m in range(4):                                               # FIFO within a model
        mine = [r for r in served if model_of[r] == m]
        assert mine == sorted(mine)


def test_single_queue_batch_one_is_the_textbook_single_server_recursion():
    rng = np.random.default_rng(0)
    arrival = np.cumsum(rng.exponential(1.0, 200)).tolist()
    s = 0.8
    batches, _ = simulate(arrival, [0] * 200, 1, 1, 10, [10], lambda m, b, miss: s)
    finish, prev = [], 0.0
    for a in arrival:                 # Lindley: departure_i = max(arrival_i, departure_{i-1}) + s
        prev = max(a, prev) + s
        finish.append(prev)
    assert np.allclose([b[1] for b in batches], finish)
    assert np.allclose(latencies(arrival, batches), np.array(finish) - np.array(arrival))


def test_paper_batch_caps():
    g = golden()
    arrival = [0.0] * 40
    for cap in (int(g["sim3_max_batch"]), int(g["sim6_max_batch"])):
        batches, _ = simulate(arrival, [0] * 40, 1, cap, 10, [10], lambda m, b, miss: 1.0)
        assert [len(b[3]) for b in batches] == [cap] * (40 // cap) + ([40 % cap] if 40 % cap else [])


# ---- the two-lane engine (asynchronous load entries) -------------------------------------------

def tick_simulation_async(arrival, model_of, n_models, max_batch, capacity, t_hit, t_miss):
    """Independent brute force on integer times for the two-lane engine."""
    n = len(arrival)
    taken = [False] * n
    resident, order = [], []
    busy = {0: 0, 1: 0}
    loading = {}
    t = 0
    while not all(taken):
        for m in list(loading):
            if loading[m] <= t:
                del loading[m]
        while True:
            waiting = [i for i in range(n) if not taken[i] and arrival[i] <= t]
            heads = {}
            for i in waiting:
                heads.setdefault(model_of[i], i)           # first waiting request of each model
            choice = None
            for i in sorted(heads.values(), key=lambda i: (arrival[i], model_of[i])):
                m = model_of[i]
                lane = 0 if m in resident else 1
                if m not in loading and busy[lane] <= t:
                    choice = (m, lane)
                    break
            if choice is None:
                break
            m, lane = choice
            batch = [i for i in waiting if model_of[i] == m][:max_batch]
            miss = lane == 1
            if miss:
                if len(resident) == capacity:
                    resident.pop(0)
            else:
                resident.remove(m)
            resident.append(m)
            busy[lane] = t + (t_miss if miss else t_hit)
            if miss:
                loading[m] = busy[lane]
            for i in batch:
                taken[i] = True
            order.append((t, busy[lane], m, tuple(batch), miss, lane))
        t += 1
    return order


@given(trace, st.integers(1, 4), st.integers(1, 3), st.integers(1, 3), st.integers(3, 7))
@settings(max_examples=300, deadline=None)
def test_async_equals_tick_by_tick_brute_force(reqs, max_batch, capacity, t_hit, t_miss):
    from oracle.engine import simulate_async
    reqs = sorted(reqs, key=lambda r: r[0])
    arrival = [float(a) for a, _ in reqs]
    model_of = [m for _, m in reqs]
    got, lru = simulate_async(arrival, model_of, 4, max_batch, capacity * 10, [10] * 4,
                              lambda m, b, miss: float(t_miss if miss else t_hit))
    want = tick_simulation_async([int(a) for a in arrival], model_of, 4, max_batch, capacity, t_hit, t_miss)
    assert [(int(a), int(b), m, r, x, l) for a, b, m, r, x, l in got] == want
    assert lru.peak_resident <= capacity * 10


@given(trace, st.integers(1, 5))
@settings(max_examples=200, deadline=None)
def test_async_invariants(reqs, max_batch):
    from oracle.engine import simulate_async
    reqs = sorted(reqs, key=lambda r: r[0])
    arrival = [float(a) for a, _ in reqs]
    model_of = [m for _, m in reqs]
    batches, _ = simulate_async(arrival, model_of, 4, max_batch, 20, [10] * 4, lambda m, b, miss: 1.0 + b + 5 * miss)
    served = [r for b in batches for r in b[3]]
    assert sorted(served) == list(range(len(reqs)))
    for lane in (0, 1):                                              # a lane runs one batch at a time
        mine = sorted(b for b in batches if b[5] == lane)
        for a, b in zip(mine, mine[1:]):
            assert b[0] >= a[1]
    for start, finish, m, rs, miss, lane in batches:
        assert 1 <= len(rs) <= max_batch and all(model_of[r] == m for r in rs)
        assert all(arrival[r] <= start for r in rs) and finish > start
        assert lane == (1 if miss else 0)
        # no other batch of the same model runs while its miss is in flight
        if miss:
            assert not [b for b in batches if b[2] == m and start < b[0] < finish]
    for m in range(4):
        mine = [r for b in sorted(batches) for r in b[3] if model_of[r] == m]
        assert mine == sorted(mine)                                  # FIFO within a model


def test_async_single_model_equals_the_serial_engine():
    from oracle.engine import simulate_async
    rng = np.random.default_rng(5)
    arrival = np.cumsum(rng.exponential(0.7, 120)).tolist()
    svc = lambda m, b, miss: 0.5 + 0.1 * b + (2.0 if miss else 0.0)
    serial, _ = simulate(arrival, [0] * 120, 1, 4, 10, [10], svc)
    two_lane, _ = simulate_async(arrival, [0] * 120, 1, 4, 10, [10], svc)
    assert [b[:5] for b in two_lane] == list(serial)


def test_async_hit_overtakes_a_miss_in_flight_hand_derived():
    """Room for two models.  A is loaded by its first request (5 s).  B's first request arrives at 6 and
    loads until 11; a request for A at 7 is a hit and finishes at 8 on the other lane, where the serial
    engine would have made it wait until 12."""
    from oracle.engine import simulate_async
    arrival, model_of = [0.0, 6.0, 7.0, 7.5], [0, 1, 0, 1]
    svc = lambda m, b, miss: 5.0 if miss else 1.0
    got, _ = simulate_async(arrival, model_of, 2, 1, 20, [10, 10], svc)
    assert got == [(0.0, 5.0, 0, (0,), True, 1), (6.0, 11.0, 1, (1,), True, 1), (7.0, 8.0, 0, (2,), False, 0),
                   (11.0, 12.0, 1, (3,), False, 0)]          # B's second request waits for B's load, then hits
    serial, _ = simulate(arrival, model_of, 2, 1, 20, [10, 10], svc)
    assert serial[2][:3] == (11.0, 12.0, 0)
