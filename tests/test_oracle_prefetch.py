"""Pins of the load-ahead predictor oracle (oracle/prefetch.py)."""
import numpy as np

from oracle.prefetch import TransitionPredictor, replay


def test_hand_derived_sequence():
    # transitions: 0>1, 1>2, 2>0, 0>1, 1>0, 0>1
    seq = [0, 1, 2, 0, 1, 0, 1]
    #        after 0: none seen; after 1 (0>1 once): 1>? none; ...
    got = replay(3, seq, min_count=2, min_share_percent=50)
    # after index 3 (last=0): row0 = {1:1} -> count 1 < 2 -> None
    # after index 4 (last=1): row1 = {2:1} -> None
    # after index 5 (last=0): row0 = {1:2} -> 1
    # after index 6 (last=1): row1 = {2:1, 0:1} -> best count 1 < 2 -> None
    assert got == [None, None, None, None, None, 1, None]
    assert replay(3, seq, min_count=1, min_share_percent=50) == [None, None, None, 1, 2, 1, 0]   # tie 0/2 -> lowest index
    assert replay(3, seq, min_count=1, min_share_percent=51)[-1] is None                       # 1 of 2 is not 51 %


def test_periodic_sequences_are_learnt_after_min_count_periods():
    for n, period in ((3, [0, 1, 2]), (4, [2, 0, 3, 1]), (5, [1, 1, 4]), (2, [0, 1])):
        for min_count in (1, 2, 3):
            seq = period * 8
            got = replay(n, seq, min_count=min_count, min_share_percent=50)
            # transitions out of every element have been seen min_count times once min_count full
            # periods plus one step have gone by
            start = min_count * len(period)
            for i in range(start, len(seq) - 1):
                if len(set(period)) == len(period):        # each element has one successor
                    assert got[i] == seq[i + 1], (period, min_count, i)
            if len(set(period)) == len(period):
                assert all(g is None for g in got[:min_count])


def test_constant_sequence_predicts_itself():
    got = replay(3, [2] * 6, min_count=2)
    assert got == [None, None, 2, 2, 2, 2]


def test_independent_recount_from_history():
    rng = np.random.default_rng(4)
    for case in range(100):
        n = int(rng.integers(2, 6))
        seq = [int(x) for x in rng.integers(0, n, size=60)]
        mc, share = int(rng.integers(1, 4)), int(rng.integers(1, 101))
        got = replay(n, seq, mc, share)
        for i in range(len(seq)):
            a = seq[i]
            followers = [seq[j + 1] for j in range(i) if seq[j] == a]       # successors of a seen so far
            if not followers:
                assert got[i] is None
                continue
            tally = np.bincount(followers, minlength=n)
            best = int(np.argmax(tally))                                    # first maximum = lowest index
            ok = tally[best] >= mc and 100 * int(tally[best]) >= share * len(followers)
            assert got[i] == (best if ok else None)


def test_rejects_unknown_models():
    p = TransitionPredictor(2)
    try:
        p.observe(2)
    except KeyError:
        return
    raise AssertionError("model index out of range accepted")
