"""CPU oracle: which model to load ahead of its next request.

TEST INFRASTRUCTURE ONLY (never imported by the product path).

The paper's closing section proposes loading models speculatively because
real request streams have structure: the same model many times in a row, or
a subset of models requested in a fixed order.  It gives no algorithm.  The
definition used here is the simplest predictor of that structure, a
first-order transition table over the engine's dispatches:

  * `count[a][b]` = number of times a dispatch of model b directly followed a
    dispatch of model a (a == b included);
  * after a dispatch of model a, the prediction is the b with the largest
    `count[a][b]` (ties: lowest index), provided it was seen at least
    `min_count` times and makes up at least `min_share_percent` per cent of
    the transitions out of a (integer arithmetic:
    `100 * count[a][b] >= min_share_percent * sum(count[a])`); otherwise there
    is no prediction;
  * the engine acts on a prediction only when it is idle (no request queued)
    and the predicted model is not completely resident; the load is an
    ordinary swap-in and therefore a use for the replacement policy.

Parity status: pinned by hand-derived examples, by the closed form on
periodic sequences (after `min_count` periods every prediction is the next
element of the cycle), by the closed form on a constant sequence, and by an
independent recount from the raw history (tests/test_oracle_prefetch.py).
"""
from __future__ import annotations

from typing import List, Optional, Sequence


class TransitionPredictor:
    def __init__(self, n_models: int, min_count: int = 2, min_share_percent: int = 50):
        self.n = int(n_models)
        self.min_count = int(min_count)
        self.min_share_percent = int(min_share_percent)
        self.count = [[0] * self.n for _ in range(self.n)]
        self.last: Optional[int] = None

    def observe(self, m: int) -> None:
        if not 0 <= m < self.n:
            raise KeyError(m)
        if self.last is not None:
            self.count[self.last][m] += 1
        self.last = m

    def predict(self) -> Optional[int]:
        if self.last is None:
            return None
        row = self.count[self.last]
        best = max(range(self.n), key=lambda b: (row[b], -b))
        if row[best] < self.min_count or row[best] == 0:
            return None
        if 100 * row[best] < self.min_share_percent * sum(row):
            return None
        return best


def replay(n_models: int, dispatches: Sequence[int], min_count: int = 2,
           min_share_percent: int = 50) -> List[Optional[int]]:
    """Prediction after each dispatch of the sequence."""
    p = TransitionPredictor(n_models, min_count, min_share_percent)
    out = []
    for m in dispatches:
        p.observe(int(m))
        out.append(p.predict())
    return out
