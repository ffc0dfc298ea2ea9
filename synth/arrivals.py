"""Request arrival traces shaped like the paper's simulated workloads.

Section 5.2: every model receives requests from its own independent Gamma
renewal process; the mean rate differs per model (skew) and one coefficient
of variation is shared by all models (burstiness).  A Gamma inter-arrival
time with mean 1/rate and CV c has shape 1/c^2 and scale c^2/rate.
"""
from __future__ import annotations

from typing import Sequence, Tuple

import numpy as np


def _renewal(rng: np.random.Generator, rate: float, cv: float, horizon: float) -> np.ndarray:
    shape, scale = 1.0 / (cv * cv), (cv * cv) / rate
    out, t = [], 0.0
    # draw in blocks until the horizon is passed
    block = max(16, int(rate * horizon * 1.5) + 16)
    while True:
        gaps = rng.gamma(shape, scale, size=block)
        times = t + np.cumsum(gaps)
        out.append(times)
        t = float(times[-1])
        if t > horizon:
            break
    times = np.concatenate(out)
    return times[times <= horizon]


def gamma_rates_trace(rates: Sequence[float], cv: float, duration: float,
                      seed: int) -> Tuple[np.ndarray, np.ndarray]:
    """Merge one Gamma renewal process per model over `duration` seconds.

    Returns (arrival_time float64[n], model int32[n]) sorted by arrival time.
    """
    ts, ms = [], []
    for k, rate in enumerate(rates):
        rng = np.random.Generator(np.random.Philox(key=[seed, k]))
        t = _renewal(rng, float(rate), cv, duration)
        ts.append(t)
        ms.append(np.full(t.shape, k, dtype=np.int32))
    t = np.concatenate(ts)
    m = np.concatenate(ms)
    order = np.argsort(t, kind="stable")
    return t[order], m[order]


def zipf_popularity(n_models: int, s: float) -> np.ndarray:
    w = np.arange(1, n_models + 1, dtype=np.float64) ** (-s)
    return w / w.sum()


def gamma_zipf_trace(n_models: int, total_rate: float, cv: float, zipf_s: float,
                     n_requests: int, seed: int) -> Tuple[np.ndarray, np.ndarray]:
    """Zipf(s)-skewed per-model rates summing to `total_rate`; first `n_requests` arrivals."""
    rates = total_rate * zipf_popularity(n_models, zipf_s)
    horizon = 1.25 * n_requests / total_rate
    while True:
        t, m = gamma_rates_trace(rates, cv, horizon, seed)
        if t.size >= n_requests:
            return t[:n_requests].copy(), m[:n_requests].copy()
        horizon *= 1.5


def cyclic_trace(n_models: int, period_s: float, n_requests: int, jitter: float = 0.0,
                 seed: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """Models requested in a fixed order (0, 1, ..., n-1, 0, ...), one request every `period_s`
    seconds, each arrival shifted by a uniform draw from [0, jitter * period_s).  The kind of
    structured stream the paper's closing section gives as a case for loading ahead."""
    rng = np.random.Generator(np.random.Philox(key=[seed, 0]))
    t = period_s * (np.arange(n_requests, dtype=np.float64) + jitter * rng.random(n_requests))
    m = (np.arange(n_requests) % n_models).astype(np.int32)
    return t, m
