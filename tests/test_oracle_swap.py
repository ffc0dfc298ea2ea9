"""Pins for oracle/swap.py: byte identity under any swap sequence."""
import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from oracle.swap import DeviceImage, as_bytes


def make(sizes, seed):
    rng = np.random.default_rng(seed)
    return [rng.integers(0, 256, size=n, dtype=np.uint8).view(np.float16) for n in sizes]


@given(st.lists(st.integers(1, 40).map(lambda k: 16 * k), min_size=1, max_size=12), st.integers(0, 2**31))
@settings(max_examples=100, deadline=None)
def test_round_trip_and_scribble(sizes, seed):
    host = make(sizes, seed)
    orig = [h.copy() for h in host]
    img = DeviceImage(sizes)
    img.swap_in(host)
    for t, o in zip(img.tensors, orig):
        assert np.array_equal(t, as_bytes(o))
    for h in host:                      # overwrite the host copy: swap-out must be a real copy
        as_bytes(h)[:] = 0xA5
    img.swap_out(host)
    for h, o in zip(host, orig):
        assert np.array_equal(as_bytes(h), as_bytes(o))


def test_poison_never_survives_and_errors():
    sizes = [32, 2560, 48]
    host = make(sizes, 1)
    img = DeviceImage(sizes, poison=0x7E)
    assert all((t == 0x7E).all() for t in img.tensors)
    with pytest.raises(RuntimeError):
        img.swap_out(host)
    img.swap_in(host)
    assert all(np.array_equal(t, as_bytes(h)) for t, h in zip(img.tensors, host))
    with pytest.raises(ValueError):
        img.swap_in(host[:2])
    with pytest.raises(ValueError):
        DeviceImage([32, 16, 48]).swap_in(host)
