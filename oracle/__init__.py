"""CPU oracle for the swap / residency / shard-forward hot path.

TEST INFRASTRUCTURE ONLY: imported by tests/, by `__graft_entry__.smoke()` and
by the `cpu_baseline` leg of `bench.py`, never by the product package.  It
shares no code with the HIP library and takes every input as plain arrays.
"""
