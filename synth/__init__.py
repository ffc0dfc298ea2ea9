"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

This package holds input *recipes* only: the shape of one tensor-parallel
rank's OPT parameter list, seeded weight / token-id fills and the request
arrival traces.  It contains none of the method's arithmetic (no copy logic,
no replacement policy, no forward pass) and imports neither the oracle nor
the HIP binding.
"""
from .shapes import ShardDesc, CONFIGS, param_list, shard_bytes, shard_params, forward_flop
from .weights import fill_shard, token_ids
from .arrivals import gamma_zipf_trace, gamma_rates_trace, cyclic_trace

__all__ = [
    "ShardDesc", "CONFIGS", "param_list", "shard_bytes", "shard_params",
    "forward_flop", "fill_shard", "token_ids", "gamma_zipf_trace",
    "gamma_rates_trace", "cyclic_trace",
]
