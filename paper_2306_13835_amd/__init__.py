"""MI355X-native model swapping: ctypes binding over libcomputron_mi355.so.

Argument marshalling only: every step of the path (copies, residency
decisions, the shard forward pass) runs inside the HIP library.  Importing the
package does not load the library; `paper_2306_13835_amd.lib()` does and
raises if it has not been built (there is no CPU fallback).
"""
from .binding import (lib, Context, Engine, engine_replay, HostPool, CtnError, XFER_DMA, XFER_KERNEL, XFER_AUTO, XFER_DMA_IN_KERNEL_OUT,
                      XFER_KERNEL_IN_DMA_OUT, XFER_DMA_RUNS, EPI_BIAS_F16,
                      EPI_BIAS_RELU_F16, EPI_BIAS_RESID_F32, EPI_F32, residency_replay,
                      workspace_bytes, arena_bytes, slot_bytes, block_residency_replay, predictor_replay, LIB_PATH, DECLARED_SYMBOLS)

__all__ = ["lib", "Context", "Engine", "engine_replay", "HostPool", "CtnError", "XFER_DMA", "XFER_KERNEL", "XFER_AUTO", "XFER_DMA_IN_KERNEL_OUT",
           "XFER_KERNEL_IN_DMA_OUT", "XFER_DMA_RUNS", "EPI_BIAS_F16",
           "EPI_BIAS_RELU_F16", "EPI_BIAS_RESID_F32", "EPI_F32", "residency_replay",
           "workspace_bytes", "arena_bytes", "slot_bytes", "block_residency_replay", "predictor_replay", "LIB_PATH", "DECLARED_SYMBOLS"]
