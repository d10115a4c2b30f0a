"""Seeded synthetic inputs for chunk attention: segment tables and bf16 tensors.

Shared by the oracle's tests and by the GPU tests / benchmark so that both sides see
the same inputs.  Nothing here performs any attention arithmetic.
"""
from .configs import (BASE_SEED, ChunkCase, Seg, case_by_index, hybrid_chunk, lognormal_lengths,
                      packed_chunk, scaled_case, split_slice)
from .tensors import normal_bf16, to_f64, uniform_u32

__all__ = ["BASE_SEED", "ChunkCase", "Seg", "case_by_index", "hybrid_chunk", "lognormal_lengths",
           "packed_chunk", "scaled_case", "split_slice", "normal_bf16", "to_f64", "uniform_u32"]
