"""Seeded synthetic inputs shared by tests, benchmark and smoke check (no resharding arithmetic)."""
from .generator import (MIX_GPT, MIX_INDEX_GPT, MIX_INDEX_TINY, MIX_TINY, ShardDesc, block_values,
                        canonical_strides, count_mismatch, epoch_order, fill_buffer, linear_index, values)

__all__ = ["MIX_GPT", "MIX_INDEX_GPT", "MIX_INDEX_TINY", "MIX_TINY", "ShardDesc", "block_values",
           "canonical_strides", "count_mismatch", "epoch_order", "fill_buffer", "linear_index", "values"]
