"""Alias kept for the oracle tests: the recipes live in fs_inputs.workloads."""
from fs_inputs.workloads import (alloc_sequences, blocks_needed, make_tables, shuffle_free_slabs,  # noqa: F401
                                 source_rows, token_index)
from fs_inputs.workloads import fp8_scales_from_rows as fp8_scales  # noqa: F401
