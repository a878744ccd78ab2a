"""GRAT grouped sparse attention for AMD MI355X: Python binding over the libgrat C ABI."""
from .grat import (GratError, grat_attention_fwd, grat_attention_global_fwd, grat_attention_packed_fwd,
                   grat_block_list_shape, grat_build_block_lists, grat_dense_attention_fwd,
                   grat_validate_block_lists, lib)
from .probe import grat_probe_mfma

__all__ = ["GratError", "grat_attention_fwd", "grat_attention_global_fwd", "grat_attention_packed_fwd",
           "grat_block_list_shape", "grat_build_block_lists", "grat_dense_attention_fwd", "grat_probe_mfma",
           "grat_validate_block_lists", "lib"]
