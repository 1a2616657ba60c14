"""RevFFN reversible MoE block for AMD MI355X: thin Python binding over librevffn.so.

Every arithmetic step runs in the HIP kernels of the shared library; this package
only marshals arguments (torch tensors are used for device memory and streams).
Importing the package does not load the library; the first call does, and raises
if it has not been built (there is no CPU fallback).
"""
from .binding import (Config, Weights, Grads, Context, load_library, library_path,
                      revffn_forward, revffn_inverse, revffn_backward, revffn_backward_stored, revffn_inverse_backward,
                      revffn_stack_forward, revffn_stack_backward, revffn_get_routing,
                      revffn_get_branch, revffn_strerror, RevffnError, EXPORTED_SYMBOLS,
                      WEIGHT_FIELDS, revffn_op_gemm, revffn_op_attention_fwd, revffn_op_attention_bwd,
                      revffn_op_attention_bwd_noalloc, revffn_op_tile_placement,
                      Merged, MERGED_FIELDS, revffn_merge_adapters, revffn_forward_merged, revffn_inverse_merged)

__all__ = ["Config", "Weights", "Grads", "Context", "load_library", "library_path",
           "revffn_forward", "revffn_inverse", "revffn_backward", "revffn_backward_stored", "revffn_inverse_backward",
           "revffn_stack_forward",
           "revffn_stack_backward", "revffn_get_routing", "revffn_get_branch",
           "revffn_strerror", "RevffnError", "EXPORTED_SYMBOLS", "WEIGHT_FIELDS", "revffn_op_gemm",
           "revffn_op_attention_fwd", "revffn_op_attention_bwd", "revffn_op_attention_bwd_noalloc",
           "revffn_op_tile_placement", "Merged", "MERGED_FIELDS", "revffn_merge_adapters", "revffn_forward_merged",
           "revffn_inverse_merged"]
