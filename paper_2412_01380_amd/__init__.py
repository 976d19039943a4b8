"""Python binding of libdip (Dynamic Input Pruning / DIP-CA on MI355X).

Argument marshalling only: every step of the hot path runs in the HIP kernels of
libdip.so behind the C ABI declared in include/dip.h.  There is no CPU fallback: if the
shared library has not been built, importing the binding's functions raises.
"""
from .libdip import (  # noqa: F401
    DIP_BF16, DIP_F32, DIP_INT4_G128, DIP_LFU, DIP_LRU, DIP_MAX_N, DIP_OK,
    DIP_ERR_HIP, DIP_ERR_INVALID_ARG, DIP_ERR_UNSUPPORTED, DIP_ERR_WORKSPACE,
    DipError, Cache, Debug, Mlp, Weight, lib, lib_path,
    dip_ca_scores, dip_cache_init, dip_cache_update, dip_gathered_gemv,
    dip_gathered_gemv_workspace_bytes, dip_last_error, dip_prune_topk,
    dip_swiglu_mlp_forward, dip_swiglu_mlp_forward_stack, dip_swiglu_mlp_forward_noalloc,
    DIP_STATIC_SCRATCH_BYTES, dip_swiglu_mlp_forward_stack_workspace_bytes,
    dip_swiglu_mlp_forward_workspace_bytes, dip_tune_gemv, dip_version, MlpStack, EXPORTS, META,
    dip_gemv_launch_shape, dip_profile_enable, dip_set_fusion, dip_fused_launch_shape, dip_stream_read,
    dip_cache_state_bytes, dip_cache_blob_bytes, dip_cache_export, dip_cache_import,
    TieredWeight, TieredMlp, dip_tier_init, dip_tier_init_workspace_bytes, dip_tiered_mlp_forward,
    dip_tiered_mlp_forward_workspace_bytes,
    DIP_GATE_PRUNING, DIP_UP_PRUNING, MlpSplit, PartialDebug, glu_debug, dip_glu_pruning_forward,
    dip_glu_pruning_forward_workspace_bytes, dip_gathered_rowdot, dip_partial_pruning_forward,
    dip_partial_pruning_forward_workspace_bytes,
    dip_swiglu_mlp_forward_batched, dip_swiglu_mlp_forward_batched_workspace_bytes,
    dip_swiglu_mlp_forward_batched_stack, dip_swiglu_mlp_forward_batched_stack_workspace_bytes, dip_profile_read, dip_profile_disable,
)
