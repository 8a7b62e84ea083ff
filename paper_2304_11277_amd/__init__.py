"""MI355X-native FlatParameter data path of FSDP (arXiv 2304.11277).

The product is the C-ABI library libfsdp_flat (HIP, gfx950); this package is a
thin ctypes binding with the same entry-point names.  PyTorch supplies device
memory and streams only.
"""
from .binding import (  # noqa: F401
    Batch,
    FSDP_BF16,
    FSDP_F16,
    FSDP_F32,
    FSDP_WALK_AUTO,
    FSDP_WALK_DEEP,
    FSDP_WALK_HALF,
    FSDP_WALK_WIDE,
    FsdpError,
    Layout,
    PtrArray,
    fsdp_cast_shard,
    fsdp_default_divide_factors,
    fsdp_flatten_shard,
    fsdp_found_inf_combine,
    fsdp_grad_scaler_update,
    fsdp_layout_init,
    fsdp_layout_init_ex,
    fsdp_reduce_scatter_adam_fused,
    fsdp_reduce_scatter_adam_prefetch_unshard,
    fsdp_grad_accumulate,
    fsdp_reduce_scatter_accumulate,
    fsdp_reduce_scatter_accumulate_adam_fused,
    fsdp_reduce_scatter_hybrid,
    fsdp_reduce_scatter_hybrid_adam_fused,
    fsdp_reduce_scatter_local,
    fsdp_reduce_scatter_unscale,
    fsdp_shard_adam_step,
    fsdp_shard_adam_step_guarded,
    fsdp_unshard,
    fsdp_unshard_lp,
    fsdp_view_ptr,
    fsdp_views,
    lib,
    library_path,
)
