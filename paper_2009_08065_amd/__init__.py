"""Block-structured-pruned linear layers on AMD MI355X (gfx950).

Thin Python binding over the C-ABI library libbsp.so (include/bsp.h).  Every operation runs
in the library's HIP kernels; this package only marshals torch tensors into pointers.
"""
from .bsp import (  # noqa: F401
    ALPHA_NORM, ALPHA_SQNORM, BF16, F16, F32, SCOPE_BLOCK, SCOPE_MATRIX, BspError, Packed,
    bsp_adam_step, bsp_compression_rate, bsp_group_norms, bsp_group_norms_grad, bsp_linear, bsp_linear_dvals, bsp_linear_transposed, bsp_linear_transposed_dense, bsp_pack, bsp_pack_count, bsp_packed_validate,
    bsp_linear_plan, bsp_linear_plan_supported, bsp_linear_planned, bsp_linear_planned_fused, ACT_NONE, ACT_GELU, DVALS_BUILD, DVALS_REUSE, bsp_mask_weights, bsp_penalty_grad,
    bsp_prune_mask, bsp_prune_mask_count, bsp_prune_mask_static, bsp_tile_sumsq, bsp_expand_tile_mask, bsp_rowseg_norms,
    bsp_mask_weights_rowseg, lib,
    library_path,
)
