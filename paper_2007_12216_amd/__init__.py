"""rnswino: exact INT8 convolution by Winograd-in-RNS on MI355X (thin binding over the C-ABI library).

Every step of the method runs in the HIP library (`librnswino.so`, built by `build.py` from `csrc/`);
this package only marshals arguments.  PyTorch is used by callers for device memory and streams.
"""
from .binding import (  # noqa: F401
    RnsWinoError, Plan, lib, library_path,
    rnswino_plan, rnswino_plan_destroy, rnswino_filter_transform, rnswino_conv2d, rnswino_conv2d_requant, rnswino_conv2d_events, rnswino_conv2d_static, STATIC_WORKSPACE_BYTES,
    rnswino_direct_filter_bytes, rnswino_direct_workspace_bytes, rnswino_direct_filter_pack, rnswino_direct_conv2d, rnswino_requant_pool,
    rnswino_filter_bytes, rnswino_workspace_bytes, rnswino_output_dims, rnswino_plan_get_matrix, rnswino_plan_get_table,
    rnswino_plan_get_mrc_inverse, rnswino_plan_dynamic_range, rnswino_plan_describe, rnswino_kernel_variants, rnswino_debug_empty_launch, rnswino_debug_stage, rnswino_strerror,
    MATRIX_AT, MATRIX_G, MATRIX_BT, TABLE_INPUT, TABLE_INVERSE, STAGE_U, STAGE_V, STAGE_O,
    FLAG_ALLOW_UNCHECKED_RANGE, FLAG_HOST_ONLY, FLAG_GEMM_BLOCK_64X16, EXPORTED_SYMBOLS,
)
