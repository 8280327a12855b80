"""MI355X-native RainFusion hot path: ARM head classifier + block-sparse attention.

The work is done by hand-written HIP kernels behind the C ABI in include/rainfusion.h;
this package is only the ctypes binding over torch device tensors.
"""
from .binding import (  # noqa: F401
    RF_SPATIAL, RF_TEMPORAL, RF_TEXTURAL, RF_DENSE, RF_SAMPLE_FIRST_FRAME, RF_SAMPLE_EQUAL_INTERVAL,
    RF_PLAN_PARTIAL, RF_KEY_TILE, RF_FLAG_TWO_HEAD, RF_FLAG_TEXT_FIRST, RF_FLAG_FORCE_DENSE, RF_FLAG_FIXED_ORDER, RF_FLAG_WIDE_ROWS, RfError, rf_layout, rf_params, library_path, load_library, rf_version,
    rf_status_string, rf_arm_workspace_bytes, rf_arm_classify, rf_sparse_attention, rf_attention_workspace_bytes, rf_arm_classify_plus, rf_sparse_attention_plus, rf_plan_host, rf_plan_order, rf_plan_position_major, RF_LIST_TEMPORAL_POSITION_MAJOR,
    rf_plan_clear, plan_block_counts, rf_arm_classify_noalloc, RF_ATTENTION_MIN_WORKSPACE, RF_ARM_STATIC_SCRATCH_BYTES,
)
