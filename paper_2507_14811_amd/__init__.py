"""MI355X-native SegLinear + DualScale quantized linear layer (SegQuant, arXiv 2507.14811).

`binding` mirrors the C ABI of libsegquant.so (include/segquant.h); `workloads` holds the seeded
synthetic layer generators; `build` compiles the HIP sources for gfx950.
"""
from .binding import (  # noqa: F401
    GroupItems,
    Layer,
    SqError,
    load_library,
    sq_probe_mfma,
    sq_calibrate_act,
    sq_calibrate_act_percentile,
    sq_calibrate_workspace_bytes,
    SQ_ACT_GELU,
    SQ_ACT_NONE,
    SQ_ACT_SILU,
    sq_quantize_act,
    sq_quantize_act_dynamic,
    sq_quantize_act_fused,
    sq_quantize_act_fused_workspace_bytes,
    sq_quantize_weight,
    sq_quantize_weight_block,
    sq_quantize_weight_w4,
    sq_seglinear,
    sq_seglinear_debug_acc,
    sq_seglinear_dynamic,
    sq_seglinear_grouped,
    sq_seglinear_fused,
    sq_unpack_w4,
    sq_seglinear_fused_dynamic,
    sq_quantize_act_geglu,
    sq_seglinear_grouped_fused,
    sq_seglinear_w4,
    sq_seglinear_w4_debug_acc,
    sq_tuning_set,
    sq_version,
    status_string,
)
