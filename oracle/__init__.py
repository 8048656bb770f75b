"""CPU oracle (test infrastructure only).

Importable from tests, the smoke check and the benchmark's cpu_baseline leg.
The product package never imports this.
"""
from .segquant_oracle import (  # noqa: F401
    ACT_GELU,
    ACT_NONE,
    ACT_SILU,
    OracleResult,
    activation,
    build,
    calibrate_act,
    calibrate_act_percentile,
    cast_bf16,
    dequant,
    error_bound,
    fp_reference,
    int_gemm,
    num_threads,
    quantize_act,
    quantize_act_dynamic,
    geglu,
    quantize_act_geglu,
    quantize_act_fused,
    quantize_weight,
    quantize_weight_block,
    quantize_weight_w4,
    pack_w4,
    seglinear,
    seglinear_dynamic,
    widen_bf16,
    channel_amax,
    smooth_factors,
    quantize_weight_smoothed,
    smooth_act,
    lowrank,
)
