"""CPU oracle for fused residual-add + RMSNorm.  Test infrastructure only.

Nothing in the product package may import this; the test-suite, the smoke
check and the benchmark's CPU-baseline leg are its only callers.
"""
from .addrms_oracle import (  # noqa: F401
    BF16, FP16, FP16_RES32, FP32, VARIANTS,
    addrms, addrms_y64, build, rstd_canonical, silumul, silumul_f64, mergestates,
    bf16_to_f32, f32_to_bf16, f16_to_f32, f32_to_f16,
    bf16_to_f32_array, f32_to_bf16_array, f16_to_f32_array, f32_to_f16_array,
)
