"""TEST INFRASTRUCTURE: the fp64 CPU oracle for the fused reduce + residual-add
+ RMSNorm path and its GEMM stand-in (TokenWeave, arXiv 2505.11329, Appendix A
Listing 1 and Sections 4.2-4.3).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this package. It imports nothing from the HIP library's package.
"""
from .oracle import (  # noqa: F401
    build,
    fused,
    fused_rounded_x,
    unfused,
    unfused_f32sum,
    fused_mt,
    gemm,
    gemm_samples,
    bf16_to_f64,
    f64_to_bf16,
)
