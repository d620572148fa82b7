"""libtw for MI355X: fused reduce + residual-add + RMSNorm, token split, GEMM
stand-in (TokenWeave, arXiv 2505.11329). Thin ctypes binding over libtw.so; all
work happens in the HIP library. There is no CPU fallback: if the library is
missing and cannot be built, importing the binding's functions raises."""
from .binding import (  # noqa: F401
    TwError,
    lib,
    library_path,
    status_str,
    version,
    device_cu_count,
    split_point,
    fused_grid,
    reduce_add_rmsnorm,
    prepare_reduce_add_rmsnorm,
    reduce_add_rmsnorm_traced,
    reduce_add_rmsnorm_unfused,
    split_launch,
    gemm_bf16,
    overlap_launch,
    hbm_probe,
    hbm_probe_mixed,
    weave_layer,
    smart_split_point,
    gemm_tile_shape,
    should_split,
    fused_layout,
    LayerArgs,
    FusedArgs,
    GemmArgs,
    STATUS,
    PROBE_READ, PROBE_COPY, PROBE_WRITE,
    B_NK, B_KN, CU_SHARED, WEAVE_AUTO, WEAVE_ORDERED, WEAVE_CHAINS,
)
