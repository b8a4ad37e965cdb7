"""MI355X-native LRQMM hot path: thin Python binding over the C-ABI library.

The binding only marshals arguments (torch tensors -> device pointers); every
step of the path runs in the HIP kernels of liblrqmm.so.  There is no CPU
fallback: importing the binding without the built library raises.
"""
from .binding import (  # noqa: F401
    AXIS_COL, AXIS_ROW, ROUND_FLOOR, ROUND_NEAREST, MAX_SKETCH, LrqmmError,
    lib_path, load_library, lrqmm_fill_sketch, lrqmm_gemm, lrqmm_matmul, lrqmm_quantize,
    lrqmm_rsvd, lrqmm_workspace_bytes, lrqmm_status_string, Workspace, lrqmm_profile_enable,
    lrqmm_profile_read, PROF_STAGES, SCALE_VECTOR, SCALE_TENSOR, lrqmm_quantize_ex, lrqmm_rsvd_ex,
    lrqmm_gemm_ex, lrqmm_matmul_ex, lrqmm_quantize_residual, lrqmm_residual_workspace_bytes,
    lrqmm_residual_matmul, PROF_GEMM_ONLY, lrqmm_gemm_static, STATIC_SCRATCH_BYTES, ERR_STATIC_LIMIT,
    PREC_FP32, PREC_BF16X2, PREC_BF16, PREC_SUBSPACE_BF16X2,
)
