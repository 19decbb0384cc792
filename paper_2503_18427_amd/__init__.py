"""MI355X (gfx950) adaptive-edge-sampling SpMM: Python binding of libaes_spmm.so.

The functions here have the names of the C entry points declared in
include/aes_spmm.h and only marshal arguments: every step of the method runs in
the HIP kernels.  torch is used for device memory and streams, nothing else.
There is no CPU or eager fallback: if the library is missing or cannot be
loaded the import of a function's first call raises.
"""
from .binding import (  # noqa: F401
    AES_NOALLOC_MAX_ROWS,
    AES_MAX_W,
    AES_Q_AFFINE_FLOOR_U8,
    AES_Q_PER_COLUMN,
    AES_Q_PER_ROW,
    AES_Q_PER_ROW_FOLDED,
    AES_Q_PER_ROW_INLINE,
    AES_Q_PER_TENSOR,
    AES_Q_SYMMETRIC_RNE_I8,
    AES_STRATEGY_ADAPTIVE,
    AES_STRATEGY_AFS,
    AES_STRATEGY_SFS,
    AesError,
    Plan,
    aes_dequantize_features,
    aes_gcn_layer_f32,
    aes_gcn_layer_q8,
    aes_last_error,
    aes_plan_fold_row_constants,
    aes_quantize_features,
    aes_quantize_inline_ld,
    aes_quantize_workspace_bytes,
    aes_sample_build,
    aes_sample_build_noalloc,
    aes_sample_capacity,
    aes_sample_workspace_bytes,
    aes_spmm_f32,
    aes_spmm_fused_f32,
    aes_spmm_fused_q8,
    aes_spmm_q8,
    library,
)
