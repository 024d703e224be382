"""DecDEC decode-step hot path for AMD MI355X (gfx950).

Thin Python binding over the C-ABI library libdecdec.so (include/decdec.h).
Everything the path computes runs in the library's HIP kernels; PyTorch is
used only for device memory, pinned host memory and streams.
"""
from .binding import (  # noqa: F401
    DecdecError, Desc, Workspace, lib, lib_path,
    W_UNIFORM_G128, W_LUT_COL8, R_FP16, R_INT4_SYM_COL, R_INT2_SYM_COL, R_INT8_SYM_COL, R_FMT_OF_BITS, MODE_FUSED, MODE_SERIAL, MODE_TWO_STREAMS,
    decdec_select_topk, decdec_select_bucket, decdec_gemv, decdec_gemv_static, decdec_gemv_idx, decdec_gemv_multi, make_linears, Linear,
    decdec_packed_bytes, decdec_pack_weights, decdec_unpack_weights, decdec_pack_residual_int4, decdec_pack_residual_int,
    decdec_quantize_uniform, decdec_residual_f32, decdec_quantize_residual, decdec_check_pinned, decdec_check_residual_pointer, decdec_sc_buffer_bytes, decdec_partial_buffer_bytes, decdec_strerror,
    STATIC_MAX_N, STATIC_MAX_SELECTED,
    EXPORTED_SYMBOLS,
)
