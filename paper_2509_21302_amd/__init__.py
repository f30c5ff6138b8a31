"""qvggt: W4A4 Dual-Smoothed Fine-Grained Quantization linear layer for MI355X (gfx950).

The product is the C-ABI shared library libqvggt.so (declared in include/qvggt.h, built from
csrc/ by build.py); `binding` is the thin ctypes layer with the same entry-point names.
"""
from .binding import (  # noqa: F401
    QvggtError,
    lib_path,
    load_library,
    EXPORTS,
    qvggt_status_string,
    qvggt_rotated_col_absmax,
    qvggt_prep_weights,
    qvggt_rotate_smooth_quant,
    qvggt_rotate_smooth_quant_static,
    qvggt_layernorm_rotate_smooth_quant,
    qvggt_rotate_smooth_quant_asym,
    qvggt_weight_code_sums,
    qvggt_w4a4_gemm_asym,
    qvggt_e2m3_bytes,
    qvggt_rotate_smooth_quant_e2m3,
    qvggt_workspace_bytes_e2m3,
    qvggt_linear_e2m3,
    qvggt_layernorm_rotate_smooth_quant_e2m3,
    qvggt_codes_to_e2m3,
    qvggt_e2m3_gemm,
    qvggt_w4a4_gemm,
    qvggt_linear,
    qvggt_workspace_bytes,
    qvggt_pack_int4,
    qvggt_unpack_int4,
    qvggt_prep_weights_i8,
    qvggt_rotate_smooth_quant_i8,
    qvggt_i8_gemm,
    qvggt_linear_i8,
    qvggt_workspace_bytes_i8,
    qvggt_layout_int8,
    qvggt_nfds_workspace_bytes,
    qvggt_nfds_moments,
    qvggt_nfds_frame_correlation,
    qvggt_nfds_scores,
    qvggt_nfds_keep_lowest,
    qvggt_nfds_kmeans_step,
    QVGGT_BF16,
    QVGGT_F32,
)

from .module import DsfqLinear  # noqa: E402,F401
