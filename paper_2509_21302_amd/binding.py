"""ctypes binding of libqvggt.so: argument marshalling only.

Every function takes torch tensors that already live on the GPU (or None where the C ABI
accepts NULL), passes their data pointers and the current HIP stream to the entry point of
the same name, and raises QvggtError on a non-zero status.  No arithmetic happens here, and
there is no fallback: if the library is missing the import of this module fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
QVGGT_BF16, QVGGT_F32 = 0, 1

EXPORTS = [
    "qvggt_status_string", "qvggt_init", "qvggt_mfma_ceiling", "qvggt_rotated_col_absmax", "qvggt_prep_weights", "qvggt_rotate_smooth_quant",
    "qvggt_rotate_smooth_quant_static", "qvggt_layernorm_rotate_smooth_quant",
    "qvggt_rotate_smooth_quant_asym", "qvggt_weight_code_sums", "qvggt_w4a4_gemm_asym",
    "qvggt_e2m3_bytes", "qvggt_codes_to_e2m3", "qvggt_e2m3_gemm",
    "qvggt_rotate_smooth_quant_e2m3", "qvggt_workspace_bytes_e2m3", "qvggt_linear_e2m3",
    "qvggt_own_workspace_bytes", "qvggt_linear_e2m3_own_workspace",
    "qvggt_layernorm_rotate_smooth_quant_e2m3",
    "qvggt_prep_weights_given", "qvggt_gelu_table_bytes", "qvggt_gelu_table", "qvggt_gelu_rotate_smooth_quant", "qvggt_gelu_rotate_smooth_quant_e2m3", "qvggt_gelu_linear_e2m3",
    "qvggt_i8b_bytes", "qvggt_int8_to_blocks", "qvggt_rotate_smooth_quant_i8b", "qvggt_i8b_gemm", "qvggt_workspace_bytes_i8b",
    "qvggt_linear_i8b",
    "qvggt_rotate_smooth_quant_asym_e2m3", "qvggt_rotate_smooth_quant_static_e2m3", "qvggt_e2m3_gemm_shifted",
    "qvggt_w4a4_gemm", "qvggt_linear", "qvggt_workspace_bytes", "qvggt_pack_int4", "qvggt_unpack_int4",
    "qvggt_prep_weights_i8", "qvggt_rotate_smooth_quant_i8", "qvggt_i8_gemm", "qvggt_linear_i8",
    "qvggt_workspace_bytes_i8", "qvggt_layout_int8",
    "qvggt_nfds_workspace_bytes", "qvggt_nfds_moments", "qvggt_nfds_frame_correlation", "qvggt_nfds_scores",
    "qvggt_nfds_keep_lowest", "qvggt_nfds_kmeans_step",
    "qvggt_rotate_rows", "qvggt_calib_workspace_bytes", "qvggt_calib_loss_grad", "qvggt_calib_descent_step",
]


class QvggtError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {qvggt_status_string(status)} (status {status})")


def lib_path() -> str:
    return os.path.join(_HERE, "libqvggt.so")


_lib = None


def load_library() -> C.CDLL:
    """Load libqvggt.so (built in-tree by paper_2509_21302_amd.build); fails loudly if absent."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} not found: build it with `python -m paper_2509_21302_amd.build`")
    lib = C.CDLL(path)
    vp, i, f, sz = C.c_void_p, C.c_int, C.c_float, C.c_size_t
    lib.qvggt_status_string.restype = C.c_char_p
    lib.qvggt_status_string.argtypes = [i]
    lib.qvggt_init.restype = i
    lib.qvggt_init.argtypes = []
    lib.qvggt_mfma_ceiling.restype = i
    lib.qvggt_mfma_ceiling.argtypes = [i, i, vp, vp]
    lib.qvggt_rotated_col_absmax.restype = i
    lib.qvggt_rotated_col_absmax.argtypes = [vp, i, i, i, vp, vp, vp]
    lib.qvggt_prep_weights.restype = i
    lib.qvggt_prep_weights.argtypes = [vp, i, i, i, vp, vp, f, vp, vp, vp, vp]
    lib.qvggt_rotate_smooth_quant.restype = i
    lib.qvggt_rotate_smooth_quant.argtypes = [vp, i, i, i, vp, vp, vp, vp, vp]
    lib.qvggt_rotate_smooth_quant_static.restype = i
    lib.qvggt_rotate_smooth_quant_static.argtypes = [vp, i, i, i, vp, vp, vp, i, vp, vp, vp]
    lib.qvggt_layernorm_rotate_smooth_quant.restype = i
    lib.qvggt_layernorm_rotate_smooth_quant.argtypes = [vp, i, i, i, vp, vp, f, vp, vp, vp, vp, vp]
    lib.qvggt_rotate_smooth_quant_asym.restype = i
    lib.qvggt_rotate_smooth_quant_asym.argtypes = [vp, i, i, i, vp, vp, vp, vp, vp, vp]
    lib.qvggt_weight_code_sums.restype = i
    lib.qvggt_weight_code_sums.argtypes = [vp, i, i, vp, vp]
    lib.qvggt_w4a4_gemm_asym.restype = i
    lib.qvggt_w4a4_gemm_asym.argtypes = [vp, vp, vp, vp, vp, vp, vp, i, i, i, vp, vp]
    lib.qvggt_rotate_smooth_quant_e2m3.restype = i
    lib.qvggt_rotate_smooth_quant_e2m3.argtypes = [vp, i, i, i, vp, vp, vp, vp, vp]
    lib.qvggt_layernorm_rotate_smooth_quant_e2m3.restype = i
    lib.qvggt_layernorm_rotate_smooth_quant_e2m3.argtypes = [vp, i, i, i, vp, vp, f, vp, vp, vp, vp, vp]
    lib.qvggt_rotate_smooth_quant_asym_e2m3.restype = i
    lib.qvggt_rotate_smooth_quant_asym_e2m3.argtypes = [vp, i, i, i, vp, vp, vp, vp, vp, vp]
    lib.qvggt_rotate_smooth_quant_static_e2m3.restype = i
    lib.qvggt_rotate_smooth_quant_static_e2m3.argtypes = [vp, i, i, i, vp, vp, vp, i, vp, vp, vp, vp]
    lib.qvggt_e2m3_gemm_shifted.restype = i
    lib.qvggt_e2m3_gemm_shifted.argtypes = [vp, vp, vp, vp, vp, vp, vp, i, i, i, vp, vp]
    for fn in (lib.qvggt_gelu_rotate_smooth_quant, lib.qvggt_gelu_rotate_smooth_quant_e2m3):
        fn.restype = i
        fn.argtypes = [vp, i, i, i, vp, vp, vp, vp, vp, vp]
    lib.qvggt_gelu_table_bytes.restype = C.c_size_t
    lib.qvggt_gelu_table_bytes.argtypes = []
    lib.qvggt_gelu_table.restype = i
    lib.qvggt_gelu_table.argtypes = [vp, vp]
    lib.qvggt_i8b_bytes.restype = C.c_size_t
    lib.qvggt_i8b_bytes.argtypes = [i, i]
    lib.qvggt_int8_to_blocks.restype = i
    lib.qvggt_int8_to_blocks.argtypes = [vp, i, i, vp, vp]
    lib.qvggt_rotate_smooth_quant_i8b.restype = i
    lib.qvggt_rotate_smooth_quant_i8b.argtypes = [vp, i, i, i, vp, vp, i, vp, vp, vp]
    lib.qvggt_i8b_gemm.restype = i
    lib.qvggt_i8b_gemm.argtypes = [vp, vp, vp, vp, vp, i, i, i, vp, vp, vp]
    lib.qvggt_workspace_bytes_i8b.restype = C.c_size_t
    lib.qvggt_workspace_bytes_i8b.argtypes = [i, i, i]
    lib.qvggt_linear_i8b.restype = i
    lib.qvggt_linear_i8b.argtypes = [vp, i, i, i, i, vp, vp, i, vp, vp, vp, vp, vp, C.c_size_t, vp]
    lib.qvggt_workspace_bytes_e2m3.restype = C.c_size_t
    lib.qvggt_workspace_bytes_e2m3.argtypes = [i, i, i]
    lib.qvggt_gelu_linear_e2m3.restype = i
    lib.qvggt_gelu_linear_e2m3.argtypes = [vp, i, i, i, i, vp, vp, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
    lib.qvggt_linear_e2m3.restype = i
    lib.qvggt_linear_e2m3.argtypes = [vp, i, i, i, i, vp, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
    lib.qvggt_own_workspace_bytes.restype = C.c_size_t
    lib.qvggt_own_workspace_bytes.argtypes = []
    lib.qvggt_linear_e2m3_own_workspace.restype = i
    lib.qvggt_linear_e2m3_own_workspace.argtypes = [vp, i, i, i, i, vp, vp, vp, vp, vp, vp, vp]
    lib.qvggt_e2m3_bytes.restype = C.c_size_t
    lib.qvggt_e2m3_bytes.argtypes = [i, i]
    lib.qvggt_codes_to_e2m3.restype = i
    lib.qvggt_codes_to_e2m3.argtypes = [vp, i, i, vp, vp, vp]
    lib.qvggt_e2m3_gemm.restype = i
    lib.qvggt_e2m3_gemm.argtypes = [vp, vp, vp, vp, vp, i, i, i, vp, vp, vp]
    lib.qvggt_w4a4_gemm.restype = i
    lib.qvggt_w4a4_gemm.argtypes = [vp, vp, vp, vp, vp, i, i, i, vp, vp, vp]
    lib.qvggt_linear.restype = i
    lib.qvggt_linear.argtypes = [vp, i, i, i, i, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.qvggt_prep_weights_given.restype = i
    lib.qvggt_prep_weights_given.argtypes = [vp, i, i, i, vp, vp, vp, i, vp, vp, vp, vp]
    lib.qvggt_prep_weights_i8.restype = i
    lib.qvggt_prep_weights_i8.argtypes = [vp, i, i, i, vp, vp, f, i, vp, vp, vp, vp]
    lib.qvggt_rotate_smooth_quant_i8.restype = i
    lib.qvggt_rotate_smooth_quant_i8.argtypes = [vp, i, i, i, vp, vp, i, vp, vp, vp]
    lib.qvggt_i8_gemm.restype = i
    lib.qvggt_i8_gemm.argtypes = [vp, vp, vp, vp, vp, i, i, i, vp, vp, vp]
    lib.qvggt_linear_i8.restype = i
    lib.qvggt_linear_i8.argtypes = [vp, i, i, i, i, vp, vp, i, vp, vp, vp, vp, vp, sz, vp]
    lib.qvggt_workspace_bytes_i8.restype = sz
    lib.qvggt_workspace_bytes_i8.argtypes = [i, i, i]
    lib.qvggt_layout_int8.restype = i
    lib.qvggt_layout_int8.argtypes = [vp, i, i, vp, i, vp]
    ll, dbl = C.c_longlong, C.c_double
    lib.qvggt_nfds_workspace_bytes.restype = sz
    lib.qvggt_nfds_workspace_bytes.argtypes = [i, ll, i]
    lib.qvggt_nfds_moments.restype = i
    lib.qvggt_nfds_moments.argtypes = [vp, i, i, ll, vp, vp, vp, sz, vp]
    lib.qvggt_nfds_frame_correlation.restype = i
    lib.qvggt_nfds_frame_correlation.argtypes = [vp, i, i, i, ll, vp, vp, sz, vp]
    lib.qvggt_nfds_scores.restype = i
    lib.qvggt_nfds_scores.argtypes = [vp, vp, i, i, dbl, vp, vp]
    lib.qvggt_nfds_keep_lowest.restype = i
    lib.qvggt_nfds_keep_lowest.argtypes = [vp, i, dbl, vp, vp]
    lib.qvggt_nfds_kmeans_step.restype = i
    lib.qvggt_nfds_kmeans_step.argtypes = [vp, i, i, i, vp, vp, vp, vp]
    lib.qvggt_rotate_rows.restype = i
    lib.qvggt_rotate_rows.argtypes = [vp, i, i, i, vp, vp, vp]
    lib.qvggt_calib_workspace_bytes.restype = sz
    lib.qvggt_calib_workspace_bytes.argtypes = [i, i, i]
    lib.qvggt_calib_loss_grad.restype = i
    lib.qvggt_calib_loss_grad.argtypes = [vp, vp, vp, vp, vp, vp, vp, i, i, i, i, vp, vp, vp, vp, vp, sz, vp]
    lib.qvggt_calib_descent_step.restype = i
    lib.qvggt_calib_descent_step.argtypes = [vp, vp, i, f, f, vp]
    lib.qvggt_workspace_bytes.restype = sz
    lib.qvggt_workspace_bytes.argtypes = [i, i, i]
    lib.qvggt_pack_int4.restype = i
    lib.qvggt_pack_int4.argtypes = [vp, i, i, vp, vp]
    lib.qvggt_unpack_int4.restype = i
    lib.qvggt_unpack_int4.argtypes = [vp, i, i, vp, vp]
    _lib = lib
    return lib


# ------------------------------------------------------------------ marshalling helpers
def _ptr(t) -> Optional[int]:
    """Device pointer of a tensor (None -> NULL).  Tensors must be contiguous and on the GPU."""
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("qvggt takes device tensors only")
    if not t.is_contiguous():
        raise ValueError("qvggt takes contiguous tensors only")
    return t.data_ptr()


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.bfloat16:
        return QVGGT_BF16
    if t.dtype == torch.float32:
        return QVGGT_F32
    raise ValueError(f"unsupported dtype {t.dtype}: bf16 or f32")


def _stream(stream) -> Optional[int]:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream or None


def _check(status: int, where: str):
    if status != 0:
        raise QvggtError(status, where)


# ------------------------------------------------------------------ entry points
def qvggt_status_string(status: int) -> str:
    return load_library().qvggt_status_string(int(status)).decode()


def qvggt_init():
    _check(load_library().qvggt_init(), "qvggt_init")


def qvggt_mfma_ceiling(kind, iters, sink, stream=None):
    _check(load_library().qvggt_mfma_ceiling(int(kind), int(iters), _ptr(sink), _stream(stream)), "qvggt_mfma_ceiling")


def qvggt_rotated_col_absmax(X_cal, signs, absmax_rot, stream=None):
    M, K = X_cal.shape
    _check(load_library().qvggt_rotated_col_absmax(_ptr(X_cal), _dtype_code(X_cal), M, K, _ptr(signs),
                                                   _ptr(absmax_rot), _stream(stream)), "qvggt_rotated_col_absmax")


def qvggt_prep_weights(W, act_absmax_rot, signs, alpha, Wq, w_scale, inv_smooth, stream=None):
    N, K = W.shape
    _check(load_library().qvggt_prep_weights(_ptr(W), _dtype_code(W), N, K, _ptr(act_absmax_rot), _ptr(signs),
                                             float(alpha), _ptr(Wq), _ptr(w_scale), _ptr(inv_smooth),
                                             _stream(stream)), "qvggt_prep_weights")


def qvggt_rotate_smooth_quant(X, signs, inv_smooth, Xq, x_scale, stream=None):
    M, K = X.shape
    _check(load_library().qvggt_rotate_smooth_quant(_ptr(X), _dtype_code(X), M, K, _ptr(signs), _ptr(inv_smooth),
                                                    _ptr(Xq), _ptr(x_scale), _stream(stream)),
           "qvggt_rotate_smooth_quant")


def qvggt_rotate_smooth_quant_static(X, signs, inv_smooth, x_step, per_token, Xq, x_scale, stream=None):
    M, K = X.shape
    _check(load_library().qvggt_rotate_smooth_quant_static(_ptr(X), _dtype_code(X), M, K, _ptr(signs), _ptr(inv_smooth),
                                                           _ptr(x_step), int(per_token), _ptr(Xq), _ptr(x_scale),
                                                           _stream(stream)),
           "qvggt_rotate_smooth_quant_static")


def qvggt_layernorm_rotate_smooth_quant(X, gamma, beta, eps, signs, inv_smooth, Xq, x_scale, stream=None):
    M, K = X.shape
    _check(load_library().qvggt_layernorm_rotate_smooth_quant(_ptr(X), _dtype_code(X), M, K, _ptr(gamma), _ptr(beta), float(eps),
                                                              _ptr(signs), _ptr(inv_smooth), _ptr(Xq), _ptr(x_scale),
                                                              _stream(stream)), "qvggt_layernorm_rotate_smooth_quant")


def qvggt_rotate_smooth_quant_asym(X, signs, inv_smooth, Xq, x_scale, x_zero, stream=None):
    M, K = X.shape
    _check(load_library().qvggt_rotate_smooth_quant_asym(_ptr(X), _dtype_code(X), M, K, _ptr(signs), _ptr(inv_smooth), _ptr(Xq),
                                                         _ptr(x_scale), _ptr(x_zero), _stream(stream)),
           "qvggt_rotate_smooth_quant_asym")


def qvggt_weight_code_sums(Wq, N, K, w_codesum, stream=None):
    _check(load_library().qvggt_weight_code_sums(_ptr(Wq), N, K, _ptr(w_codesum), _stream(stream)), "qvggt_weight_code_sums")


def qvggt_w4a4_gemm_asym(Xq, x_scale, x_zero, Wq, w_scale, w_codesum, bias, M, N, K, Y, stream=None):
    _check(load_library().qvggt_w4a4_gemm_asym(_ptr(Xq), _ptr(x_scale), _ptr(x_zero), _ptr(Wq), _ptr(w_scale), _ptr(w_codesum),
                                               _ptr(bias), M, N, K, _ptr(Y), _stream(stream)), "qvggt_w4a4_gemm_asym")


def qvggt_rotate_smooth_quant_e2m3(X, signs, inv_smooth, Xf, x_scale, stream=None):
    M, K = X.shape
    _check(load_library().qvggt_rotate_smooth_quant_e2m3(_ptr(X), _dtype_code(X), M, K, _ptr(signs), _ptr(inv_smooth), _ptr(Xf),
                                                         _ptr(x_scale), _stream(stream)), "qvggt_rotate_smooth_quant_e2m3")


def qvggt_layernorm_rotate_smooth_quant_e2m3(X, gamma, beta, eps, signs, inv_smooth, Xf, x_scale, stream=None):
    M, K = X.shape
    _check(load_library().qvggt_layernorm_rotate_smooth_quant_e2m3(_ptr(X), _dtype_code(X), M, K, _ptr(gamma), _ptr(beta), float(eps),
                                                                   _ptr(signs), _ptr(inv_smooth), _ptr(Xf), _ptr(x_scale),
                                                                   _stream(stream)), "qvggt_layernorm_rotate_smooth_quant_e2m3")


def qvggt_rotate_smooth_quant_asym_e2m3(X, signs, inv_smooth, Xf, x_scale, x_zero, stream=None):
    M, K = X.shape
    _check(load_library().qvggt_rotate_smooth_quant_asym_e2m3(_ptr(X), _dtype_code(X), M, K, _ptr(signs), _ptr(inv_smooth), _ptr(Xf),
                                                              _ptr(x_scale), _ptr(x_zero), _stream(stream)),
           "qvggt_rotate_smooth_quant_asym_e2m3")


def qvggt_rotate_smooth_quant_static_e2m3(X, signs, inv_smooth, x_step, per_token, Xf, x_scale, x_zero, stream=None):
    M, K = X.shape
    _check(load_library().qvggt_rotate_smooth_quant_static_e2m3(_ptr(X), _dtype_code(X), M, K, _ptr(signs), _ptr(inv_smooth),
                                                                _ptr(x_step), int(per_token), _ptr(Xf), _ptr(x_scale), _ptr(x_zero),
                                                                _stream(stream)), "qvggt_rotate_smooth_quant_static_e2m3")


def qvggt_e2m3_gemm_shifted(Xf, x_scale, x_zero, Wf, w_scale, w_codesum, bias, M, N, K, Y, stream=None):
    _check(load_library().qvggt_e2m3_gemm_shifted(_ptr(Xf), _ptr(x_scale), _ptr(x_zero), _ptr(Wf), _ptr(w_scale), _ptr(w_codesum),
                                                  _ptr(bias), M, N, K, _ptr(Y), _stream(stream)), "qvggt_e2m3_gemm_shifted")


def qvggt_gelu_table_bytes():
    return int(load_library().qvggt_gelu_table_bytes())


def qvggt_gelu_table(table, stream=None):
    _check(load_library().qvggt_gelu_table(_ptr(table), _stream(stream)), "qvggt_gelu_table")


def qvggt_gelu_rotate_smooth_quant(X, signs, inv_smooth, gelu_table, Xq, x_scale, stream=None):
    M, K = X.shape
    _check(load_library().qvggt_gelu_rotate_smooth_quant(_ptr(X), _dtype_code(X), M, K, _ptr(signs), _ptr(inv_smooth),
                                                         _ptr(gelu_table), _ptr(Xq), _ptr(x_scale), _stream(stream)),
           "qvggt_gelu_rotate_smooth_quant")


def qvggt_gelu_rotate_smooth_quant_e2m3(X, signs, inv_smooth, gelu_table, Xf, x_scale, stream=None):
    M, K = X.shape
    _check(load_library().qvggt_gelu_rotate_smooth_quant_e2m3(_ptr(X), _dtype_code(X), M, K, _ptr(signs), _ptr(inv_smooth),
                                                              _ptr(gelu_table), _ptr(Xf), _ptr(x_scale), _stream(stream)),
           "qvggt_gelu_rotate_smooth_quant_e2m3")


def qvggt_i8b_bytes(rows, K):
    return int(load_library().qvggt_i8b_bytes(rows, K))


def qvggt_int8_to_blocks(src, rows, K, dst, stream=None):
    _check(load_library().qvggt_int8_to_blocks(_ptr(src), rows, K, _ptr(dst), _stream(stream)), "qvggt_int8_to_blocks")


def qvggt_rotate_smooth_quant_i8b(X, signs, inv_smooth, bits, Xb, x_scale, stream=None):
    M, K = X.shape
    _check(load_library().qvggt_rotate_smooth_quant_i8b(_ptr(X), _dtype_code(X), M, K, _ptr(signs), _ptr(inv_smooth), int(bits),
                                                        _ptr(Xb), _ptr(x_scale), _stream(stream)), "qvggt_rotate_smooth_quant_i8b")


def qvggt_i8b_gemm(Xb, x_scale, Wb, w_scale, bias, M, N, K, Y, acc_debug=None, stream=None):
    _check(load_library().qvggt_i8b_gemm(_ptr(Xb), _ptr(x_scale), _ptr(Wb), _ptr(w_scale), _ptr(bias), M, N, K, _ptr(Y),
                                         _ptr(acc_debug), _stream(stream)), "qvggt_i8b_gemm")


def qvggt_workspace_bytes_i8b(M, N, K):
    return int(load_library().qvggt_workspace_bytes_i8b(M, N, K))


def qvggt_linear_i8b(X, signs, inv_smooth, bits, Wb, w_scale, bias, Y, workspace, stream=None):
    M, K = X.shape
    N = Y.shape[1]
    _check(load_library().qvggt_linear_i8b(_ptr(X), _dtype_code(X), M, N, K, _ptr(signs), _ptr(inv_smooth), int(bits), _ptr(Wb),
                                           _ptr(w_scale), _ptr(bias), _ptr(Y), _ptr(workspace),
                                           workspace.numel() * workspace.element_size(), _stream(stream)), "qvggt_linear_i8b")


def qvggt_workspace_bytes_e2m3(M, N, K):
    return int(load_library().qvggt_workspace_bytes_e2m3(M, N, K))


def qvggt_gelu_linear_e2m3(X, signs, inv_smooth, gelu_table, Wf, w_scale, bias, Y, workspace, stream=None):
    M, K = X.shape
    N = Y.shape[1]
    _check(load_library().qvggt_gelu_linear_e2m3(_ptr(X), _dtype_code(X), M, N, K, _ptr(signs), _ptr(inv_smooth), _ptr(gelu_table), _ptr(Wf),
                                                 _ptr(w_scale), _ptr(bias), _ptr(Y), _ptr(workspace),
                                                 workspace.numel() * workspace.element_size(), _stream(stream)), "qvggt_gelu_linear_e2m3")


def qvggt_linear_e2m3(X, signs, inv_smooth, Wf, w_scale, bias, Y, workspace, stream=None):
    M, K = X.shape
    N = Y.shape[1]
    _check(load_library().qvggt_linear_e2m3(_ptr(X), _dtype_code(X), M, N, K, _ptr(signs), _ptr(inv_smooth), _ptr(Wf), _ptr(w_scale),
                                            _ptr(bias), _ptr(Y), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                            _stream(stream)), "qvggt_linear_e2m3")


def qvggt_own_workspace_bytes():
    return int(load_library().qvggt_own_workspace_bytes())


def qvggt_linear_e2m3_own_workspace(X, signs, inv_smooth, Wf, w_scale, bias, Y, stream=None):
    M, K = X.shape
    N = Y.shape[1]
    _check(load_library().qvggt_linear_e2m3_own_workspace(_ptr(X), _dtype_code(X), M, N, K, _ptr(signs), _ptr(inv_smooth), _ptr(Wf),
                                                          _ptr(w_scale), _ptr(bias), _ptr(Y), _stream(stream)),
           "qvggt_linear_e2m3_own_workspace")


def qvggt_e2m3_bytes(rows, K):
    return int(load_library().qvggt_e2m3_bytes(rows, K))


def qvggt_codes_to_e2m3(packed, rows, K, out, n_unrepresentable, stream=None):
    _check(load_library().qvggt_codes_to_e2m3(_ptr(packed), rows, K, _ptr(out), _ptr(n_unrepresentable), _stream(stream)),
           "qvggt_codes_to_e2m3")


def qvggt_e2m3_gemm(Xf, x_scale, Wf, w_scale, bias, M, N, K, Y, acc_debug=None, stream=None):
    _check(load_library().qvggt_e2m3_gemm(_ptr(Xf), _ptr(x_scale), _ptr(Wf), _ptr(w_scale), _ptr(bias), M, N, K, _ptr(Y),
                                          _ptr(acc_debug), _stream(stream)), "qvggt_e2m3_gemm")


def qvggt_w4a4_gemm(Xq, x_scale, Wq, w_scale, bias, M, N, K, Y, acc_debug=None, stream=None):
    _check(load_library().qvggt_w4a4_gemm(_ptr(Xq), _ptr(x_scale), _ptr(Wq), _ptr(w_scale), _ptr(bias), M, N, K,
                                          _ptr(Y), _ptr(acc_debug), _stream(stream)), "qvggt_w4a4_gemm")


def qvggt_workspace_bytes(M: int, N: int, K: int) -> int:
    return int(load_library().qvggt_workspace_bytes(M, N, K))


def qvggt_linear(X, signs, inv_smooth, Wq, w_scale, bias, Y, workspace, stream=None):
    M, K = X.shape
    N = Y.shape[1]
    _check(load_library().qvggt_linear(_ptr(X), _dtype_code(X), M, N, K, _ptr(signs), _ptr(inv_smooth), _ptr(Wq),
                                       _ptr(w_scale), _ptr(bias), _ptr(Y), _ptr(workspace),
                                       workspace.numel() * workspace.element_size(), _stream(stream)), "qvggt_linear")


def qvggt_pack_int4(codes, packed, stream=None):
    rows, K = codes.shape
    _check(load_library().qvggt_pack_int4(_ptr(codes), rows, K, _ptr(packed), _stream(stream)), "qvggt_pack_int4")


def qvggt_unpack_int4(packed, codes, stream=None):
    rows, K = codes.shape
    _check(load_library().qvggt_unpack_int4(_ptr(packed), rows, K, _ptr(codes), _stream(stream)), "qvggt_unpack_int4")


# ---- the 8-bit / 6-bit settings: int8 codes
def qvggt_prep_weights_given(W, c_hat, signs, w_step, bits, Wq, w_scale, inv_smooth, stream=None):
    N, K = W.shape
    _check(load_library().qvggt_prep_weights_given(_ptr(W), _dtype_code(W), N, K, _ptr(c_hat), _ptr(signs), _ptr(w_step), int(bits),
                                                   _ptr(Wq), _ptr(w_scale), _ptr(inv_smooth), _stream(stream)),
           "qvggt_prep_weights_given")


def qvggt_prep_weights_i8(W, act_absmax_rot, signs, alpha, bits, Wq, w_scale, inv_smooth, stream=None):
    N, K = W.shape
    _check(load_library().qvggt_prep_weights_i8(_ptr(W), _dtype_code(W), N, K, _ptr(act_absmax_rot), _ptr(signs),
                                                float(alpha), int(bits), _ptr(Wq), _ptr(w_scale), _ptr(inv_smooth),
                                                _stream(stream)), "qvggt_prep_weights_i8")


def qvggt_rotate_smooth_quant_i8(X, signs, inv_smooth, bits, Xq, x_scale, stream=None):
    M, K = X.shape
    _check(load_library().qvggt_rotate_smooth_quant_i8(_ptr(X), _dtype_code(X), M, K, _ptr(signs), _ptr(inv_smooth),
                                                       int(bits), _ptr(Xq), _ptr(x_scale), _stream(stream)),
           "qvggt_rotate_smooth_quant_i8")


def qvggt_i8_gemm(Xq, x_scale, Wq, w_scale, bias, M, N, K, Y, acc_debug=None, stream=None):
    _check(load_library().qvggt_i8_gemm(_ptr(Xq), _ptr(x_scale), _ptr(Wq), _ptr(w_scale), _ptr(bias), M, N, K,
                                        _ptr(Y), _ptr(acc_debug), _stream(stream)), "qvggt_i8_gemm")


def qvggt_workspace_bytes_i8(M: int, N: int, K: int) -> int:
    return int(load_library().qvggt_workspace_bytes_i8(M, N, K))


def qvggt_linear_i8(X, signs, inv_smooth, bits, Wq, w_scale, bias, Y, workspace, stream=None):
    M, K = X.shape
    N = Y.shape[1]
    _check(load_library().qvggt_linear_i8(_ptr(X), _dtype_code(X), M, N, K, _ptr(signs), _ptr(inv_smooth), int(bits),
                                          _ptr(Wq), _ptr(w_scale), _ptr(bias), _ptr(Y), _ptr(workspace),
                                          workspace.numel() * workspace.element_size(), _stream(stream)),
           "qvggt_linear_i8")


def qvggt_layout_int8(src, dst, to_library, stream=None):
    rows, K = src.shape
    _check(load_library().qvggt_layout_int8(_ptr(src), rows, K, _ptr(dst), int(to_library), _stream(stream)),
           "qvggt_layout_int8")


# ---- calibration-set arithmetic (Sec. 3.3)
def qvggt_nfds_workspace_bytes(rows: int, count: int, dtype_code: int) -> int:
    return int(load_library().qvggt_nfds_workspace_bytes(rows, count, dtype_code))


def qvggt_nfds_moments(A, mean, var, workspace, stream=None):
    rows, count = A.shape
    _check(load_library().qvggt_nfds_moments(_ptr(A), _dtype_code(A), rows, count, _ptr(mean), _ptr(var), _ptr(workspace),
                                             workspace.numel() * workspace.element_size(), _stream(stream)), "qvggt_nfds_moments")


def qvggt_nfds_frame_correlation(A, corr, workspace, stream=None):
    samples, frames, frame_elems = A.shape
    _check(load_library().qvggt_nfds_frame_correlation(_ptr(A), _dtype_code(A), samples, frames, frame_elems, _ptr(corr),
                                                       _ptr(workspace), workspace.numel() * workspace.element_size(),
                                                       _stream(stream)), "qvggt_nfds_frame_correlation")


def qvggt_nfds_scores(m, s, eps, score, stream=None):
    D, L = m.shape
    _check(load_library().qvggt_nfds_scores(_ptr(m), _ptr(s), D, L, float(eps), _ptr(score), _stream(stream)), "qvggt_nfds_scores")


def qvggt_nfds_keep_lowest(score, p, keep, stream=None):
    _check(load_library().qvggt_nfds_keep_lowest(_ptr(score), score.numel(), float(p), _ptr(keep), _stream(stream)),
           "qvggt_nfds_keep_lowest")


def qvggt_nfds_kmeans_step(c, centres_in, centres_out, labels, stream=None):
    n, dim = c.shape
    _check(load_library().qvggt_nfds_kmeans_step(_ptr(c), n, dim, centres_in.shape[0], _ptr(centres_in), _ptr(centres_out),
                                                 _ptr(labels), _stream(stream)), "qvggt_nfds_kmeans_step")


# ---- calibration: learnable smoothing factor and steps (appendix "Experiment Settings")
def qvggt_rotate_rows(X, signs, R, stream=None):
    M, K = X.shape
    _check(load_library().qvggt_rotate_rows(_ptr(X), _dtype_code(X), M, K, _ptr(signs), _ptr(R), _stream(stream)), "qvggt_rotate_rows")


def qvggt_calib_workspace_bytes(T: int, N: int, K: int) -> int:
    return int(load_library().qvggt_calib_workspace_bytes(T, N, K))


def qvggt_calib_loss_grad(R, V, y_ref, bias, c_hat, w_step, x_step, bits, loss, grad_c, grad_w_step, grad_x_step, workspace, stream=None):
    T, K = R.shape
    N = V.shape[0]
    _check(load_library().qvggt_calib_loss_grad(_ptr(R), _ptr(V), _ptr(y_ref), _ptr(bias), _ptr(c_hat), _ptr(w_step), _ptr(x_step), T, N, K,
                                                int(bits), _ptr(loss), _ptr(grad_c), _ptr(grad_w_step), _ptr(grad_x_step), _ptr(workspace),
                                                workspace.numel() * workspace.element_size(), _stream(stream)), "qvggt_calib_loss_grad")


def qvggt_calib_descent_step(theta, grad, lr, floor=1e-8, stream=None):
    _check(load_library().qvggt_calib_descent_step(_ptr(theta), _ptr(grad), theta.numel(), float(lr), float(floor), _stream(stream)),
           "qvggt_calib_descent_step")
