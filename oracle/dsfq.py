"""numpy front end of the C oracle (dsfq_oracle.c).  Test infrastructure only.

Every function here converts its arguments to exact doubles / int8, calls one C
routine, and returns numpy arrays.  `prepare_weights` and `linear` chain the
routines in the order the paper states the method (Sec. 3.2: rotate, smooth,
quantize per token / per output channel, integer product, dequantise).
"""
from __future__ import annotations

import ctypes as C
from dataclasses import dataclass
from typing import Optional

import numpy as np

from . import build as _build

_lib = C.CDLL(_build.build())

_dp = C.POINTER(C.c_double)
_i8p = C.POINTER(C.c_int8)
_u8p = C.POINTER(C.c_uint8)
_u16p = C.POINTER(C.c_uint16)
_i32p = C.POINTER(C.c_int32)

_lib.orc_bf16_from_double.restype = C.c_uint16
_lib.orc_bf16_from_double.argtypes = [C.c_double]
_lib.orc_bf16_from_double_array.restype = None
_lib.orc_bf16_to_double.restype = C.c_double
_lib.orc_bf16_to_double.argtypes = [C.c_uint16]


class OracleError(RuntimeError):
    pass


def _chk(rc: int, what: str):
    if rc != 0:
        raise OracleError(f"{what}: oracle status {rc}")


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _ptr(a: Optional[np.ndarray], typ):
    return None if a is None else a.ctypes.data_as(typ)


def _signs(s) -> Optional[np.ndarray]:
    if s is None:
        return None
    s = np.ascontiguousarray(s, dtype=np.int8)
    if not np.all(np.abs(s) == 1):
        raise ValueError("signs must be +1/-1")
    return s


# ------------------------------------------------------------------ conversions
def bf16_bits_to_f64(bits) -> np.ndarray:
    """bf16 bit patterns (uint16) -> double, exact."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def to_f64(x) -> np.ndarray:
    """Exact double copy of a synthetic tensor: uint16 arrays are bf16 bits, float arrays are values."""
    x = np.asarray(x)
    return bf16_bits_to_f64(x) if x.dtype == np.uint16 else _f64(x)


def bf16_from_f64(v) -> np.ndarray:
    """double -> bf16 bits, one rounding (nearest, ties to even)."""
    v = _f64(v)
    out = np.empty(v.shape, dtype=np.uint16)
    _lib.orc_bf16_from_double_array(_ptr(v, _dp), C.c_size_t(v.size), _ptr(out, _u16p))
    return out


# ------------------------------------------------------------------ steps
def hadamard(K: int, form: str = "recursive") -> np.ndarray:
    """Unnormalised K x K Sylvester Hadamard matrix (int8 entries +-1)."""
    H = np.empty((K, K), dtype=np.int8)
    fn = _lib.orc_hadamard_recursive if form == "recursive" else _lib.orc_hadamard_popcount
    _chk(fn(C.c_int(K), _ptr(H, _i8p)), "hadamard")
    return H


def hadamard_paley(m: int) -> np.ndarray:
    """Unnormalised m x m Hadamard matrix of Paley's construction, m in {12, 20, 28}."""
    H = np.empty((m, m), dtype=np.int8)
    _chk(_lib.orc_hadamard_paley(C.c_int(m), _ptr(H, _i8p)), "hadamard_paley")
    return H


def hadamard_general(K: int) -> np.ndarray:
    """Unnormalised K x K matrix H_{2^n} (x) H_m for K = 2^n m, m in {1, 12, 20, 28} (Sec. 3.2)."""
    H = np.empty((K, K), dtype=np.int8)
    _chk(_lib.orc_hadamard_general(C.c_int(K), _ptr(H, _i8p)), "hadamard_general")
    return H


def rotate(X, pre_signs=None, post_signs=None) -> np.ndarray:
    """X . H with H = diag(pre) . Hhat . diag(post), Hhat the orthonormal Hadamard."""
    X = _f64(X)
    rows, K = X.shape
    pre, post = _signs(pre_signs), _signs(post_signs)
    out = np.empty_like(X)
    _chk(_lib.orc_rotate(_ptr(X, _dp), C.c_int(rows), C.c_int(K), _ptr(pre, _i8p), _ptr(post, _i8p),
                         _ptr(out, _dp)), "rotate")
    return out


def col_absmax(A) -> np.ndarray:
    A = _f64(A)
    out = np.empty(A.shape[1], dtype=np.float64)
    _chk(_lib.orc_col_absmax(_ptr(A, _dp), C.c_int(A.shape[0]), C.c_int(A.shape[1]), _ptr(out, _dp)),
         "col_absmax")
    return out


SMOOTH_FLOOR = 1e-5
MIN_STEP = 2.0 ** -126        # a quantization step below the smallest normal single-precision number counts as 0 (dsfq_oracle.c)


def smooth_factor(a, w, alpha: float = 0.5, floor: float = SMOOTH_FLOOR) -> np.ndarray:
    a, w = _f64(a), _f64(w)
    c = np.empty_like(a)
    _chk(_lib.orc_smooth_factor(_ptr(a, _dp), _ptr(w, _dp), C.c_int(a.size), C.c_double(alpha),
                                C.c_double(floor), _ptr(c, _dp)), "smooth_factor")
    return c


def scale_columns(A, c, inverse: bool) -> np.ndarray:
    A = _f64(A).copy()
    c = _f64(c)
    _chk(_lib.orc_scale_columns(_ptr(A, _dp), C.c_int(A.shape[0]), C.c_int(A.shape[1]), _ptr(c, _dp),
                                C.c_int(1 if inverse else 0)), "scale_columns")
    return A


def quantize_rows(A, bits: int = 4):
    """Per-row symmetric quantizer: returns (delta [rows] f64, codes [rows, K] int8)."""
    A = _f64(A)
    rows, K = A.shape
    delta = np.empty(rows, dtype=np.float64)
    q = np.empty((rows, K), dtype=np.int8)
    _chk(_lib.orc_quantize_rows(_ptr(A, _dp), C.c_int(rows), C.c_int(K), C.c_int(bits), _ptr(delta, _dp),
                                _ptr(q, _i8p)), "quantize_rows")
    return delta, q


def quantize_rows_static(A, delta, bits: int = 4) -> np.ndarray:
    A, delta = _f64(A), _f64(delta)
    rows, K = A.shape
    q = np.empty((rows, K), dtype=np.int8)
    _chk(_lib.orc_quantize_rows_static(_ptr(A, _dp), C.c_int(rows), C.c_int(K), C.c_int(bits),
                                       _ptr(delta, _dp), _ptr(q, _i8p)), "quantize_rows_static")
    return q


def int_gemm(qx, qw) -> np.ndarray:
    qx = np.ascontiguousarray(qx, dtype=np.int8)
    qw = np.ascontiguousarray(qw, dtype=np.int8)
    M, K = qx.shape
    N, K2 = qw.shape
    if K != K2:
        raise ValueError("inner dimensions differ")
    acc = np.empty((M, N), dtype=np.int32)
    _chk(_lib.orc_int_gemm(_ptr(qx, _i8p), _ptr(qw, _i8p), C.c_int(M), C.c_int(N), C.c_int(K),
                           _ptr(acc, _i32p)), "int_gemm")
    return acc


def dequant_bias(acc, dx, dw, bias=None, want_f64: bool = False):
    """Y = bf16(acc * dx[:,None] * dw[None,:] + bias): returns bf16 bits (and the f64 values)."""
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    M, N = acc.shape
    dx, dw = _f64(dx), _f64(dw)
    b = None if bias is None else _f64(bias)
    Y = np.empty((M, N), dtype=np.uint16)
    y = np.empty((M, N), dtype=np.float64) if want_f64 else None
    _chk(_lib.orc_dequant_bias(_ptr(acc, _i32p), _ptr(dx, _dp), _ptr(dw, _dp), _ptr(b, _dp), C.c_int(M),
                               C.c_int(N), _ptr(Y, _u16p), _ptr(y, _dp)), "dequant_bias")
    return (Y, y) if want_f64 else Y


def pack_int4(q) -> np.ndarray:
    q = np.ascontiguousarray(q, dtype=np.int8)
    rows, K = q.shape
    out = np.empty((rows, K // 2), dtype=np.uint8)
    _chk(_lib.orc_pack_int4(_ptr(q, _i8p), C.c_int(rows), C.c_int(K), _ptr(out, _u8p)), "pack_int4")
    return out


def unpack_int4(packed, K: int) -> np.ndarray:
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    rows = packed.shape[0]
    out = np.empty((rows, K), dtype=np.int8)
    _chk(_lib.orc_unpack_int4(_ptr(packed, _u8p), C.c_int(rows), C.c_int(K), _ptr(out, _i8p)), "unpack_int4")
    return out


# ------------------------------------------------------------------ the method, step by step
@dataclass
class PreparedWeights:
    qw: np.ndarray        # [N, K] int8 codes of diag(c) H^T W^T, per output channel
    dw: np.ndarray        # [N] weight steps
    c_hat: np.ndarray     # [K] smoothing factor
    w_colmax: np.ndarray  # [K] max_o |W H|[o, j]
    Ws: np.ndarray        # [N, K] rotated, smoothed weights before quantization


def prepare_weights(W, act_absmax_rot=None, pre_signs=None, post_signs=None, alpha: float = 0.5,
                    bits: int = 4) -> PreparedWeights:
    """Offline half: rotate W, form c_hat from the rotated statistics, smooth, quantize per output channel.

    act_absmax_rot[j] = max_t |X_cal H|[t, j]; None means no smoothing (c_hat = 1).
    """
    Wr = rotate(to_f64(W), pre_signs, post_signs)
    w_colmax = col_absmax(Wr)
    if act_absmax_rot is None:
        c_hat = np.ones(Wr.shape[1], dtype=np.float64)
    else:
        c_hat = smooth_factor(act_absmax_rot, w_colmax, alpha)
    Ws = scale_columns(Wr, c_hat, inverse=False)
    dw, qw = quantize_rows(Ws, bits)
    return PreparedWeights(qw, dw, c_hat, w_colmax, Ws)


def prepare_weights_given(W, c_hat=None, w_step=None, pre_signs=None, post_signs=None, bits: int = 4) -> PreparedWeights:
    """Offline half with the calibrated parameters handed in (appendix, implementation details: the channel-wise factor
    c_hat and the quantization steps are learnable during calibration; what is deployed afterwards is this): rotate W,
    scale column j by the given c_hat[j] (None: 1), and quantize output channel o with the given step w_step[o], codes
    clamped to the signed range (None: the channel's own absmax step, as prepare_weights)."""
    Wr = rotate(to_f64(W), pre_signs, post_signs)
    c = np.ones(Wr.shape[1], dtype=np.float64) if c_hat is None else _f64(c_hat)
    Ws = scale_columns(Wr, c, inverse=False)
    if w_step is None:
        dw, qw = quantize_rows(Ws, bits)
    else:
        dw = _f64(w_step).copy()
        qw = quantize_rows_static(Ws, dw, bits)
    return PreparedWeights(qw, dw, c, col_absmax(Wr), Ws)


def rotated_col_absmax(X_cal, pre_signs=None, post_signs=None) -> np.ndarray:
    return col_absmax(rotate(to_f64(X_cal), pre_signs, post_signs))


def layernorm(X, gamma=None, beta=None, eps: float = 1e-5, round_to_bf16: bool = True) -> np.ndarray:
    """Row-wise LayerNorm as it stands in front of VGGT's qkv and fc1 layers (the "neighbouring normalization layer" of
    Sec. 3.2): y = (x - mean) / sqrt(var + eps) * gamma + beta, mean and (population) variance over the K channels of a
    token, in float64.  With round_to_bf16 the result is rounded to bfloat16 (nearest even) and returned as the exact
    doubles of those bf16 values: what a bf16 LayerNorm kernel hands to the next layer."""
    x = to_f64(X)
    K = x.shape[1]
    mean = x.sum(axis=1, keepdims=True) / K
    var = ((x - mean) ** 2).sum(axis=1, keepdims=True) / K
    y = (x - mean) / np.sqrt(var + eps)
    if gamma is not None:
        y = y * _f64(gamma)[None, :]
    if beta is not None:
        y = y + _f64(beta)[None, :]
    return bf16_bits_to_f64(bf16_from_f64(y)) if round_to_bf16 else y


def gelu(X, round_to_bf16: bool = True) -> np.ndarray:
    """The activation between fc1 and fc2 of VGGT's MLP blocks (the layers of Sec. 3.2 are this network's linear layers):
    GELU(x) = x * Phi(x), Phi the standard normal distribution function, written as erfc(-x / sqrt 2) / 2 so that the
    negative tail keeps its relative accuracy; float64, the library's complementary error function.  With round_to_bf16 the result
    is rounded to bfloat16 (nearest even) and returned as the exact doubles of those values: what a bf16 activation kernel
    hands to fc2."""
    from scipy.special import erfc
    x = to_f64(X)
    y = x * (0.5 * erfc(-x / np.sqrt(2.0)))
    return bf16_bits_to_f64(bf16_from_f64(y)) if round_to_bf16 else y


def rotate_smooth_quant(X, c_hat=None, pre_signs=None, post_signs=None, bits: int = 4):
    """Online half up to the codes: returns (dx [M], qx [M, K] int8, Xs [M, K] f64)."""
    Xr = rotate(to_f64(X), pre_signs, post_signs)
    Xs = Xr if c_hat is None else scale_columns(Xr, c_hat, inverse=True)
    dx, qx = quantize_rows(Xs, bits)
    return dx, qx, Xs


def quantize_rows_asym(A, bits: int = 4):
    """Per-row asymmetric (affine) quantizer, the "Asymmetric" setting of the appendix table of further quantization
    settings; the paper gives no formula, this is the usual min / max one with the range widened to contain 0:
        lo = min(0, min_j a_j), hi = max(0, max_j a_j), delta = (hi - lo) / (2^bits - 1),
        zp = rne(-lo / delta), u_j = clamp(rne(a_j / delta) + zp, 0, 2^bits - 1);   a_j ~ delta * (u_j - zp).
    A row of zeros has delta = 0, zp = 0, u = 0, and so has a row whose step would lie below 2^-126 (as in quantize_rows).
    Returns (delta [rows] f64, zp [rows] int, u [rows, K] uint8)."""
    A = _f64(A)
    levels = (1 << bits) - 1
    lo = np.minimum(A.min(axis=1), 0.0)
    hi = np.maximum(A.max(axis=1), 0.0)
    delta = (hi - lo) / levels
    delta = np.where(delta >= MIN_STEP, delta, 0.0)
    safe = np.where(delta > 0, delta, 1.0)
    zp = np.where(delta > 0, np.rint(-lo / safe), 0.0)
    u = np.clip(np.rint(A / safe[:, None]) + zp[:, None], 0, levels)
    u = np.where(delta[:, None] > 0, u, 0.0)
    return delta, zp.astype(np.int64), u.astype(np.uint8)


def weight_code_sums(qw) -> np.ndarray:
    """sum_j qw[o, j]: what multiplies a token's zero-point offset in the integer product below."""
    return np.asarray(qw, dtype=np.int64).sum(axis=1)


def rotate_smooth_quant_asym(X, c_hat=None, pre_signs=None, post_signs=None, bits: int = 4):
    """Online half with the asymmetric activation quantizer: returns (dx [M], zp [M], u [M, K] uint8, Xs [M, K] f64)."""
    Xr = rotate(to_f64(X), pre_signs, post_signs)
    Xs = Xr if c_hat is None else scale_columns(Xr, c_hat, inverse=True)
    dx, zp, u = quantize_rows_asym(Xs, bits)
    return dx, zp, u, Xs


def int_gemm_asym(u, zp, qw) -> np.ndarray:
    """acc[t, o] = sum_j (u[t, j] - zp[t]) * qw[o, j], int64: activations affine, weights symmetric."""
    e = np.asarray(u, dtype=np.int64) - np.asarray(zp, dtype=np.int64)[:, None]
    return e @ np.asarray(qw, dtype=np.int64).T


def linear_asym(X, prep: "PreparedWeights", bias=None, pre_signs=None, post_signs=None, bits: int = 4):
    """The layer with asymmetric activation codes (weights keep the symmetric per-channel grid):
    returns (Y bf16 bits, y f64, acc int64, u, zp, dx)."""
    dx, zp, u, _ = rotate_smooth_quant_asym(X, prep.c_hat, pre_signs, post_signs, bits)
    acc = int_gemm_asym(u, zp, prep.qw)
    y = acc.astype(np.float64) * dx[:, None] * _f64(prep.dw)[None, :]
    if bias is not None:
        y = y + to_f64(bias)[None, :]
    return bf16_from_f64(y), y, acc, u, zp, dx


@dataclass
class LinearResult:
    Y: np.ndarray     # bf16 bits [M, N]
    y: np.ndarray     # f64 [M, N] before the bf16 rounding
    acc: np.ndarray   # int32 [M, N]
    qx: np.ndarray    # int8 [M, K]
    dx: np.ndarray    # f64 [M]


def linear(X, prep: PreparedWeights, bias=None, pre_signs=None, post_signs=None, bits: int = 4) -> LinearResult:
    dx, qx, _ = rotate_smooth_quant(X, prep.c_hat, pre_signs, post_signs, bits)
    acc = int_gemm(qx, prep.qw)
    b = None if bias is None else to_f64(bias)
    Y, y = dequant_bias(acc, dx, prep.dw, b, want_f64=True)
    return LinearResult(Y, y, acc, qx, dx)
