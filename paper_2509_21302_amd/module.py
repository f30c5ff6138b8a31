"""A small convenience object around the C ABI: one quantized linear layer, prepared once, applied many times.

It only allocates device tensors with torch and calls the entry points of the same names; no arithmetic of the
method happens here.  `bits` = 4 uses the packed 4-bit path, 5..8 the int8-code path (Sec. 4.1 settings, appendix);
`act_bits` different from `bits` is a mixed-precision layer (e.g. 4-bit weights, 8-bit activations) on the int8-code path.
"""
from __future__ import annotations

from typing import Optional

import torch

from . import binding as q


class DsfqLinear:
    """Y = X W^T + b with W and X quantized as in Sec. 3.2 (rotation, smoothing, per-channel / per-token codes).

    weight: [N, K] bf16 or f32 device tensor; bias: [N] bf16 device tensor or None; signs: int8 [K] of +-1 or None;
    calibration: [M_cal, K] activations for the smoothing statistic, or None for rotation only (c = 1).
    """

    def __init__(self, weight: torch.Tensor, bias: Optional[torch.Tensor] = None, signs: Optional[torch.Tensor] = None,
                 calibration: Optional[torch.Tensor] = None, alpha: float = 0.5, bits: int = 4,
                 act_bits: Optional[int] = None, pre_gelu: bool = False):
        act_bits = bits if act_bits is None else act_bits
        if not 4 <= bits <= 8 or not 4 <= act_bits <= 8:
            raise ValueError("bits and act_bits must be in 4..8")
        self.N, self.K = weight.shape
        # pre_gelu: the layer computes GELU(X) W^T + b, the activation applied as X is read (fc2 of an MLP block fed with fc1's output)
        if pre_gelu and not (bits == 4 and act_bits == 4 and self.K in (1024, 2048, 4096)):
            raise ValueError("pre_gelu needs the 4-bit setting and K = 1024, 2048 or 4096")
        self.pre_gelu = pre_gelu
        self.gelu_table = None
        if pre_gelu:         # the activation as a table of correctly rounded bf16 results, built on the device once
            self.gelu_table = torch.empty(q.qvggt_gelu_table_bytes(), dtype=torch.uint8, device=weight.device)
            q.qvggt_gelu_table(self.gelu_table)
        self.bits, self.act_bits, self.bias, self.signs = bits, act_bits, bias, signs
        self.packed = bits == 4 and act_bits == 4            # both 4-bit: two codes per byte; otherwise int8 codes
        dev = weight.device
        absmax = None
        if calibration is not None:
            absmax = torch.empty(self.K, dtype=torch.float32, device=dev)
            q.qvggt_rotated_col_absmax(calibration, signs, absmax)
        self.w_scale = torch.empty(self.N, dtype=torch.float32, device=dev)
        self.inv_smooth = torch.empty(self.K, dtype=torch.float32, device=dev)
        if self.packed:
            self.Wq = torch.empty(self.N, self.K // 2, dtype=torch.uint8, device=dev)
            q.qvggt_prep_weights(weight, absmax, signs, alpha, self.Wq, self.w_scale, self.inv_smooth)
            # the same codes as E2M3 numbers for the 6-bit floating-point matrix path (bf16 inputs, K = 1024 / 2048 / 4096)
            self.Wf = None
            if self.K in (1024, 2048, 4096):
                self.Wf = torch.empty(q.qvggt_e2m3_bytes(self.N, self.K), dtype=torch.uint8, device=dev)
                lost = torch.zeros(1, dtype=torch.int32, device=dev)
                q.qvggt_codes_to_e2m3(self.Wq, self.N, self.K, self.Wf, lost)
                if int(lost.item()) != 0:        # cannot happen with the absmax steps of qvggt_prep_weights (codes lie in [-7, 7])
                    raise RuntimeError(f"{int(lost.item())} weight codes -8 have no E2M3 value")
        else:
            self.Wq = torch.empty(self.N, self.K, dtype=torch.int8, device=dev)
            q.qvggt_prep_weights_i8(weight, absmax, signs, alpha, bits, self.Wq, self.w_scale, self.inv_smooth)
            # the same codes in 128-row blocks for the GEMM with contiguous operand transfers (bf16 inputs, K = 1024 / 2048 / 4096)
            self.Wb = None
            if self.K in (1024, 2048, 4096):
                self.Wb = torch.empty(q.qvggt_i8b_bytes(self.N, self.K), dtype=torch.int8, device=dev)
                q.qvggt_int8_to_blocks(self.Wq, self.N, self.K, self.Wb)
        self._ws = None

    def _workspace(self, M: int, dev) -> torch.Tensor:
        need = q.qvggt_workspace_bytes(M, self.N, self.K) if self.packed else q.qvggt_workspace_bytes_i8(M, self.N, self.K)
        if self.packed and self.Wf is not None:
            need = max(need, q.qvggt_workspace_bytes_e2m3(M, self.N, self.K))
        if not self.packed and self.Wb is not None:
            need = max(need, q.qvggt_workspace_bytes_i8b(M, self.N, self.K))
        if self._ws is None or self._ws.numel() < need or self._ws.device != dev:
            self._ws = torch.empty(need, dtype=torch.uint8, device=dev)
        return self._ws

    def __call__(self, X: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """X: [M, K] bf16 or f32 on the GPU; returns bf16 [M, N] (written into `out` when given)."""
        M = X.shape[0]
        Y = out if out is not None else torch.empty(M, self.N, dtype=torch.bfloat16, device=X.device)
        ws = self._workspace(M, X.device)
        if self.pre_gelu:
            if X.dtype != torch.bfloat16:
                raise ValueError("pre_gelu needs bf16 input")
            q.qvggt_gelu_linear_e2m3(X, self.signs, self.inv_smooth, self.gelu_table, self.Wf, self.w_scale, self.bias, Y, ws)
        elif self.packed and self.Wf is not None and X.dtype == torch.bfloat16:
            q.qvggt_linear_e2m3(X, self.signs, self.inv_smooth, self.Wf, self.w_scale, self.bias, Y, ws)      # same Y, bit for bit
        elif self.packed:
            q.qvggt_linear(X, self.signs, self.inv_smooth, self.Wq, self.w_scale, self.bias, Y, ws)
        elif self.Wb is not None and X.dtype == torch.bfloat16:
            q.qvggt_linear_i8b(X, self.signs, self.inv_smooth, self.act_bits, self.Wb, self.w_scale, self.bias, Y, ws)   # same Y
        else:
            q.qvggt_linear_i8(X, self.signs, self.inv_smooth, self.act_bits, self.Wq, self.w_scale, self.bias, Y, ws)
        return Y
