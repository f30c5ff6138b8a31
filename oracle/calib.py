"""CPU oracle of the calibration step that refines the smoothing factor and the quantization steps of one layer (paper,
appendix "Experiment Settings": during calibration the channel-wise scale c_hat and the quantization parameters Delta are
learnable, learning rates 5e-3 and 5e-2; Sec. 3.1.2, Eq. "loss_ori_overall": the objective is the squared distance between
the full-precision and the quantized function over the calibration set).  Test infrastructure only: plain numpy in float64.

The paper gives the objective and the two learning rates and nothing else; the readings taken here (also listed in the design notes):
  * the function is ONE linear layer (the block-wise pipelines the paper cites reconstruct block by block; a block needs the
    model): L = (1 / T) sum_t || y_ref[t] - y_q[t] ||^2 over the T calibration tokens, y_ref handed in (the full-precision output),
    y_q = x_hat . w_hat^T + b with
        z = (X H) / c,  x_hat = step_x * clamp(round(z / step_x)),      v = (W H) * c,  w_hat[o] = step_w[o] * clamp(round(v[o] / step_w[o]));
  * rounding is passed straight through: d round(u) / du = 1, and a clamped value passes nothing: a value counts as clamped
    when its ROUNDED code leaves [-2^(b-1), 2^(b-1) - 1] (so the largest element of a row quantized with its own absmax step,
    u = +-qmax up to rounding error, is inside whichever way that quotient rounds); the derivative of a quantized value with
    respect to its step is round(u) - u inside the range and the clamp bound outside (the usual learned-step-size rule);
  * what moves: c_hat (through both operands: the weights are multiplied, the activations divided by it), the per-channel
    weight steps, and the activation step when it is a static one (a single value for the tensor).  A dynamic per-token
    activation step (the paper's default) is recomputed from the row, max |z| / qmax, and treated as a constant in the derivative;
  * one update is plain gradient descent with the paper's learning rates, theta <- max(theta - lr * dL/dtheta, floor), the floor
    keeping factors and steps positive (which optimiser the paper's pipeline runs it does not say).
"""
from __future__ import annotations

import numpy as np

from . import dsfq

LR_C_HAT = 5e-3      # appendix "Experiment Settings"
LR_STEP = 5e-2


def fake_quantize(v, step, bits: int = 4, rounding: bool = True):
    """step * clamp(round(v / step), -2^(b-1), 2^(b-1) - 1) (Eq. "quantization" with a given step), and what the
    straight-through rules above need: `inside` (the value was not clamped) and `dstep` = d(result) / d(step).
    v [rows, K]; step a scalar or [rows] (a step per row); steps below the smallest normal fp32 number count as 0
    (result 0, nothing passes).  rounding=False leaves out the rounding (for checks of the chain rule only)."""
    v = np.asarray(v, dtype=np.float64)
    step = np.asarray(step, dtype=np.float64)
    st = step[:, None] if step.ndim == 1 else step
    live = st >= dsfq.MIN_STEP
    safe = np.where(live, st, 1.0)
    lo, hi = -float(1 << (bits - 1)), float((1 << (bits - 1)) - 1)
    u = v / safe
    r = np.rint(u) if rounding else u
    q = np.clip(r, lo, hi)
    inside = (np.rint(u) >= lo) & (np.rint(u) <= hi) & live
    dstep = np.where(inside, q - u, q) * live
    return np.where(live, safe * q, 0.0), inside, dstep


def reconstruction_loss_and_grads(X, W, y_ref, c_hat, w_step, x_step=None, bias=None, pre_signs=None, bits: int = 4,
                                  rounding: bool = True):
    """Loss of one layer over a calibration batch and its derivatives (see the module text).
    X [T, K], W [N, K] (bf16 bits or floats), y_ref [T, N] floats, c_hat [K] > 0, w_step [N] > 0,
    x_step: None (dynamic per-token steps, constants in the derivative) or a positive scalar (static, tensor-wise, learnable).
    Returns dict(loss, grad_c [K], grad_w_step [N], grad_x_step (float or None), y_q [T, N])."""
    R = dsfq.rotate(dsfq.to_f64(X), pre_signs)
    V = dsfq.rotate(dsfq.to_f64(W), pre_signs)
    c = np.asarray(c_hat, dtype=np.float64)
    T = R.shape[0]
    qmax = float((1 << (bits - 1)) - 1)
    z = R / c[None, :]
    v = V * c[None, :]
    if x_step is None:
        dx = np.abs(z).max(axis=1) / qmax
        x_hat, inside_x, dstep_x = fake_quantize(z, dx, bits, rounding)
    else:
        x_hat, inside_x, dstep_x = fake_quantize(z, float(x_step), bits, rounding)
    w_hat, inside_w, dstep_w = fake_quantize(v, np.asarray(w_step, dtype=np.float64), bits, rounding)
    y_q = x_hat @ w_hat.T
    if bias is not None:
        y_q = y_q + dsfq.to_f64(bias)[None, :]
    E = y_q - np.asarray(y_ref, dtype=np.float64)
    loss = float((E ** 2).sum() / T)
    G = 2.0 * E / T                                   # dL / dy_q
    GX = G @ w_hat                                    # dL / dx_hat   [T, K]
    GW = G.T @ x_hat                                  # dL / dw_hat   [N, K]
    grad_w_step = (GW * dstep_w).sum(axis=1)
    gv = GW * inside_w                                # dL / dv
    gz = GX * inside_x                                # dL / dz
    grad_c = (gv * V).sum(axis=0) + (gz * (-z / c[None, :])).sum(axis=0)
    grad_x_step = None if x_step is None else float((GX * dstep_x).sum())
    return dict(loss=loss, grad_c=grad_c, grad_w_step=grad_w_step, grad_x_step=grad_x_step, y_q=y_q)


def descent_step(theta, grad, lr: float, floor: float = 1e-8):
    """theta <- max(theta - lr * grad, floor)"""
    return np.maximum(np.asarray(theta, dtype=np.float64) - lr * np.asarray(grad, dtype=np.float64), floor)
