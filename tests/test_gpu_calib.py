"""GPU parity of the calibration-side kernels (rotation to fp32, reconstruction loss of one layer and its straight-through
derivatives, the descent step) against oracle/calib.py.  Both sides take the same bf16 / f32 inputs; the GPU computes in fp32,
the oracle in float64: a fake-quantized value falls on the other side of a rounding knife edge on about 1e-6 of the elements
(one or two weight codes of a layer), and one flipped weight code moves that channel's derivatives by a percent: the bars are
1e-3 on the loss and 1e-2 (relative, in the 2-norm) on each derivative vector, the measured figures are recorded."""
import numpy as np
import pytest
import torch

import oracle
import synth
from oracle import calib
from tests import gpu_util as G

pytestmark = pytest.mark.gpu
q = G.q


def _rel(a, b):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


@pytest.mark.parametrize("K,dtype", [(128, "f32"), (1024, "bf16"), (4096, "bf16"), (8192, "f32")])
def test_rotate_rows(K, dtype):
    rows = 37
    rng = np.random.default_rng(K)
    x = rng.standard_t(3, (rows, K)).astype(np.float32)
    X = synth.f32_to_bf16_bits(x) if dtype == "bf16" else x
    signs = np.where(rng.random(K) < 0.5, -1, 1).astype(np.int8)
    want = oracle.rotate(oracle.to_f64(X), signs)
    R = torch.full((rows, K), float("nan"), dtype=torch.float32, device=G.DEV)
    q.qvggt_rotate_rows(G.to_dev(X), G.to_dev(signs), R)
    got = R.cpu().numpy().astype(np.float64)
    assert np.abs(got - want).max() <= 2e-6 * np.abs(want).max()
    R2 = torch.empty_like(R)
    q.qvggt_rotate_rows(G.to_dev(X), None, R2)
    assert np.abs(R2.cpu().numpy() - oracle.rotate(oracle.to_f64(X))).max() <= 2e-6 * np.abs(want).max()


def _layer(T, N, K, seed, bias=True):
    rng = np.random.default_rng(seed)
    x = rng.standard_t(3, (T, K)).astype(np.float32)
    x[:, rng.choice(K, max(1, K // 100), replace=False)] *= 50
    x[: min(5, T)] *= 20
    X = synth.f32_to_bf16_bits(x)
    W = synth.f32_to_bf16_bits((rng.standard_normal((N, K)) * 0.02).astype(np.float32))
    b = synth.f32_to_bf16_bits((rng.standard_normal(N) * 0.02).astype(np.float32)) if bias else None
    signs = np.where(rng.random(K) < 0.5, -1, 1).astype(np.int8)
    y_ref = oracle.to_f64(X) @ oracle.to_f64(W).T + (oracle.to_f64(b) if bias else 0.0)
    return X, W, b, signs, y_ref.astype(np.float32)


def _gpu_loss_grad(X, W, b, signs, y_ref, c, w_step, x_step, bits):
    T, K = X.shape
    N = W.shape[0]
    R = torch.empty(T, K, dtype=torch.float32, device=G.DEV)
    V = torch.empty(N, K, dtype=torch.float32, device=G.DEV)
    q.qvggt_rotate_rows(G.to_dev(X), G.to_dev(signs), R)
    q.qvggt_rotate_rows(G.to_dev(W), G.to_dev(signs), V)
    f = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(G.DEV)
    loss = torch.full((1,), float("nan"), dtype=torch.float32, device=G.DEV)
    gc = torch.full((K,), float("nan"), dtype=torch.float32, device=G.DEV)
    gw = torch.full((N,), float("nan"), dtype=torch.float32, device=G.DEV)
    gx = torch.full((1,), float("nan"), dtype=torch.float32, device=G.DEV) if x_step is not None else None
    xs = f(np.array([x_step])) if x_step is not None else None
    ws = torch.empty(q.qvggt_calib_workspace_bytes(T, N, K), dtype=torch.uint8, device=G.DEV)
    q.qvggt_calib_loss_grad(R, V, f(y_ref), G.to_dev(b), f(c), f(w_step), xs, bits, loss, gc, gw, gx, ws)
    torch.cuda.synchronize()
    return float(loss.item()), gc.cpu().numpy(), gw.cpu().numpy(), (None if gx is None else float(gx.item()))


@pytest.mark.parametrize("T,N,K,bits,static", [(1374, 3072, 1024, 4, False), (300, 144, 4096, 4, True), (257, 65, 128, 8, True),
                                               (70, 16, 1024, 6, False)])
def test_loss_and_derivatives(T, N, K, bits, static):
    """One frame of config 2's shape (dynamic per-token steps, the paper's default) and smaller ragged shapes with a static
    activation step and other widths, from the starting point of the offline half (Eq. "smooth_factor", absmax steps)."""
    X, W, b, signs, y_ref = _layer(T, N, K, T + N + K)
    a = oracle.rotated_col_absmax(X, pre_signs=signs)
    prep = oracle.prepare_weights(W, a, pre_signs=signs, bits=bits)
    c, w_step = prep.c_hat.astype(np.float32), (prep.dw * 0.9).astype(np.float32)       # steps a little below absmax: some clamping
    x_step = None
    if static:
        z = oracle.rotate(oracle.to_f64(X), signs) / c
        x_step = float(np.float32(np.quantile(np.abs(z), 0.999) / ((1 << (bits - 1)) - 1)))
    want = calib.reconstruction_loss_and_grads(X, W, y_ref, c, w_step, x_step=x_step, bias=b, pre_signs=signs, bits=bits)
    loss, gc, gw, gx = _gpu_loss_grad(X, W, b, signs, y_ref, c, w_step, x_step, bits)
    errs = dict(loss=abs(loss - want["loss"]) / want["loss"], grad_c=_rel(gc, want["grad_c"]), grad_w_step=_rel(gw, want["grad_w_step"]))
    if static:
        errs["grad_x_step"] = abs(gx - want["grad_x_step"]) / abs(want["grad_x_step"])
    G.report("calib_loss_grad", T=T, N=N, K=K, bits=bits, static=static, **errs)
    assert errs["loss"] <= 1e-3 and errs["grad_c"] <= 1e-2 and errs["grad_w_step"] <= 1e-2, errs
    assert not static or errs["grad_x_step"] <= 1e-2, errs
    # the same call again gives the same bits (fixed-order sums)
    loss2, gc2, gw2, _ = _gpu_loss_grad(X, W, b, signs, y_ref, c, w_step, x_step, bits)
    assert loss2 == loss and np.array_equal(gc2, gc) and np.array_equal(gw2, gw)


def test_descent_lowers_the_loss_and_deploys():
    """A few descent steps on the GPU from the offline starting point (step lengths normalised to the parameters' size, as in the
    oracle's check), the loss evaluated by the oracle before and after; the refined parameters go through
    qvggt_prep_weights_given and the layer still runs."""
    T, N, K = 700, 256, 1024
    X, W, b, signs, y_ref = _layer(T, N, K, 9)
    a = oracle.rotated_col_absmax(X, pre_signs=signs)
    prep = oracle.prepare_weights(W, a, pre_signs=signs)
    R = torch.empty(T, K, dtype=torch.float32, device=G.DEV)
    V = torch.empty(N, K, dtype=torch.float32, device=G.DEV)
    q.qvggt_rotate_rows(G.to_dev(X), G.to_dev(signs), R)
    q.qvggt_rotate_rows(G.to_dev(W), G.to_dev(signs), V)
    f = lambda v: torch.from_numpy(np.ascontiguousarray(v, dtype=np.float32)).to(G.DEV)
    c, w_step, yr = f(prep.c_hat), f(prep.dw), f(y_ref)
    loss = torch.zeros(1, dtype=torch.float32, device=G.DEV)
    gc, gw = torch.zeros(K, dtype=torch.float32, device=G.DEV), torch.zeros(N, dtype=torch.float32, device=G.DEV)
    ws = torch.empty(q.qvggt_calib_workspace_bytes(T, N, K), dtype=torch.uint8, device=G.DEV)
    losses = []
    for it in range(10):
        q.qvggt_calib_loss_grad(R, V, yr, G.to_dev(b), c, w_step, None, 4, loss, gc, gw, None, ws)
        losses.append(float(loss.item()))
        q.qvggt_calib_descent_step(c, gc, 0.02 * float(c.abs().mean()) / max(float(gc.abs().max()), 1e-30))
        q.qvggt_calib_descent_step(w_step, gw, 0.02 * float(w_step.mean()) / max(float(gw.abs().max()), 1e-30))
    assert min(losses[1:]) < losses[0]
    before = calib.reconstruction_loss_and_grads(X, W, y_ref, prep.c_hat, prep.dw, bias=b, pre_signs=signs)["loss"]
    after = calib.reconstruction_loss_and_grads(X, W, y_ref, c.cpu().numpy(), w_step.cpu().numpy(), bias=b, pre_signs=signs)["loss"]
    assert abs(losses[0] - before) <= 1e-4 * before
    G.report("calib_descent", loss_start=before, loss_after_10_steps=after, losses=[round(v, 6) for v in losses])
    assert after < before
    # deployment of the refined parameters: the given-parameter weight preparation and the ordinary online path
    Wq = torch.empty(N, K // 2, dtype=torch.uint8, device=G.DEV)
    sw, inv = torch.empty(N, dtype=torch.float32, device=G.DEV), torch.empty(K, dtype=torch.float32, device=G.DEV)
    q.qvggt_prep_weights_given(G.to_dev(W), c, G.to_dev(signs), w_step, 4, Wq, sw, inv)
    Y = torch.empty(T, N, dtype=torch.bfloat16, device=G.DEV)
    wsl = torch.empty(q.qvggt_workspace_bytes(T, N, K), dtype=torch.uint8, device=G.DEV)
    q.qvggt_linear(G.to_dev(X), G.to_dev(signs), inv, Wq, sw, G.to_dev(b), Y, wsl)
    p2 = oracle.prepare_weights_given(W, c.cpu().numpy().astype(np.float64), w_step.cpu().numpy().astype(np.float64), pre_signs=signs)
    want = oracle.linear(X, p2, bias=b, pre_signs=signs)
    assert G.rel_fro(G.bf16_bits(Y), want.Y) <= G.Y_REL_FRO
    # the deployed layer's error against the full-precision output is the loss that was minimised (up to the bf16 output rounding)
    got = oracle.bf16_bits_to_f64(G.bf16_bits(Y))
    assert abs(((got - y_ref) ** 2).sum() / T - after) <= 0.02 * after


def test_descent_step_floor_and_errors():
    th = torch.tensor([1.0, 1e-9, 0.5], dtype=torch.float32, device=G.DEV)
    g = torch.tensor([10.0, 1.0, -2.0], dtype=torch.float32, device=G.DEV)
    q.qvggt_calib_descent_step(th, g, calib.LR_STEP)
    assert np.allclose(th.cpu().numpy(), calib.descent_step([1.0, 1e-9, 0.5], [10.0, 1.0, -2.0], calib.LR_STEP), rtol=1e-6)
