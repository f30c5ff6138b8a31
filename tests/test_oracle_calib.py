"""Pins of oracle/calib.py (the reconstruction loss of one layer and its straight-through derivatives): a layer worked by
hand, the cancellation of the two paths of the smoothing factor when nothing is rounded, finite differences where the loss
is smooth (everything clamped: the quantized values are linear in their steps), and a descent check on a synthetic layer."""
import numpy as np

import oracle
from oracle import calib


def test_fake_quantize_values_and_rules():
    v = np.array([[0.0, 1.0, -1.26, 2.5, 100.0, -100.0]])
    y, inside, ds = calib.fake_quantize(v, 0.5, bits=4)
    assert y[0].tolist() == [0.0, 1.0, -1.5, 2.5, 3.5, -4.0]               # u = 0, 2, -2.52 -> -3, 5, clamp 7, clamp -8
    assert inside[0].tolist() == [True, True, True, True, False, False]
    assert np.allclose(ds[0], [0.0, 0.0, -3 + 2.52, 0.0, 7.0, -8.0])
    y, inside, ds = calib.fake_quantize(v, np.array([0.0]), bits=4)          # a dead step: nothing
    assert not y.any() and not inside.any() and not ds.any()
    # the clamp is judged on the rounded code: 7.4 rounds to 7 and is inside, 7.6 rounds to 8 and is clamped, and a row's own
    # absmax step puts its largest element inside however 7 * (x / x) rounds
    y, inside, ds = calib.fake_quantize(np.array([[7.4, 7.6, -8.4, -8.6]]), 1.0, bits=4)
    assert y[0].tolist() == [7.0, 7.0, -8.0, -8.0] and inside[0].tolist() == [True, False, True, False]
    assert np.allclose(ds[0], [7 - 7.4, 7.0, -8 + 8.4, -8.0])
    for x in (0.1, 1 / 3, 2.7e-5, 123.456):
        _, inside, _ = calib.fake_quantize(np.array([[x, -x]]), np.array([x / 7]), bits=4)
        assert inside.all()
    # per-row steps
    y, _, _ = calib.fake_quantize(np.array([[1.0, 2.0], [1.0, 2.0]]), np.array([1.0, 0.8]), bits=4)
    assert np.allclose(y, [[1.0, 2.0], [0.8, 1.6]])                          # 1.25 -> 1, 2.5 -> 2 (ties to even)


def test_layer_worked_by_hand():
    """T = 1, N = 1, K = 4.  X = [1, 1, 1, 1] rotates to [2, 0, 0, 0] and W = [.5, .5, .5, .5] to [1, 0, 0, 0] (first Hadamard
    row all +1/2).  c = [2, 1, 1, 1]: z = [1, 0, 0, 0], v = [2, 0, 0, 0].  Static activation step 0.4: u = 2.5 -> 2 (tie to even),
    x_hat = 0.8, d x_hat / d step = 2 - 2.5 = -0.5.  Weight step 0.3: u = 6.667 -> 7, w_hat = 2.1, d w_hat / d step = 1/3.
    y_q = 1.68 against y_ref = 2: E = -0.32, L = 0.1024, G = -0.64; dL/dx_hat = -1.344, dL/dw_hat = -0.512."""
    X = np.ones((1, 4)); W = np.full((1, 4), 0.5)
    r = calib.reconstruction_loss_and_grads(X, W, np.array([[2.0]]), np.array([2.0, 1, 1, 1]), np.array([0.3]), x_step=0.4)
    assert abs(r["y_q"][0, 0] - 1.68) < 1e-12 and abs(r["loss"] - 0.1024) < 1e-12
    assert abs(r["grad_w_step"][0] - (-0.512 / 3)) < 1e-12
    assert abs(r["grad_x_step"] - 0.672) < 1e-12
    # c_0: through the weights -0.512 * 1 (d v / d c = V), through the activations -1.344 * (-z / c) = +0.672
    assert np.allclose(r["grad_c"], [0.16, 0, 0, 0], atol=1e-12)
    # the same layer with the dynamic step: step = 1 / 7, z / step = 7 exactly, x_hat = 1: y_q = 2.1, E = 0.1
    r = calib.reconstruction_loss_and_grads(X, W, np.array([[2.0]]), np.array([2.0, 1, 1, 1]), np.array([0.3]))
    assert abs(r["y_q"][0, 0] - 2.1) < 1e-12 and abs(r["loss"] - 0.01) < 1e-12 and r["grad_x_step"] is None
    assert abs(r["grad_w_step"][0] - 0.2 * 1.0 / 3) < 1e-12                   # G = 0.2, dL/dw_hat = 0.2 * x_hat
    assert np.allclose(r["grad_c"], [0.2 * 1.0 * 1.0 + 0.2 * 2.1 * (-0.5), 0, 0, 0], atol=1e-12)
    # a bias shifts y_q and nothing else
    rb = calib.reconstruction_loss_and_grads(X, W, np.array([[2.0]]), np.array([2.0, 1, 1, 1]), np.array([0.3]), bias=np.array([-0.1]))
    assert abs(rb["y_q"][0, 0] - 2.0) < 1e-12 and rb["loss"] < 1e-24


def _layer(T, N, K, seed):
    rng = np.random.default_rng(seed)
    X = rng.standard_t(3, (T, K))
    X[:, rng.choice(K, 2, replace=False)] *= 30
    W = rng.standard_normal((N, K)) * 0.05
    signs = np.where(rng.random(K) < 0.5, -1, 1).astype(np.int8)
    y_ref = X @ W.T + rng.standard_normal((T, N)) * 0.01
    return X, W, signs, y_ref


def test_without_rounding_the_smoothing_factor_cancels():
    """(R / c)(V c)^T = R V^T whatever c is: with the rounding left out and nothing clamped, the loss does not depend on c and
    the two paths of its derivative cancel term by term; the steps do not matter either.  A sign or index slip in either path shows here."""
    X, W, signs, y_ref = _layer(24, 12, 64, 0)
    rng = np.random.default_rng(1)
    c = np.exp(rng.uniform(-1, 1, 64))
    big = 1e3                                            # steps so that |u| stays far below the clamp... no: u must stay inside [-8, 7]
    z = oracle.rotate(X, signs) / c
    v = oracle.rotate(W, signs) * c
    w_step = np.abs(v).max(axis=1) / 6.9
    x_step = float(np.abs(z).max() / 6.9)
    r = calib.reconstruction_loss_and_grads(X, W, y_ref, c, w_step, x_step=x_step, pre_signs=signs, rounding=False)
    E = X @ W.T - y_ref
    assert abs(r["loss"] - (E ** 2).sum() / 24) < 1e-9 * r["loss"]
    assert np.abs(r["grad_c"]).max() < 1e-9 * np.abs(E).max()
    assert np.abs(r["grad_w_step"]).max() < 1e-12 and abs(r["grad_x_step"]) < 1e-12


def test_finite_differences_where_everything_is_clamped():
    """Steps so small that every value sits on a clamp bound: the quantized values are step * (-8 or 7), the loss is a smooth
    (quadratic) function of the steps and does not depend on c at all."""
    X, W, signs, y_ref = _layer(16, 8, 32, 2)
    rng = np.random.default_rng(3)
    c = np.exp(rng.uniform(-0.5, 0.5, 32))
    z = oracle.rotate(X, signs) / c
    v = oracle.rotate(W, signs) * c
    assert np.abs(z).min() > 1e-6 and np.abs(v).min() > 1e-6
    w_step = np.full(8, np.abs(v).min() / 20) * np.exp(rng.uniform(0, 0.3, 8))
    x_step = float(np.abs(z).min() / 20)
    f = lambda ws, xs, cc: calib.reconstruction_loss_and_grads(X, W, y_ref, cc, ws, x_step=xs, pre_signs=signs)
    r = f(w_step, x_step, c)
    assert np.abs(r["grad_c"]).max() == 0.0
    for o in range(8):
        h = w_step[o] * 1e-2           # the loss is quadratic in a step here: a central difference is exact at any width
        e = np.zeros(8); e[o] = h
        fd = (f(w_step + e, x_step, c)["loss"] - f(w_step - e, x_step, c)["loss"]) / (2 * h)
        assert abs(fd - r["grad_w_step"][o]) <= 1e-6 * abs(fd) + 1e-7 * np.abs(r["grad_w_step"]).max()     # differences of O(1) losses: absolute roundoff
    h = x_step * 1e-2
    fd = (f(w_step, x_step + h, c)["loss"] - f(w_step, x_step - h, c)["loss"]) / (2 * h)
    assert abs(fd - r["grad_x_step"]) <= 1e-6 * abs(fd)
    assert f(w_step, x_step, c * 1.01)["loss"] == r["loss"]


def test_descent_on_a_heavy_tailed_layer_lowers_the_loss():
    """Start from what the offline half computes (Eq. "smooth_factor" with alpha = 0.5, absmax steps) and take steps of plain
    gradient descent: the straight-through derivative is a descent direction in practice; with step lengths normalised to the
    parameters' size the loss goes down over a few updates (a qualitative check: the paper prints no numbers for this)."""
    X, W, signs, _ = _layer(96, 48, 128, 4)
    y_ref = X @ W.T
    a = oracle.rotated_col_absmax(X, pre_signs=signs)
    prep = oracle.prepare_weights(W, a, pre_signs=signs)
    c, w_step = prep.c_hat.copy(), prep.dw.copy()
    losses = []
    for it in range(12):
        r = calib.reconstruction_loss_and_grads(X, W, y_ref, c, w_step, pre_signs=signs)
        losses.append(r["loss"])
        gc, gw = r["grad_c"], r["grad_w_step"]
        c = calib.descent_step(c, gc, 0.02 * np.abs(c).mean() / max(np.abs(gc).max(), 1e-30))
        w_step = calib.descent_step(w_step, gw, 0.02 * w_step.mean() / max(np.abs(gw).max(), 1e-30))
    assert min(losses[1:]) < losses[0]
    assert np.all(c > 0) and np.all(w_step > 0)
    assert np.array_equal(calib.descent_step(np.array([1.0, 1e-9]), np.array([10.0, 1.0]), calib.LR_STEP), [0.5, 1e-8])
