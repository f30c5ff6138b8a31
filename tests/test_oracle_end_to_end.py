"""The oracle's whole quantized linear on the synthetic configs: structural and error-budget checks.

The paper prints no worked example, so absolute end-to-end values are unpinned; what is
checked here is what the paper states qualitatively (rotation and smoothing each reduce
the W4A4 error on heavy-tailed inputs: architecture ablation table) and exact invariants.
"""
import os

import numpy as np
import pytest

import oracle
import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rel_fro(a, b):
    return np.linalg.norm(a - b) / np.linalg.norm(b)


def _naive_w4a4(X, W):
    dx, qx = oracle.quantize_rows(X, 4)
    dw, qw = oracle.quantize_rows(W, 4)
    return oracle.int_gemm(qx, qw) * dx[:, None] * dw[None, :]


@pytest.fixture(scope="module")
def cfg1():
    s = synth.layer_spec(1)
    return s, oracle.to_f64(synth.make_activation_frames(s)), oracle.to_f64(synth.make_weights(s)), synth.make_signs(s)


def test_config1_error_ordering(cfg1):
    s, X, W, u = cfg1
    exact = X @ W.T
    e_naive = _rel_fro(_naive_w4a4(X, W), exact)
    # rotation only
    prep_r = oracle.prepare_weights(W, None, pre_signs=u)
    e_rot = _rel_fro(oracle.linear(X, prep_r, pre_signs=u).y, exact)
    # rotation + post-rotation smoothing (the full method), calibrated on X itself
    a = oracle.rotated_col_absmax(X, pre_signs=u)
    prep = oracle.prepare_weights(W, a, pre_signs=u, alpha=0.5)
    e_dsfq = _rel_fro(oracle.linear(X, prep, pre_signs=u).y, exact)
    assert e_naive > e_rot > e_dsfq, (e_naive, e_rot, e_dsfq)
    assert e_dsfq < 0.25


def test_post_signs_leave_accumulators_unchanged(cfg1):
    # H = Hhat diag(v): the signs flip matching columns of both operands, so the integer sums are identical
    s, X, W, u = cfg1
    a0 = oracle.rotated_col_absmax(X)
    r0 = oracle.linear(X, oracle.prepare_weights(W, a0))
    av = oracle.rotated_col_absmax(X, post_signs=u)
    rv = oracle.linear(X, oracle.prepare_weights(W, av, post_signs=u), post_signs=u)
    assert np.array_equal(r0.acc, rv.acc)
    assert np.array_equal(r0.Y, rv.Y)
    assert np.array_equal(rv.qx, r0.qx * u[None, :])
    # pre-rotation signs do change the codes (the seed matters, as the paper's seed ablation shows)
    ru = oracle.linear(X, oracle.prepare_weights(W, oracle.rotated_col_absmax(X, pre_signs=u), pre_signs=u), pre_signs=u)
    assert not np.array_equal(ru.acc, r0.acc)


def test_quantized_product_error_budget(cfg1):
    # |y - exact| is bounded through the per-element quantizer bounds:
    # xs = dx*qx + ex, ws = dw*qw + ew with |ex| <= dx/2, |ew| <= dw/2
    s, X, W, u = cfg1
    a = oracle.rotated_col_absmax(X, pre_signs=u)
    prep = oracle.prepare_weights(W, a, pre_signs=u)
    res = oracle.linear(X, prep, pre_signs=u)
    dx, qx, Xs = oracle.rotate_smooth_quant(X, prep.c_hat, pre_signs=u)
    exact = X @ W.T
    bound = (dx[:, None] / 2) * np.abs(prep.Ws).sum(axis=1)[None, :] \
        + (np.abs(Xs).sum(axis=1)[:, None]) * (prep.dw[None, :] / 2) \
        + s.K * (dx[:, None] / 2) * (prep.dw[None, :] / 2)
    assert np.all(np.abs(res.y - exact) <= bound * (1 + 1e-9) + 1e-9)
    assert np.abs(res.acc).max() <= 49 * s.K


def test_zero_row_gives_bias(cfg1):
    s, X, W, u = cfg1
    X2 = X.copy()
    X2[3] = 0.0
    prep = oracle.prepare_weights(W, oracle.rotated_col_absmax(X, pre_signs=u), pre_signs=u)
    bias = np.linspace(-1, 1, s.N)
    res = oracle.linear(X2, prep, bias=bias, pre_signs=u)
    assert res.dx[3] == 0.0 and not res.qx[3].any()
    assert np.array_equal(res.Y[3], oracle.bf16_from_f64(bias))


def test_config2_shape_statistics_and_dispersal():
    # the synthetic qkv input has the structure the paper describes (salient first five tokens,
    # outlier channels, heavy tails), and the rotation removes the channel outliers
    s = synth.layer_spec(2)
    Xb = synth.make_activation_rows(s, list(range(0, 64)))
    X = oracle.to_f64(Xb)
    ch = synth.outlier_channels(s)
    assert len(ch) == 10
    body = np.delete(X[5:], ch, axis=1)
    assert np.abs(X[:5]).mean() > 10 * np.abs(body).mean()
    assert np.abs(X[5:, ch]).mean() > 20 * np.abs(body).mean()
    u = synth.make_signs(s)
    Xr = oracle.rotate(X, pre_signs=u)
    kurt = lambda r: np.mean((r - r.mean()) ** 4) / np.var(r) ** 2
    assert np.median([kurt(r) for r in X[5:]]) > 20
    assert np.median([kurt(r) for r in Xr[5:]]) < 6          # close to Gaussian (3): Lemma 1


def test_config1_golden_digest(cfg1):
    """Drift detector: the committed digest was written by tests/golden/make_golden.py from the oracle alone."""
    from tests.golden.make_golden import config1_digest
    want = open(os.path.join(GOLD, "config1_oracle.txt")).read()
    assert config1_digest() == want
