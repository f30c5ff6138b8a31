"""GPU parity of the offline half with calibrated parameters handed in (qvggt_prep_weights_given) against
oracle.prepare_weights_given, and of the deployed layer (given factor, given weight steps, given activation step) end to end."""
import numpy as np
import pytest
import torch

import oracle
import synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu


def _learned(s, seed, shrink):
    """Stand-ins for calibrated values: the closed-form factor perturbed per channel, the channels' own steps shrunk (clamp live)."""
    rng = np.random.default_rng(seed)
    signs = synth.make_signs(s)
    W = synth.make_weights(s)
    base = oracle.prepare_weights(W, oracle.rotated_col_absmax(synth.make_calibration(s), pre_signs=signs), pre_signs=signs)
    c_hat = (base.c_hat * np.exp(rng.normal(0, 0.2, s.K))).astype(np.float32)
    own = oracle.prepare_weights_given(W, c_hat, None, pre_signs=signs)
    w_step = (own.dw * rng.uniform(shrink, 1.0, s.N)).astype(np.float32) if shrink else None
    return W, signs, c_hat, w_step


def _gpu_given(W, c_hat, signs, w_step, bits):
    Wd = G.to_dev(W)
    N, K = Wd.shape
    Wq = torch.full((N, K // 2 if bits == 4 else K), 0x5A, dtype=torch.uint8, device=G.DEV)
    sw = torch.empty(N, dtype=torch.float32, device=G.DEV)
    inv = torch.empty(K, dtype=torch.float32, device=G.DEV)
    G.q.qvggt_prep_weights_given(Wd, G.to_dev(c_hat), G.to_dev(signs), G.to_dev(w_step), bits, Wq, sw, inv)
    return Wq, sw, inv


@pytest.mark.parametrize("config,name", [(1, "tiny"), (2, "qkv"), (3, "fc2")])
@pytest.mark.parametrize("bits,shrink", [(4, 0.6), (4, 0.0), (8, 0.6), (6, 0.0)])
def test_prep_weights_given(config, name, bits, shrink):
    s = synth.layer_spec(config, name)
    W, signs, c_hat, w_step = _learned(s, 40 + config, shrink)
    if bits != 4 and w_step is not None:
        w_step = (w_step * 7.0 / (2 ** (bits - 1) - 1)).astype(np.float32)        # the same clipping ratio on the finer grid
    want = oracle.prepare_weights_given(W, c_hat, w_step, pre_signs=signs, bits=bits)
    Wq, sw, inv = _gpu_given(W, c_hat, signs, w_step, bits)
    G.check_scales(inv.cpu().numpy(), 1.0 / (np.sqrt(s.K) * c_hat.astype(np.float64)), "inv_smooth")
    codes = G.gpu_unpack(Wq, s.K) if bits == 4 else G.gpu_layout_int8(Wq.view(torch.int8), 0).cpu().numpy()
    G.check_codes(codes, want.qw, f"{name} bits={bits}")
    if w_step is not None:
        assert np.array_equal(sw.cpu().numpy(), w_step)                             # given steps are handed on as they are
        top = 2 ** (bits - 1) - 1
        assert (want.qw == -top - 1).any() and (codes == -top - 1).any()            # the clamp at the negative end is exercised
    else:
        G.check_scales(sw.cpu().numpy(), want.dw, "w_scale")


def test_prep_weights_given_without_factor_equals_rotation_only():
    s = synth.layer_spec(2)
    W, signs = synth.make_weights(s), synth.make_signs(s)
    Wq, sw, inv = _gpu_given(W, None, signs, None, 4)
    g = G.gpu_prep(W, None, signs)
    assert torch.equal(Wq, g["Wq"]) and torch.equal(sw, g["sw"]) and torch.equal(inv, g["inv"])


def test_deployed_layer_with_given_parameters():
    """Config 2 with every calibrated quantity handed in: factor, weight steps, one tensor-wise activation step; both sides
    run qvggt / oracle from the same parameters, the GEMM is the unchanged one."""
    s = synth.layer_spec(2)
    W, signs, c_hat, w_step = _learned(s, 77, 0.8)
    X, bias = synth.make_activation_frames(s), synth.make_bias(s)
    po = oracle.prepare_weights_given(W, c_hat, w_step, pre_signs=signs)
    _, _, Z = oracle.rotate_smooth_quant(X, po.c_hat, pre_signs=signs)
    x_step = np.array([np.percentile(np.abs(Z), 99.95) / 7.0], dtype=np.float32)
    qx = oracle.quantize_rows_static(Z, np.full(s.M, float(x_step[0])), 4)
    want = oracle.dequant_bias(oracle.int_gemm(qx, po.qw), np.full(s.M, float(x_step[0])), po.dw, oracle.to_f64(bias))
    Wq, sw, inv = _gpu_given(W, c_hat, signs, w_step, 4)
    Xq, sx = G.gpu_rsq_static(G.to_dev(X), G.to_dev(signs), inv, G.to_dev(x_step), 0)
    Y = torch.empty(s.M, s.N, dtype=torch.bfloat16, device=G.DEV)
    G.q.qvggt_w4a4_gemm(Xq, sx, Wq, sw, G.to_dev(bias), s.M, s.N, s.K, Y)
    assert G.rel_fro(G.bf16_bits(Y), want) <= G.Y_REL_FRO
