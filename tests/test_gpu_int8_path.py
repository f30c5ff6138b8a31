"""GPU parity of the 8-bit and 6-bit settings (int8 codes, no nibble expansion in the GEMM) against the
oracle run with the same bit-width: codes, scales, exact accumulators and the final output, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import synth
import paper_2509_21302_amd as q
from tests import gpu_util as G

pytestmark = pytest.mark.gpu


def _heavy(rows, K, seed, dtype="bf16"):
    rng = np.random.default_rng(seed)
    x = rng.standard_t(3, (rows, K)).astype(np.float32)
    x[:, rng.choice(K, max(1, K // 100), replace=False)] *= 50
    x[: min(5, rows)] *= 20
    return synth.f32_to_bf16_bits(x) if dtype == "bf16" else x


@pytest.mark.parametrize("K", [128, 512, 1024, 2048, 4096, 8192])
def test_layout_is_the_packed_rows_permutation(K):
    """One byte per position, same positions as the 4-bit rows: checked against qvggt_pack_int4 / unpack, and inverted."""
    rng = np.random.default_rng(K)
    codes = rng.integers(-8, 8, (9, K)).astype(np.int8)
    lib = G.gpu_layout_int8(codes, 1)
    packed = G.gpu_pack(codes).cpu().numpy()
    lib_np = lib.cpu().numpy()
    lo = (packed & 0xF).astype(np.int8)
    hi = (packed >> 4).astype(np.int8)
    nib = np.stack([lo, hi], axis=2).reshape(9, K)
    nib = np.where(nib >= 8, nib - 16, nib)
    assert np.array_equal(lib_np, nib)
    assert np.array_equal(G.gpu_layout_int8(lib, 0).cpu().numpy(), codes)
    wide = rng.integers(-128, 128, (5, K)).astype(np.int8)
    assert np.array_equal(G.gpu_layout_int8(G.gpu_layout_int8(wide, 1), 0).cpu().numpy(), wide)


def _gemm(qx, qw, dx, dw, bias_bits, debug=True):
    M, K = qx.shape
    N = qw.shape[0]
    Xq, Wq = G.gpu_layout_int8(qx, 1), G.gpu_layout_int8(qw, 1)
    Y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=G.DEV)
    acc = torch.full((M, N), 12345, dtype=torch.int32, device=G.DEV) if debug else None
    q.qvggt_i8_gemm(Xq, G.to_dev(dx.astype(np.float32)), Wq, G.to_dev(dw.astype(np.float32)), G.to_dev(bias_bits), M, N, K, Y, acc)
    return (acc.cpu().numpy() if debug else None), G.bf16_bits(Y)


@pytest.mark.parametrize("M,N,K", [(64, 128, 128), (1, 16, 128), (300, 384, 256), (129, 144, 1024),
                                   (1374, 3072, 1024), (257, 1024, 4096), (33, 48, 8192), (10992, 1024, 4096)])
def test_i8_gemm_accumulators_bit_exact(M, N, K):
    rng = np.random.default_rng(M * 5 + N)
    qx = rng.integers(-128, 128, (M, K)).astype(np.int8)
    qw = rng.integers(-128, 128, (N, K)).astype(np.int8)
    dx = np.exp(rng.uniform(-3, 1, M)).astype(np.float32)
    dw = np.exp(rng.uniform(-8, -5, N)).astype(np.float32)
    bias_bits = synth.f32_to_bf16_bits((rng.standard_normal(N) * 0.02).astype(np.float32))
    acc, Y = _gemm(qx, qw, dx, dw, bias_bits)
    rows = np.unique(np.concatenate([np.arange(min(M, 40)), np.arange(max(M - 40, 0), M), rng.integers(0, M, 64)]))
    want = oracle.int_gemm(qx[rows], qw)
    assert np.array_equal(acc[rows], want)
    Yo = oracle.dequant_bias(want, dx[rows], dw, oracle.to_f64(bias_bits))
    ulp_off = np.abs(Y[rows].astype(np.int32) - Yo.astype(np.int32))
    assert ulp_off.max() <= 1 and (ulp_off != 0).mean() < 5e-3
    # the instantiation without the accumulator dump gives the same bf16 output bit for bit
    _, Y2 = _gemm(qx, qw, dx, dw, bias_bits, debug=False)
    assert np.array_equal(Y, Y2)


def test_i8_gemm_extreme_codes():
    M, N, K = 40, 32, 8192
    qx = np.full((M, K), -128, np.int8)
    qw = np.full((N, K), -128, np.int8)
    qw[1::2] = 127
    acc, Y = _gemm(qx, qw, np.ones(M), np.ones(N), None)
    assert np.array_equal(acc, oracle.int_gemm(qx, qw))
    assert acc.max() == 128 * 128 * K and acc.min() == -128 * 127 * K
    assert np.array_equal(Y, oracle.dequant_bias(acc, np.ones(M), np.ones(N)))


@pytest.mark.parametrize("bits", [8, 6])
@pytest.mark.parametrize("K", [128, 256, 1024, 2048, 4096, 8192])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_rotate_quant_i8(bits, K, dtype):
    rows = 37 if K >= 2048 else 203
    X = _heavy(rows, K, 500 + K + bits, dtype)
    rng = np.random.default_rng(K + bits)
    signs = (rng.integers(0, 2, K) * 2 - 1).astype(np.int8)
    c_hat = np.exp(rng.uniform(-1, 1, K))
    inv = (1.0 / (np.sqrt(K) * c_hat)).astype(np.float32)
    dx, qx, _ = oracle.rotate_smooth_quant(X, 1.0 / (inv.astype(np.float64) * np.sqrt(K)), pre_signs=signs, bits=bits)
    qmax = 2 ** (bits - 1) - 1
    assert qx.max() == qmax or qx.min() == -qmax
    Xq, sx = G.gpu_rsq_i8(G.to_dev(X), G.to_dev(signs), G.to_dev(inv), bits)
    G.check_codes(G.gpu_layout_int8(Xq, 0).cpu().numpy(), qx, f"K={K} bits={bits}")
    G.check_scales(sx.cpu().numpy(), dx, f"K={K} bits={bits}")


def test_rotate_quant_i8_zero_row():
    K = 1024
    X = _heavy(3, K, 9)
    X[1] = 0
    Xq, sx = G.gpu_rsq_i8(G.to_dev(X), None, None, 8)
    assert sx[1].item() == 0.0 and not Xq[1].any().item()
    dx, qx, _ = oracle.rotate_smooth_quant(X, bits=8)
    G.check_codes(G.gpu_layout_int8(Xq, 0).cpu().numpy(), qx)


@pytest.mark.parametrize("bits", [8, 6])
@pytest.mark.parametrize("config,name", [(1, "tiny"), (2, "qkv"), (3, "fc2")])
def test_prep_weights_i8(bits, config, name):
    s = synth.layer_spec(config, name)
    signs = synth.make_signs(s)
    W, Xc = synth.make_weights(s), synth.make_calibration(s)
    a = oracle.rotated_col_absmax(Xc, pre_signs=signs)
    po = oracle.prepare_weights(W, a, pre_signs=signs, alpha=0.5, bits=bits)
    pg = G.gpu_prep_i8(W, Xc, signs, bits)
    G.check_codes(G.gpu_layout_int8(pg["Wq"], 0).cpu().numpy(), po.qw, f"cfg{config} {name} bits={bits}")
    G.check_scales(pg["sw"].cpu().numpy(), po.dw)
    G.check_scales(pg["inv"].cpu().numpy(), 1.0 / (np.sqrt(s.K) * po.c_hat))


@pytest.mark.parametrize("bits", [8, 6])
@pytest.mark.parametrize("config,name", [(1, "tiny"), (2, "qkv"), (3, "fc1")])
def test_linear_i8_full_rows(bits, config, name):
    s = synth.layer_spec(config, name)
    X, bias = synth.make_activation_frames(s), synth.make_bias(s)
    signs = synth.make_signs(s)
    a = oracle.rotated_col_absmax(synth.make_calibration(s), pre_signs=signs)
    W = synth.make_weights(s)
    po = oracle.prepare_weights(W, a, pre_signs=signs, alpha=0.5, bits=bits)
    want = oracle.linear(X, po, bias=bias, pre_signs=signs, bits=bits)
    pg = G.gpu_prep_i8(W, synth.make_calibration(s), signs, bits)
    Y = G.bf16_bits(G.gpu_linear_i8(G.to_dev(X), pg, G.to_dev(bias)))
    err = G.rel_fro(Y, want.Y)
    assert err <= G.Y_REL_FRO, err
    # more bits, closer to the exact product: the error against full precision shrinks with the step
    exact = oracle.to_f64(X[:256]) @ oracle.to_f64(W).T + (0 if bias is None else oracle.to_f64(bias))
    got = oracle.bf16_bits_to_f64(Y[:256])
    assert np.linalg.norm(got - exact) / np.linalg.norm(exact) < (0.03 if bits == 8 else 0.1)


@pytest.mark.parametrize("w_bits,a_bits", [(4, 8), (8, 4), (6, 8), (4, 4)])
@pytest.mark.parametrize("config,name", [(2, "qkv"), (3, "fc1")])
def test_mixed_widths(w_bits, a_bits, config, name):
    """Mixed precision (appendix, further settings): weights and activations of different widths through the int8-code
    path, against the oracle run with the same two widths.  (4, 4) in int8 containers must equal the packed 4-bit path
    bit for bit: same codes, same integer sums, same epilogue."""
    s = synth.layer_spec(config, name)
    X, bias = synth.make_activation_frames(s), synth.make_bias(s)
    signs = synth.make_signs(s)
    cal = synth.make_calibration(s)
    W = synth.make_weights(s)
    po = oracle.prepare_weights(W, oracle.rotated_col_absmax(cal, pre_signs=signs), pre_signs=signs, alpha=0.5, bits=w_bits)
    want = oracle.linear(X, po, bias=bias, pre_signs=signs, bits=a_bits)
    pg = G.gpu_prep_i8(W, cal, signs, w_bits)
    pg["bits"] = a_bits                                   # gpu_linear_i8 quantizes the activations with pg["bits"]
    Yd = G.gpu_linear_i8(G.to_dev(X), pg, G.to_dev(bias))
    assert G.rel_fro(G.bf16_bits(Yd), want.Y) <= G.Y_REL_FRO
    if (w_bits, a_bits) == (4, 4):
        p4 = G.gpu_prep(W, cal, signs)
        assert torch.equal(G.gpu_linear(G.to_dev(X), p4, G.to_dev(bias)), Yd)
        codes = torch.empty_like(pg["Wq"])
        G.q.qvggt_layout_int8(pg["Wq"], codes, 0)
        assert np.array_equal(codes.cpu().numpy(), G.gpu_unpack(p4["Wq"], s.K))


@pytest.mark.parametrize("name,n_random", [("fc1", 800), ("fc2", 300)])
def test_linear_i8_full_size_sampled_rows(name, n_random):
    """The benchmark's shapes (137400 tokens) at 8 bits; the oracle recomputes a seeded sample of rows."""
    s = synth.layer_spec(5, name)
    rng = np.random.default_rng(len(name))
    rows = np.unique(np.concatenate([np.arange(synth.SPECIAL_TOKENS), np.arange(s.M - 64, s.M), rng.choice(s.M, n_random, replace=False)]))
    signs = synth.make_signs(s)
    W, Xc, bias = synth.make_weights(s), synth.make_calibration(s), synth.make_bias(s)
    po = oracle.prepare_weights(W, oracle.rotated_col_absmax(Xc, pre_signs=signs), pre_signs=signs, alpha=0.5, bits=8)
    pg = G.gpu_prep_i8(W, Xc, signs, 8)
    X = synth.make_activation_frames(s)
    Xd = G.to_dev(X)
    Xs = X[rows]
    del X
    want = oracle.linear(Xs, po, bias=bias, pre_signs=signs, bits=8)
    idx = torch.from_numpy(rows).to(G.DEV)
    Yd = G.gpu_linear_i8(Xd, pg, G.to_dev(bias))
    err = G.rel_fro(G.bf16_bits(Yd[idx]), want.Y)
    assert err <= G.Y_REL_FRO, err
    del Yd
    Xq, sx = G.gpu_rsq_i8(Xd, pg["signs"], pg["inv"], 8)
    G.check_codes(G.gpu_layout_int8(Xq[idx].contiguous(), 0).cpu().numpy(), want.qx, name)
    G.check_scales(sx[idx].cpu().numpy(), want.dx, name)
    # exact accumulators of the sampled rows, from the GPU's own codes (both operands in library order)
    acc = torch.empty(len(rows), s.N, dtype=torch.int32, device=G.DEV)
    Ys = torch.empty(len(rows), s.N, dtype=torch.bfloat16, device=G.DEV)
    q.qvggt_i8_gemm(Xq[idx].contiguous(), sx[idx].contiguous(), pg["Wq"], pg["sw"], None, len(rows), s.N, s.K, Ys, acc)
    qx_g = G.gpu_layout_int8(Xq[idx].contiguous(), 0).cpu().numpy()
    qw_g = G.gpu_layout_int8(pg["Wq"], 0).cpu().numpy()
    assert np.array_equal(acc.cpu().numpy(), oracle.int_gemm(qx_g, qw_g))
