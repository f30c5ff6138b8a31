"""GPU parity of online kernel 1 (rotate, smooth, per-token quantize) and of the offline weight
preparation against the CPU oracle, element by element, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu


def _heavy(rows, K, seed, dtype="bf16"):
    rng = np.random.default_rng(seed)
    x = rng.standard_t(3, (rows, K)).astype(np.float32)
    x[:, rng.choice(K, max(1, K // 100), replace=False)] *= 50
    x[: min(5, rows)] *= 20
    return synth.f32_to_bf16_bits(x) if dtype == "bf16" else x


@pytest.mark.parametrize("K", [128, 256, 512, 1024, 2048, 4096, 8192])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_rotate_quant_all_sizes(K, dtype):
    rows = 37 if K >= 2048 else 203          # ragged: not a multiple of the rows a block takes
    X = _heavy(rows, K, 100 + K, dtype)
    rng = np.random.default_rng(K)
    signs = (rng.integers(0, 2, K) * 2 - 1).astype(np.int8)
    c_hat = np.exp(rng.uniform(-1, 1, K))
    inv = (1.0 / (np.sqrt(K) * c_hat)).astype(np.float32)
    dx, qx, _ = oracle.rotate_smooth_quant(X, 1.0 / (inv.astype(np.float64) * np.sqrt(K)), pre_signs=signs)
    Xq, sx = G.gpu_rsq(G.to_dev(X), G.to_dev(signs), G.to_dev(inv))
    G.check_codes(G.gpu_unpack(Xq, K), qx, f"K={K}")
    G.check_scales(sx.cpu().numpy(), dx, f"K={K}")


@pytest.mark.parametrize("K", [128, 1024, 4096])
@pytest.mark.parametrize("per_token", [1, 0])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_rotate_quant_static_step(K, per_token, dtype):
    """A calibrated step instead of the row's own absmax: token-wise (one per row) or tensor-wise (one value).
    The steps are drawn below each row's dynamic step so that part of every row saturates at -8 / 7."""
    rows = 37 if K >= 2048 else 203
    X = _heavy(rows, K, 300 + K, dtype)
    rng = np.random.default_rng(K + per_token)
    signs = (rng.integers(0, 2, K) * 2 - 1).astype(np.int8)
    c_hat = np.exp(rng.uniform(-1, 1, K))
    inv = (1.0 / (np.sqrt(K) * c_hat)).astype(np.float32)
    dyn, _, Z = oracle.rotate_smooth_quant(X, 1.0 / (inv.astype(np.float64) * np.sqrt(K)), pre_signs=signs)
    if per_token:
        step = (dyn * rng.uniform(0.2, 1.5, rows)).astype(np.float32)
    else:
        step = np.array([np.median(dyn) * 0.5], dtype=np.float32)
    want = oracle.quantize_rows_static(Z, np.broadcast_to(step.astype(np.float64), (rows,)), 4)
    assert (want == 7).any() and (want == -8).any()          # the clamp is exercised
    Xq, sx = G.gpu_rsq_static(G.to_dev(X), G.to_dev(signs), G.to_dev(inv), G.to_dev(step), per_token)
    G.check_codes(G.gpu_unpack(Xq, K), want, f"K={K} per_token={per_token}")
    assert np.array_equal(sx.cpu().numpy(), np.broadcast_to(step, (rows,)))


# LayerNorm fused in front.  With f32 rows nothing is rounded between the normalisation and the rotation and the usual
# bars hold.  With bf16 rows the normalised value is rounded to bf16, and the kernel's fp32 value (relative error about
# 2e-7) lands on the other side of a rounding midpoint (spaced 2^-8 .. 2^-7 relative) than the oracle's fp64 value for about
# 5e-5 of the elements.  Such an element then differs by one bf16 ulp, every rotated value of its row moves by up to
# ulp / sqrt(K), and a row that holds one can see a few codes and its step move.  Measured over the cases below (the
# figures go to the measured-values log on every run): a code off by one on at most 2.9e-5 of the elements (4.7e-6 at
# the 1031-row case), the worst step 2.2e-4 off, 98.5 % of the steps within 1e-5 in the worst case (one row of 67).  The
# bars sit a factor of about four above those: 1e-4 of the codes, 1e-3 on every step, 95 % of the steps within 1e-5.
LN_BF16_CODE_FRACTION = 1e-4
LN_BF16_SCALE_RTOL_ALL = 1e-3
LN_BF16_STEPS_EXACT = 0.95


def _check_ln(Xq, sx, K, qx, dx, dtype, what):
    codes, got = G.gpu_unpack(Xq, K), sx.cpu().numpy().astype(np.float64)
    if dtype == "f32":
        G.check_codes(codes, qx, what)
        G.check_scales(got, dx, what)
        return
    d = np.abs(codes.astype(np.int16) - qx.astype(np.int16))
    assert d.max(initial=0) <= 1, f"{what}: a code differs by {d.max()}"
    assert (d != 0).mean() <= LN_BF16_CODE_FRACTION, f"{what}: {(d != 0).mean():.3e} of the codes differ"
    err = np.abs(got - dx) / np.maximum(dx, 1e-300)
    err[dx == 0] = np.abs(got[dx == 0])
    G.report("layernorm_fused_bf16", what=what, rows=int(codes.shape[0]), code_mismatch_fraction=float((d != 0).mean()),
             step_err_max=float(err.max(initial=0)), steps_within_1e5=float((err <= G.SCALE_RTOL).mean()))
    assert err.max(initial=0) <= LN_BF16_SCALE_RTOL_ALL, f"{what}: step rel err {err.max():.3e}"
    assert (err <= G.SCALE_RTOL).mean() >= LN_BF16_STEPS_EXACT, f"{what}: only {(err <= G.SCALE_RTOL).mean():.2f} of the steps within {G.SCALE_RTOL}"


@pytest.mark.parametrize("K", [128, 512, 1024, 2048, 4096])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_layernorm_rotate_quant(K, dtype):
    """LayerNorm -> rotation -> smoothing -> per-token codes in one launch against the oracle's LayerNorm followed by
    its rotate_smooth_quant.  K = 1024 bf16 is the matrix-core kernel (VGGT's qkv and fc1 inputs), the rest the generic one."""
    rows = 1031 if K == 1024 else (37 if K >= 2048 else 203)
    X = _heavy(rows, K, 500 + K, dtype)
    rng = np.random.default_rng(K + 5)
    signs = (rng.integers(0, 2, K) * 2 - 1).astype(np.int8)
    c_hat = np.exp(rng.uniform(-1, 1, K))
    inv = (1.0 / (np.sqrt(K) * c_hat)).astype(np.float32)
    gamma = np.exp(rng.normal(0, 0.3, K)).astype(np.float32)
    beta = rng.normal(0, 0.1, K).astype(np.float32)
    eps = 1e-5
    Yn = oracle.layernorm(X, gamma, beta, eps, round_to_bf16=(dtype == "bf16"))
    dx, qx, _ = oracle.rotate_smooth_quant(Yn, 1.0 / (inv.astype(np.float64) * np.sqrt(K)), pre_signs=signs)
    Xq, sx = G.gpu_ln_rsq(G.to_dev(X), G.to_dev(gamma), G.to_dev(beta), eps, G.to_dev(signs), G.to_dev(inv))
    _check_ln(Xq, sx, K, qx, dx, dtype, f"K={K} {dtype}")


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_layernorm_rotate_quant_optional_and_degenerate(dtype):
    """No gamma / beta / signs / smoothing; a constant row (variance 0) normalises to zeros: step 0, codes 0; one row."""
    K, rows, eps = 1024, 67, 1e-6
    X = _heavy(rows, K, 77, dtype)
    X[3] = X[3, 0]
    Yn = oracle.layernorm(X, None, None, eps, round_to_bf16=(dtype == "bf16"))
    assert not Yn[3].any()
    dx, qx, _ = oracle.rotate_smooth_quant(Yn)
    Xq, sx = G.gpu_ln_rsq(G.to_dev(X), None, None, eps, None, None)
    _check_ln(Xq, sx, K, qx, dx, dtype, dtype)
    assert sx[3].item() == 0.0 and not G.gpu_unpack(Xq, K)[3].any()
    Xq1, sx1 = G.gpu_ln_rsq(G.to_dev(X[:1]), None, None, eps, None, None)
    assert torch.equal(Xq1, Xq[:1]) and torch.equal(sx1, sx[:1])
    # only beta: a constant row becomes beta itself
    beta = np.random.default_rng(3).normal(0, 1, K).astype(np.float32)
    Yb = oracle.layernorm(X[3:4], None, beta, eps, round_to_bf16=(dtype == "bf16"))
    dxb, qxb, _ = oracle.rotate_smooth_quant(Yb)
    Xqb, sxb = G.gpu_ln_rsq(G.to_dev(X[3:4]), None, G.to_dev(beta), eps, None, None)
    G.check_codes(G.gpu_unpack(Xqb, K), qxb)
    G.check_scales(sxb.cpu().numpy(), dxb)


def test_layernorm_rotate_quant_feeds_the_gemm():
    """End to end: the fused kernel's codes and steps through the integer GEMM against the oracle's LayerNorm + layer."""
    K, N, rows, eps = 1024, 512, 700, 1e-5
    rng = np.random.default_rng(21)
    X = _heavy(rows, K, 22)
    W = rng.standard_normal((N, K)).astype(np.float32) * 0.05
    bias = synth.f32_to_bf16_bits(rng.normal(0, 0.1, N).astype(np.float32))
    gamma = np.exp(rng.normal(0, 0.3, K)).astype(np.float32)
    beta = rng.normal(0, 0.1, K).astype(np.float32)
    signs = synth.make_signs(synth.layer_spec(2))[:K]
    Yn = oracle.layernorm(X, gamma, beta, eps)
    act = oracle.rotated_col_absmax(Yn, pre_signs=signs)
    prep_o = oracle.prepare_weights(W, act, pre_signs=signs)
    want = oracle.linear(Yn, prep_o, bias, pre_signs=signs).Y
    prep = G.gpu_prep(W, synth.f32_to_bf16_bits(Yn.astype(np.float32)), signs)      # calibrate on the oracle's normalised rows
    Xq, sx = G.gpu_ln_rsq(G.to_dev(X), G.to_dev(gamma), G.to_dev(beta), eps, prep["signs"], prep["inv"])
    Y = torch.empty(rows, N, dtype=torch.bfloat16, device=G.DEV)
    G.q.qvggt_w4a4_gemm(Xq, sx, prep["Wq"], prep["sw"], G.to_dev(bias), rows, N, K, Y)
    assert G.rel_fro(G.bf16_bits(Y), want) <= G.Y_REL_FRO


def test_rotate_quant_static_step_feeds_the_gemm():
    """Codes and echoed steps of the static variant are valid inputs of the integer GEMM."""
    spec = synth.layer_spec(2)
    K, N, rows = 1024, 256, 300
    rng = np.random.default_rng(11)
    X = _heavy(rows, K, 12)
    W = rng.standard_normal((N, K)).astype(np.float32) * 0.05
    signs = synth.make_signs(spec)[:K]
    prep_o = oracle.prepare_weights(W, None, pre_signs=signs)
    _, _, Z = oracle.rotate_smooth_quant(X, prep_o.c_hat, pre_signs=signs)
    step = np.array([np.percentile(np.abs(Z), 99.9) / 7.0], dtype=np.float32)
    qx = oracle.quantize_rows_static(Z, np.full(rows, float(step[0])), 4)
    acc = oracle.int_gemm(qx, prep_o.qw)
    want = oracle.dequant_bias(acc, np.full(rows, float(step[0])), prep_o.dw, None)
    prep = G.gpu_prep(W, None, signs)
    Xq, sx = G.gpu_rsq_static(G.to_dev(X), prep["signs"], prep["inv"], G.to_dev(step), 0)
    Y = torch.empty(rows, N, dtype=torch.bfloat16, device=G.DEV)
    G.q.qvggt_w4a4_gemm(Xq, sx, prep["Wq"], prep["sw"], None, rows, N, K, Y)
    assert G.rel_fro(G.bf16_bits(Y), want) <= G.Y_REL_FRO


def test_rotate_quant_optional_arguments():
    K, rows = 1024, 64
    X = _heavy(rows, K, 7)
    signs = synth.make_signs(synth.layer_spec(2))
    Xd = G.to_dev(X)
    # no signs, no smoothing: plain orthonormal Hadamard
    dx, qx, _ = oracle.rotate_smooth_quant(X)
    Xq, sx = G.gpu_rsq(Xd, None, None)
    G.check_codes(G.gpu_unpack(Xq, K), qx)
    G.check_scales(sx.cpu().numpy(), dx)
    # signs only
    dx, qx, _ = oracle.rotate_smooth_quant(X, pre_signs=signs)
    Xq, sx = G.gpu_rsq(Xd, G.to_dev(signs), None)
    G.check_codes(G.gpu_unpack(Xq, K), qx)
    G.check_scales(sx.cpu().numpy(), dx)


def test_zero_rows_and_single_row():
    K = 1024
    X = _heavy(3, K, 9)
    X[1] = 0
    dx, qx, _ = oracle.rotate_smooth_quant(X)
    Xq, sx = G.gpu_rsq(G.to_dev(X), None, None)
    codes = G.gpu_unpack(Xq, K)
    assert sx[1].item() == 0.0 and not codes[1].any()
    G.check_codes(codes, qx)
    Xq1, sx1 = G.gpu_rsq(G.to_dev(X[:1]), None, None)
    assert np.array_equal(G.gpu_unpack(Xq1, K), codes[:1])


@pytest.mark.parametrize("K,dtype", [(1024, "bf16"), (4096, "bf16"), (256, "f32"), (768, "bf16")])
def test_rows_at_the_bottom_of_the_fp32_range(K, dtype):
    """A row whose step would fall below 2^-126 is a zero row on both sides (7 / absmax would overflow in fp32); rows a few
    binades above that line quantize like any other.  Covers the matrix-core kernel, the generic and the general one."""
    rows = 12
    x = np.zeros((rows, K), dtype=np.float32)
    x[0, 3] = 2.0 ** -120           # one-hot: every rotated value is +-2^-120 / sqrt(K): step below the line -> zero row
    x[1, 5] = -(2.0 ** -104)        # the same shape well above it: codes +-7 everywhere
    rng = np.random.default_rng(K)
    x[2] = rng.standard_normal(K) * 2.0 ** -128          # dense, below the normal range throughout
    x[3] = rng.standard_normal(K) * 2.0 ** -112          # dense, small but normal
    x[4] = rng.standard_normal(K)
    x[5:] = rng.standard_normal((rows - 5, K)) * np.exp2(rng.integers(-110, -90, (rows - 5, 1))).astype(np.float32)
    X = synth.f32_to_bf16_bits(x) if dtype == "bf16" else x
    dx, qx, _ = oracle.rotate_smooth_quant(X)
    assert dx[0] == 0.0 and dx[2] == 0.0 and dx[1] > 0 and dx[3] > 0
    Xq, sx = G.gpu_rsq(G.to_dev(X), None, None)
    codes, got = G.gpu_unpack(Xq, K), sx.cpu().numpy().astype(np.float64)
    assert got[0] == 0.0 and got[2] == 0.0 and not codes[0].any() and not codes[2].any()
    assert np.all(np.abs(codes[1]) == 7)
    G.check_codes(codes, qx, f"K={K}")
    G.check_scales(got, dx, f"K={K}")
    # a given step below the line: codes 0 (it cannot be inverted either)
    step = np.array([2.0 ** -127, 2.0 ** -130, 0.0, -1.0] + [2.0 ** -100] * (rows - 4), dtype=np.float32)
    Xq2, sx2 = G.gpu_rsq_static(G.to_dev(X), None, None, G.to_dev(step), 1)
    codes2 = G.gpu_unpack(Xq2, K)
    assert not codes2[:4].any()
    _, _, Xs = oracle.rotate_smooth_quant(X)
    G.check_codes(codes2, oracle.quantize_rows_static(Xs, step.astype(np.float64)), f"static K={K}")


def test_one_hot_row_is_dispersed_exactly():
    # a single outlier spreads to +-v/sqrt(K) everywhere: every code is +-7 and follows the Hadamard row
    K = 4096
    x = np.zeros((1, K), np.float32)
    x[0, 1234] = 3.0
    Xq, sx = G.gpu_rsq(G.to_dev(synth.f32_to_bf16_bits(x)), None, None)
    codes = G.gpu_unpack(Xq, K)
    assert np.array_equal(codes[0], 7 * oracle.hadamard(K)[1234])
    assert abs(sx.item() - 3.0 / 64 / 7) < 1e-7


def test_pack_unpack_roundtrip_and_determinism():
    K = 1024
    rng = np.random.default_rng(3)
    codes = rng.integers(-8, 8, (77, K)).astype(np.int8)
    packed = G.gpu_pack(codes)
    assert np.array_equal(G.gpu_unpack(packed, K), codes)
    assert np.array_equal(G.gpu_pack(codes).cpu().numpy(), packed.cpu().numpy())
    # a packed row is a permutation of the canonical nibble stream: same multiset of nibbles
    canon = oracle.pack_int4(codes)
    nib = lambda p: np.sort(np.concatenate([p & 0xF, p >> 4], axis=1), axis=1)
    assert np.array_equal(nib(packed.cpu().numpy()), nib(canon))


@pytest.mark.parametrize("config,name", [(1, "tiny"), (2, "qkv")])
def test_config_activations_and_weights(config, name):
    s = synth.layer_spec(config, name)
    X, W, signs, Xcal = synth.make_activation_frames(s), synth.make_weights(s), synth.make_signs(s), synth.make_calibration(s)
    a = oracle.rotated_col_absmax(Xcal, pre_signs=signs)
    prep_o = oracle.prepare_weights(W, a, pre_signs=signs, alpha=0.5)
    prep_g = G.gpu_prep(W, Xcal, signs, 0.5)
    G.check_scales(prep_g["a"].cpu().numpy(), a, "rotated activation absmax")
    G.check_scales(prep_g["inv"].cpu().numpy(), 1.0 / (np.sqrt(s.K) * prep_o.c_hat), "inv_smooth")
    G.check_scales(prep_g["sw"].cpu().numpy(), prep_o.dw, "w_scale")
    G.check_codes(G.gpu_unpack(prep_g["Wq"], s.K), prep_o.qw, "weight codes")
    dx, qx, _ = oracle.rotate_smooth_quant(X, prep_o.c_hat, pre_signs=signs)
    Xq, sx = G.gpu_rsq(G.to_dev(X), prep_g["signs"], prep_g["inv"])
    G.check_codes(G.gpu_unpack(Xq, s.K), qx, "activation codes")
    G.check_scales(sx.cpu().numpy(), dx, "x_scale")
    assert np.abs(G.gpu_unpack(Xq, s.K)).max() <= 7


def test_prep_without_smoothing_and_alpha_extremes():
    s = synth.layer_spec(1)
    W, signs, Xcal = synth.make_weights(s), synth.make_signs(s), synth.make_calibration(s)
    g = G.gpu_prep(W, None, signs)
    o = oracle.prepare_weights(W, None, pre_signs=signs)
    assert np.allclose(g["inv"].cpu().numpy(), 1 / np.sqrt(s.K), rtol=1e-6)
    G.check_codes(G.gpu_unpack(g["Wq"], s.K), o.qw)
    G.check_scales(g["sw"].cpu().numpy(), o.dw)
    a = oracle.rotated_col_absmax(Xcal, pre_signs=signs)
    for alpha in (0.0, 1.0, 0.3):
        g = G.gpu_prep(W, Xcal, signs, alpha)
        o = oracle.prepare_weights(W, a, pre_signs=signs, alpha=alpha)
        G.check_scales(g["inv"].cpu().numpy(), 1.0 / (np.sqrt(s.K) * o.c_hat), f"alpha={alpha}")
        G.check_codes(G.gpu_unpack(g["Wq"], s.K), o.qw, f"alpha={alpha}")


def test_run_to_run_bit_identity():
    s = synth.layer_spec(2)
    X = G.to_dev(synth.make_activation_frames(s))
    signs = G.to_dev(synth.make_signs(s))
    a, b = G.gpu_rsq(X, signs, None), G.gpu_rsq(X, signs, None)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


GENERAL_K = [768, 1536, 3072, 6144, 1280, 2560, 5120, 1792, 3584]       # 2^n * m, m = 12, 20, 28


@pytest.mark.parametrize("K", GENERAL_K)
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_rotate_quant_sizes_with_a_paley_factor(K, dtype):
    """H_K = H_{2^n} (x) H_m (Sec. 3.2): codes and scales against the oracle's dense product with the same matrix."""
    rows = 41
    X = _heavy(rows, K, 700 + K, dtype)
    rng = np.random.default_rng(K)
    signs = (rng.integers(0, 2, K) * 2 - 1).astype(np.int8)
    c_hat = np.exp(rng.uniform(-1, 1, K))
    inv = (1.0 / (np.sqrt(K) * c_hat)).astype(np.float32)
    for bits in (4, 8):
        dx, qx, _ = oracle.rotate_smooth_quant(X, 1.0 / (inv.astype(np.float64) * np.sqrt(K)), pre_signs=signs, bits=bits)
        if bits == 4:
            Xq, sx = G.gpu_rsq(G.to_dev(X), G.to_dev(signs), G.to_dev(inv))
            codes = G.gpu_unpack(Xq, K)
        else:
            Xq, sx = G.gpu_rsq_i8(G.to_dev(X), G.to_dev(signs), G.to_dev(inv), bits)
            codes = G.gpu_layout_int8(Xq, 0).cpu().numpy()
        G.check_codes(codes, qx, f"K={K} bits={bits}")
        G.check_scales(sx.cpu().numpy(), dx, f"K={K} bits={bits}")


@pytest.mark.parametrize("K,N", [(768, 256), (2560, 144), (3584, 512)])
def test_linear_end_to_end_with_a_paley_factor(K, N):
    """Whole path (statistic, weight preparation, rotate-quantize, integer GEMM, epilogue) on a size 2^n * m."""
    rng = np.random.default_rng(K + N)
    M = 300
    X = _heavy(M, K, K)
    Xc = _heavy(64, K, K + 1)
    W = (rng.standard_normal((N, K)) * 0.03).astype(np.float32)
    bias = synth.f32_to_bf16_bits((rng.standard_normal(N) * 0.02).astype(np.float32))
    signs = (rng.integers(0, 2, K) * 2 - 1).astype(np.int8)
    a = oracle.rotated_col_absmax(Xc, pre_signs=signs)
    po = oracle.prepare_weights(W, a, pre_signs=signs, alpha=0.5)
    want = oracle.linear(X, po, bias=bias, pre_signs=signs)
    pg = G.gpu_prep(W, Xc, signs, 0.5)
    G.check_scales(pg["a"].cpu().numpy(), a)
    G.check_codes(G.gpu_unpack(pg["Wq"], K), po.qw, f"weights K={K}")
    Y = G.bf16_bits(G.gpu_linear(G.to_dev(X), pg, G.to_dev(bias)))
    err = G.rel_fro(Y, want.Y)
    assert err <= G.Y_REL_FRO, err
    exact = oracle.to_f64(X) @ W.astype(np.float64).T + oracle.to_f64(bias)
    assert np.linalg.norm(oracle.bf16_bits_to_f64(Y) - exact) / np.linalg.norm(exact) < 0.35


@pytest.mark.parametrize("K", [256, 1024, 2048, 4096])
@pytest.mark.parametrize("rows", [1, 37, 1374, 5003])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_rotated_col_absmax(K, rows, dtype):
    """The smoothing statistic max_t |X H|[t, j] (Sec. 3.2): matrix-core kernel for bf16 at K = 1024 / 2048 / 4096, the generic
    one otherwise; ragged row counts leave the last tile partial."""
    import paper_2509_21302_amd as q
    X = _heavy(rows, K, rows + K, dtype)
    rng = np.random.default_rng(rows * K)
    signs = (rng.integers(0, 2, K) * 2 - 1).astype(np.int8)
    for sg in (signs, None):
        a = torch.full((K,), -1.0, dtype=torch.float32, device=G.DEV)
        q.qvggt_rotated_col_absmax(G.to_dev(X), G.to_dev(sg), a)
        want = oracle.rotated_col_absmax(X, pre_signs=sg)
        # a column's maximum can be a small number left by cancellation (one row: it is the rotated value itself), so the
        # fp32 butterflies are held to the row's magnitude as well as to the value: |err| <= 1e-5 |want| + 2e-6 max|want|
        assert np.allclose(a.cpu().numpy(), want, rtol=G.SCALE_RTOL, atol=2e-6 * want.max()), f"K={K} rows={rows}"
