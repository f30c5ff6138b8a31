"""Pins of the oracle's smoothing, quantizer, integer GEMM, epilogue and packing."""
import os

import numpy as np
import pytest
import torch

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------- smoothing (Eq. "smooth_factor")
def _smooth_setup(alpha, seed=0, K=128):
    rng = np.random.default_rng(seed)
    X = rng.standard_t(3, (40, K)) * rng.choice([1.0, 30.0], size=K, p=[0.95, 0.05])
    W = rng.standard_normal((24, K)) * 0.02
    Xr, Wr = oracle.rotate(X), oracle.rotate(W)
    a, w = oracle.col_absmax(Xr), oracle.col_absmax(Wr)
    c = oracle.smooth_factor(a, w, alpha)
    return X, W, Xr, Wr, a, w, c


@pytest.mark.parametrize("alpha", [0.0, 0.3, 0.5, 1.0])
def test_smoothing_identity(alpha):
    X, W, Xr, Wr, a, w, c = _smooth_setup(alpha)
    Xs = oracle.scale_columns(Xr, c, inverse=True)
    Ws = oracle.scale_columns(Wr, c, inverse=False)
    ref = X @ W.T
    assert np.abs(Xs @ Ws.T - ref).max() <= 1e-10 * np.abs(ref).max()


def test_smoothing_closed_forms():
    # alpha = 1: every activation column is normalised to absmax 1 (and the weights take it all)
    X, W, Xr, Wr, a, w, c = _smooth_setup(1.0)
    assert np.allclose(np.abs(oracle.scale_columns(Xr, c, True)).max(axis=0), 1.0, rtol=1e-12)
    assert np.allclose(np.abs(oracle.scale_columns(Wr, c, False)).max(axis=0), a * w, rtol=1e-12)
    # alpha = 0: every weight column is normalised to absmax 1
    X, W, Xr, Wr, a, w, c = _smooth_setup(0.0)
    assert np.allclose(np.abs(oracle.scale_columns(Wr, c, False)).max(axis=0), 1.0, rtol=1e-12)
    # alpha = 0.5: both sides end at sqrt(a_j w_j)
    X, W, Xr, Wr, a, w, c = _smooth_setup(0.5)
    g = np.sqrt(a * w)
    assert np.allclose(np.abs(oracle.scale_columns(Xr, c, True)).max(axis=0), g, rtol=1e-12)
    assert np.allclose(np.abs(oracle.scale_columns(Wr, c, False)).max(axis=0), g, rtol=1e-12)


def test_col_absmax_is_over_rows():
    A = np.array([[1.0, -9.0, 2.0], [-3.0, 4.0, 0.5]])
    assert np.array_equal(oracle.col_absmax(A), np.array([3.0, 9.0, 2.0]))


def test_smooth_factor_floor_and_values():
    c = oracle.smooth_factor(np.array([4.0, 0.0, 9.0]), np.array([1.0, 4.0, 0.0]), 0.5, floor=1e-4)
    assert np.allclose(c, [2.0, 1e-2 / 2.0, 3.0 / 1e-2], rtol=1e-14)


# ----------------------------------------------------------------- quantizer (Eq. "quantization")
def _read_cases():
    cases, cur = [], {}
    for line in open(os.path.join(GOLD, "quantizer_rows.txt")):
        line = line.strip()
        if not line or line[0] == "#":
            continue
        tag, vals = line[0], [float(v) for v in line[1:].split()]
        cur[tag] = vals
        if tag == "q":
            cases.append(cur)
            cur = {}
    return cases


def test_quantizer_hand_worked_rows():
    cases = _read_cases()
    assert len(cases) == 4
    for c in cases:
        d, q = oracle.quantize_rows(np.array([c["x"]]), 4)
        assert d[0] == c["d"][0]
        assert q[0].tolist() == [int(v) for v in c["q"]]


def test_quantizer_properties():
    rng = np.random.default_rng(5)
    A = rng.standard_t(3, (50, 256)) * 3.7
    d, q = oracle.quantize_rows(A, 4)
    assert np.allclose(d, np.abs(A).max(axis=1) / 7.0, rtol=1e-15)
    assert q.min() >= -7 and q.max() <= 7            # -8 is unreachable with a dynamic absmax step
    err = np.abs(A - d[:, None] * q)
    assert np.all(err <= d[:, None] / 2 * (1 + 1e-12))
    # the absmax element gets code +-7
    j = np.abs(A).argmax(axis=1)
    assert np.array_equal(np.abs(q[np.arange(50), j]), np.full(50, 7))
    # odd symmetry and positive-scale equivariance
    d2, q2 = oracle.quantize_rows(-A, 4)
    assert np.array_equal(q2, -q) and np.array_equal(d2, d)
    d3, q3 = oracle.quantize_rows(A * 8.0, 4)         # power of two: exact
    assert np.array_equal(q3, q) and np.array_equal(d3, d * 8.0)
    # rows are quantized independently: scaling one row leaves the others alone
    B = A.copy()
    B[3] *= 1000.0
    d4, q4 = oracle.quantize_rows(B, 4)
    assert np.array_equal(np.delete(q4, 3, 0), np.delete(q, 3, 0))
    # other bit-widths follow the same definition
    d8, q8 = oracle.quantize_rows(A, 8)
    assert np.allclose(d8, np.abs(A).max(axis=1) / 127.0) and q8.max() == 127 or q8.min() == -127


@pytest.mark.parametrize("bits", [4, 5, 6, 8])
def test_quantizer_other_bit_widths(bits):
    """The 8-bit and 6-bit settings use the same quantizer with qmax = 2^(bits-1) - 1: closed forms, the error bound,
    and a brute-force re-derivation with Python's own round-half-even on every element."""
    qmax = 2 ** (bits - 1) - 1
    rng = np.random.default_rng(bits)
    A = rng.standard_t(3, (20, 96)) * 2.3
    A[4] = 0.0
    d, q = oracle.quantize_rows(A, bits)
    amax = np.abs(A).max(axis=1)
    assert np.array_equal(d, amax / qmax)
    assert q.min() >= -qmax and q.max() <= qmax and not q[4].any() and d[4] == 0.0
    live = amax > 0
    assert np.array_equal(np.abs(q[np.arange(20), np.abs(A).argmax(axis=1)])[live], np.full(live.sum(), qmax))
    assert np.all(np.abs(A - d[:, None] * q) <= d[:, None] / 2 * (1 + 1e-12))
    for r in range(20):
        if d[r] > 0:
            assert q[r].tolist() == [max(-qmax - 1, min(qmax, round(float(v) / float(d[r])))) for v in A[r]]
    # ties go to the even code, the clamp is at -qmax - 1 and qmax
    T = np.array([[0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 1e9, -1e9]])
    assert oracle.quantize_rows_static(T, np.array([1.0]), bits)[0].tolist() == [0, 2, 2, 0, -2, -2, qmax, -qmax - 1]


def test_more_bits_means_a_smaller_error_by_the_ratio_of_the_steps():
    rng = np.random.default_rng(12)
    X = rng.standard_normal((64, 256))
    W = rng.standard_normal((48, 256)) * 0.05
    exact = X @ W.T
    err = {}
    for bits in (4, 6, 8):
        prep = oracle.prepare_weights(W, None, bits=bits)
        y = oracle.linear(X, prep, bits=bits).y
        err[bits] = np.linalg.norm(y - exact) / np.linalg.norm(exact)
    # uniform rounding noise scales with the step: 7/31 and 31/127 between the settings, within a factor 1.5
    assert 0.5 * 7 / 31 < err[6] / err[4] < 1.5 * 7 / 31
    assert 0.5 * 31 / 127 < err[8] / err[6] < 1.5 * 31 / 127


def test_quantizer_clamp_is_live_with_a_static_step():
    A = np.array([[-100.0, -7.6, 7.4, 7.6, 100.0, -8.5]])
    q = oracle.quantize_rows_static(A, np.array([1.0]), 4)
    assert q[0].tolist() == [-8, -8, 7, 7, 7, -8]


# ----------------------------------------------------------------- integer GEMM
def test_steps_below_the_single_precision_normal_range_count_as_zero():
    """The steps are handed on as fp32 numbers: a row whose step absmax / qmax falls below 2^-126 (the smallest normal one) is
    quantized like a row of zeros, the row just above that line like any other; a given step below the line gives codes 0."""
    tiny = 2.0 ** -126
    for bits in (4, 8):
        qmax = (1 << (bits - 1)) - 1
        A = np.zeros((4, 8))
        A[0, :4] = [qmax * tiny * 0.999, -tiny, tiny / 3, 0.0]           # step just below the line
        A[1, :4] = [qmax * tiny, -qmax * tiny / 2, tiny, 0.0]             # step exactly on it
        A[2, :4] = [1e-30, -5e-31, 2.5e-31, 0.0]                          # far above
        A[3, :4] = [1e-39, -1e-40, 3e-41, 0.0]                            # what a GELU of x ~ -13 hands on
        d, q = oracle.quantize_rows(A, bits)
        assert d[0] == 0.0 and not q[0].any() and d[3] == 0.0 and not q[3].any()
        assert d[1] == tiny and q[1, 0] == qmax and q[1, 1] == -(qmax + 1) // 2 and q[1, 2] == 1      # -3.5 -> -4, -63.5 -> -64: ties to even
        assert d[2] == 1e-30 / qmax and q[2, 0] == qmax
        qs = oracle.quantize_rows_static(A, np.array([tiny * 0.5, tiny, -1.0, 0.0]), bits)
        assert not qs[0].any() and not qs[2].any() and not qs[3].any()
        assert qs[1, 0] == qmax and qs[1, 2] == 1
    d, zp, u = oracle.quantize_rows_asym(np.array([[15 * tiny * 0.99, 0.0, 0.0], [15 * tiny, 0.0, -0.0]]), 4)
    assert d[0] == 0.0 and zp[0] == 0 and not u[0].any()
    assert d[1] == tiny and zp[1] == 0 and u[1, 0] == 15


def test_int_gemm_brute_force_and_library():
    rng = np.random.default_rng(6)
    M, N, K = 5, 7, 12
    qx = rng.integers(-8, 8, (M, K)).astype(np.int8)
    qw = rng.integers(-8, 8, (N, K)).astype(np.int8)
    acc = oracle.int_gemm(qx, qw)
    brute = [[sum(int(qx[t, j]) * int(qw[o, j]) for j in range(K)) for o in range(N)] for t in range(M)]
    assert acc.tolist() == brute
    # second loop order: accumulate rank-1 updates over j
    acc2 = np.zeros((M, N), dtype=np.int64)
    for j in range(K):
        acc2 += np.outer(qx[:, j].astype(np.int64), qw[:, j].astype(np.int64))
    assert np.array_equal(acc, acc2)


def test_int_gemm_config1_against_numpy_and_bounds():
    rng = np.random.default_rng(7)
    qx = rng.integers(-8, 8, (64, 128)).astype(np.int8)
    qw = rng.integers(-8, 8, (128, 128)).astype(np.int8)
    acc = oracle.int_gemm(qx, qw)
    assert np.array_equal(acc, qx.astype(np.int64) @ qw.astype(np.int64).T)
    assert np.abs(acc).max() <= 64 * 128
    # extreme codes reach the bound exactly
    full = oracle.int_gemm(np.full((2, 4096), -8, np.int8), np.full((3, 4096), -8, np.int8))
    assert np.all(full == 64 * 4096)
    # selecting patterns: qw = one-hot rows picks columns of qx
    sel = np.zeros((128, 128), np.int8)
    sel[np.arange(128), (np.arange(128) * 5) % 128] = 1
    assert np.array_equal(oracle.int_gemm(qx, sel), qx[:, (np.arange(128) * 5) % 128].astype(np.int32))


# ----------------------------------------------------------------- bf16 rounding and epilogue
def test_bf16_hand_cases():
    for line in open(os.path.join(GOLD, "bf16_cases.txt")):
        line = line.strip()
        if not line or line[0] == "#":
            continue
        val, bits = line.split()
        v = float.fromhex(val) if "x" in val else float(val)
        got = int(oracle.bf16_from_f64(np.array([v]))[0])
        assert got == int(bits, 16), (val, hex(got), bits)


def test_bf16_matches_library_rounding_on_fp32_values():
    # for values that are exactly fp32, one rounding double->bf16 equals torch's fp32->bf16 (nearest even)
    rng = np.random.default_rng(8)
    x = (rng.standard_normal(200000) * np.exp(rng.uniform(-30, 30, 200000))).astype(np.float32)
    x[:7] = [0.0, -0.0, 1.0, 65504.0, 3.3e38, 1e-38, -1e-40]
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = oracle.bf16_from_f64(x.astype(np.float64))
    assert np.array_equal(got, ref)
    back = oracle.bf16_bits_to_f64(got)
    assert np.all(np.abs(back - x) <= np.abs(x) * 2.0 ** -8 + 1e-40)


def test_epilogue_exact_cases():
    acc = np.array([[3, -5, 0], [7, 1, -2]], dtype=np.int32)
    one = np.ones(3)
    # unit scales, no bias: Y is the accumulator itself
    Y = oracle.dequant_bias(acc, np.ones(2), one)
    assert np.array_equal(oracle.bf16_bits_to_f64(Y), acc.astype(np.float64))
    # per-token and per-channel steps are powers of two, so every product is exact
    dx = np.array([0.5, 4.0])              # token steps
    dw = np.array([2.0, 0.25, 8.0])        # output-channel steps
    b = np.array([1.0, -0.5, 0.0])
    Y, y = oracle.dequant_bias(acc, dx, dw, b, want_f64=True)
    expect = np.array([[3 * 0.5 * 2 + 1, -5 * 0.5 * 0.25 - 0.5, 0.0],
                       [7 * 4 * 2 + 1, 1 * 4 * 0.25 - 0.5, -2 * 4 * 8.0]])
    assert np.array_equal(y, expect)
    assert np.array_equal(oracle.bf16_bits_to_f64(Y), expect)     # all exactly representable in bf16


# ----------------------------------------------------------------- packing
def test_pack_roundtrip_all_byte_values():
    packed = np.arange(256, dtype=np.uint8).reshape(4, 64)
    q = oracle.unpack_int4(packed, 128)
    assert q.min() == -8 and q.max() == 7
    assert np.array_equal(oracle.pack_int4(q), packed)
    # byte 0xA7: low nibble 7 -> +7 (element 0), high nibble 0xA -> -6 (element 1)
    assert oracle.unpack_int4(np.array([[0xA7]], np.uint8), 2).tolist() == [[7, -6]]
    with pytest.raises(oracle.OracleError):
        oracle.pack_int4(np.array([[9, 0]], np.int8))


# ----------------------------------------------------------------- LayerNorm in front of the quantized layer
def test_layernorm_closed_forms_and_library():
    rng = np.random.default_rng(21)
    X = rng.standard_t(3, (12, 256)) * 3 + rng.standard_normal((12, 1)) * 10
    y = oracle.layernorm(X, eps=0.0, round_to_bf16=False)
    assert np.allclose(y.mean(axis=1), 0.0, atol=1e-13) and np.allclose((y ** 2).mean(axis=1), 1.0, rtol=1e-12)
    # invariant under shift and positive scale of a row (eps = 0); gamma, beta act per channel afterwards
    assert np.allclose(oracle.layernorm(7.0 * X - 3.0, eps=0.0, round_to_bf16=False), y, atol=1e-11)
    g, b = rng.uniform(0.5, 2, 256), rng.standard_normal(256)
    assert np.allclose(oracle.layernorm(X, g, b, eps=0.0, round_to_bf16=False), y * g + b, rtol=1e-13, atol=1e-13)
    # two-point row: values +-1 whatever the inputs; eps shrinks them by sqrt(var / (var + eps))
    assert oracle.layernorm(np.array([[3.0, 5.0]]), eps=0.0, round_to_bf16=False).tolist() == [[-1.0, 1.0]]
    assert np.allclose(oracle.layernorm(np.array([[3.0, 5.0]]), eps=3.0, round_to_bf16=False), [[-0.5, 0.5]], rtol=1e-15)
    # the library routine in float64
    t = torch.nn.functional.layer_norm(torch.from_numpy(X), (256,), torch.from_numpy(g), torch.from_numpy(b), eps=1e-5).numpy()
    assert np.allclose(oracle.layernorm(X, g, b, eps=1e-5, round_to_bf16=False), t, rtol=1e-12, atol=1e-12)
    # rounding to bfloat16: values are bf16-representable and within half an ulp (at most 2^-8 relative) of the exact ones
    r = oracle.layernorm(X, g, b, eps=1e-5)
    assert np.array_equal(oracle.bf16_bits_to_f64(oracle.bf16_from_f64(r)), r)
    assert np.all(np.abs(r - t) <= np.abs(t) * 2.0 ** -8 + 1e-40) and np.abs(r - t).max() > 0


def test_prepare_weights_given_hand_worked_and_reductions():
    """Given factor and steps: a K = 4 layer worked by hand with the Hadamard matrix written out, and the two reductions to
    already pinned routines (factor and steps taken from prepare_weights reproduce it; no factor, no steps = rotation only)."""
    H4 = np.array([[1, 1, 1, 1], [1, -1, 1, -1], [1, 1, -1, -1], [1, -1, -1, 1]], dtype=np.float64) / 2.0
    W = np.array([[1.0, 2.0, 3.0, 4.0], [0.5, -0.5, 0.25, 8.0]])
    c = np.array([1.0, 3.0, 0.5, 4.0])
    step = np.array([0.5, 1.0])
    # rows of W H: [5, -1, -2, 0] and [4.125, -3.375, -4.125, 4.375]; times c: [5, -3, -1, 0], [4.125, -10.125, -2.0625, 17.5]
    assert np.allclose(W @ H4, [[5, -1, -2, 0], [4.125, -3.375, -4.125, 4.375]], atol=1e-15)
    p = oracle.prepare_weights_given(W, c, step)
    # / step: [10, -6, -2, 0] -> clamp to 7;  [4.125, -10.125, -2.0625, 17.5] -> 4, clamp to -8, -2, clamp to 7
    assert p.qw.tolist() == [[7, -6, -2, 0], [4, -8, -2, 7]] and p.dw.tolist() == [0.5, 1.0]
    assert np.allclose(p.Ws, [[5, -3, -1, 0], [4.125, -10.125, -2.0625, 17.5]], atol=1e-15)
    q = oracle.prepare_weights_given(W, c, None)          # own steps: absmax / 7 of each smoothed row = 5 / 7 and 2.5
    assert np.allclose(q.dw, [5 / 7, 2.5], rtol=1e-15) and q.qw.tolist() == [[7, -4, -1, 0], [2, -4, -1, 7]]
    rng = np.random.default_rng(8)
    Wb = rng.standard_normal((24, 256))
    signs = (rng.integers(0, 2, 256) * 2 - 1).astype(np.int8)
    a = np.exp(rng.uniform(-2, 2, 256))
    ref = oracle.prepare_weights(Wb, a, pre_signs=signs, alpha=0.5)
    got = oracle.prepare_weights_given(Wb, ref.c_hat, ref.dw, pre_signs=signs)
    assert np.array_equal(got.qw, ref.qw) and np.array_equal(got.dw, ref.dw)
    plain = oracle.prepare_weights_given(Wb, None, None, pre_signs=signs)
    ref0 = oracle.prepare_weights(Wb, None, pre_signs=signs)
    assert np.array_equal(plain.qw, ref0.qw) and np.array_equal(plain.dw, ref0.dw)
    # a smaller step than the channel's own makes the clamp live, a larger one leaves the top codes unused
    tight = oracle.prepare_weights_given(Wb, ref.c_hat, 0.5 * ref.dw, pre_signs=signs)
    assert (tight.qw == 7).sum() > (ref.qw == 7).sum() and (tight.qw == -8).any()
    loose = oracle.prepare_weights_given(Wb, ref.c_hat, 2.0 * ref.dw, pre_signs=signs)
    assert np.abs(loose.qw).max() <= 4


def test_gelu_against_the_integral_and_closed_forms():
    """GELU(x) = x Phi(x): Phi from a quadrature of the normal density (no error function involved), the odd-part identity
    GELU(x) - GELU(-x) = x, printed values of Phi, the library routine in float64, and the bf16 rounding."""
    x = np.concatenate([np.linspace(-6, 6, 97), [0.0, 1e-3, -1e-3, 0.5, -7.5]])
    y = oracle.gelu(x[None, :], round_to_bf16=False)[0]
    # composite Simpson on [0, |x|] with 2000 intervals: error far below 1e-13 for the smooth density
    def phi_quad(v):
        n = 2000
        t = np.linspace(0.0, abs(v), n + 1)
        f = np.exp(-0.5 * t * t) / np.sqrt(2.0 * np.pi)
        integral = (abs(v) / n / 3.0) * (f[0] + f[-1] + 4.0 * f[1:-1:2].sum() + 2.0 * f[2:-1:2].sum())
        return 0.5 + np.sign(v) * integral
    want = np.array([v * phi_quad(v) for v in x])
    assert np.allclose(y, want, rtol=0, atol=2e-13)
    assert np.allclose(y - oracle.gelu(-x[None, :], round_to_bf16=False)[0], x, rtol=0, atol=1e-15)
    # Phi(1) = 0.841344746068543, Phi(-2) = 0.022750131948179, Phi(-6) = 9.8658764503769e-10 (standard tables)
    pts = oracle.gelu(np.array([[1.0, -2.0, -6.0, 0.0]]), round_to_bf16=False)[0]
    assert np.allclose(pts[:3], [0.841344746068543, -2 * 0.022750131948179, -6 * 9.8658764503769e-10], rtol=1e-12) and pts[3] == 0.0
    t = torch.nn.functional.gelu(torch.from_numpy(x)).numpy()
    assert np.allclose(y, t, rtol=1e-9, atol=1e-15)          # the library's 1 + erf loses relative accuracy in the negative tail
    r = oracle.gelu(x[None, :])[0]
    assert np.array_equal(oracle.bf16_bits_to_f64(oracle.bf16_from_f64(r)), r)
    assert np.all(np.abs(r - y) <= np.abs(y) * 2.0 ** -8 + 1e-40) and np.abs(r - y).max() > 0


# ----------------------------------------------------------------- asymmetric activation codes (appendix, further settings)
def test_asymmetric_quantizer_hand_worked_rows():
    # lo = -3, hi = 12: step 1, zero point 3; 4.5 and -2.5 are ties (to even: 4 and -2)
    d, zp, u = oracle.quantize_rows_asym(np.array([[-3.0, 12.0, 0.0, 4.5, 5.5, -2.5]]), 4)
    assert d[0] == 1.0 and zp[0] == 3 and u[0].tolist() == [0, 15, 3, 7, 9, 1]
    # a row without negative values: the range is [0, hi], zero point 0, unsigned round-to-nearest with step hi / 15
    d, zp, u = oracle.quantize_rows_asym(np.array([[0.0, 30.0, 2.0, 3.0, 29.0, 14.9]]), 4)
    assert d[0] == 2.0 and zp[0] == 0 and u[0].tolist() == [0, 15, 1, 2, 14, 7]          # 1.5 -> 2 (even), 14.5 -> 14 (even)
    # strictly positive values: 0 stays representable, the lowest code is unused
    d, zp, u = oracle.quantize_rows_asym(np.array([[15.0, 30.0]]), 4)
    assert d[0] == 2.0 and zp[0] == 0 and u[0].tolist() == [8, 15]
    # a range symmetric about 0: -lo / step = 7.5, tie to even: zero point 8
    d, zp, u = oracle.quantize_rows_asym(np.array([[-15.0, 15.0, 0.0, 1.0]]), 4)
    assert d[0] == 2.0 and zp[0] == 8 and u[0].tolist() == [0, 15, 8, 8]                  # -7.5 -> -8, 7.5 -> 8 clamps at 15
    # zeros
    d, zp, u = oracle.quantize_rows_asym(np.zeros((2, 8)), 4)
    assert not d.any() and not zp.any() and not u.any()


@pytest.mark.parametrize("bits", [4, 8])
def test_asymmetric_quantizer_properties(bits):
    rng = np.random.default_rng(11)
    levels = (1 << bits) - 1
    A = rng.standard_t(3, (60, 192)) * 2.3 + rng.uniform(-3, 6, (60, 1))          # rows with different offsets
    A[7] = np.abs(A[7])
    A[8] = -np.abs(A[8])
    d, zp, u = oracle.quantize_rows_asym(A, bits)
    lo, hi = np.minimum(A.min(axis=1), 0), np.maximum(A.max(axis=1), 0)
    assert np.allclose(d, (hi - lo) / levels, rtol=1e-15)
    assert zp.min() >= 0 and zp.max() <= levels and zp[7] == 0 and zp[8] == levels
    # nearest grid point: the reconstruction is within half a step everywhere, and no other code does better
    rec = d[:, None] * (u.astype(np.int64) - zp[:, None])
    assert np.all(np.abs(A - rec) <= d[:, None] / 2 * (1 + 1e-9))
    grid = d[:, None, None] * (np.arange(levels + 1)[None, None, :] - zp[:, None, None])       # [rows, 1, codes]
    best = np.abs(A[:, :, None] - grid).min(axis=2)
    assert np.allclose(np.abs(A - rec), best, rtol=0, atol=1e-12 * np.abs(A).max())
    # the extremes take the end codes when the row has both signs
    both = (A.min(axis=1) < 0) & (A.max(axis=1) > 0)
    r = np.arange(60)
    assert np.all(u[r, A.argmin(axis=1)][both] == 0) and np.all(u[r, A.argmax(axis=1)][both] == levels)
    # scale equivariance (power of two: exact), independence of rows
    d2, zp2, u2 = oracle.quantize_rows_asym(A * 4.0, bits)
    assert np.array_equal(u2, u) and np.array_equal(zp2, zp) and np.array_equal(d2, 4.0 * d)
    # shifting a row by whole steps that keeps 0 inside the range moves the zero point, not the codes
    x = np.array([[-4.0, 11.0, 0.25, 3.75, -1.5, 7.0]])
    d0, z0, u0 = oracle.quantize_rows_asym(x, 4)
    d1, z1, u1 = oracle.quantize_rows_asym(x + 2.0, 4)
    assert d0[0] == 1.0 and d1[0] == 1.0 and z1[0] == z0[0] - 2 and np.array_equal(u0, u1)


def test_asymmetric_codes_halve_the_step_on_one_sided_rows():
    """On rows without negative values (what a GELU hands on, before any rotation) the affine grid spends all 16 codes on
    [0, hi] where the symmetric one spends 8: the step is 7 / 15 of the symmetric step and the error falls accordingly."""
    rng = np.random.default_rng(12)
    A = np.abs(rng.standard_normal((40, 512)))
    ds, qs = oracle.quantize_rows(A, 4)
    da, zp, u = oracle.quantize_rows_asym(A, 4)
    assert np.allclose(da, ds * 7.0 / 15.0, rtol=1e-15)
    es = np.sqrt(((A - ds[:, None] * qs) ** 2).mean())
    ea = np.sqrt(((A - da[:, None] * (u.astype(float) - zp[:, None])) ** 2).mean())
    assert 0.40 < ea / es < 0.55


def test_asymmetric_integer_product_and_its_split():
    """sum_j (u - zp) qw is the brute-force triple loop, and equals the product of the stored signed codes u - 8 with qw plus
    (8 - zp) times the weight code sums: the split the integer GEMM uses."""
    rng = np.random.default_rng(13)
    M, N, K = 9, 7, 32
    u = rng.integers(0, 16, (M, K)).astype(np.uint8)
    zp = rng.integers(0, 16, M)
    qw = rng.integers(-8, 8, (N, K)).astype(np.int8)
    acc = oracle.int_gemm_asym(u, zp, qw)
    want = np.zeros((M, N), dtype=np.int64)
    for t in range(M):
        for o in range(N):
            for j in range(K):
                want[t, o] += (int(u[t, j]) - int(zp[t])) * int(qw[o, j])
    assert np.array_equal(acc, want)
    stored = (u.astype(np.int16) - 8).astype(np.int8)
    split = oracle.int_gemm(stored, qw).astype(np.int64) + (8 - zp)[:, None] * oracle.weight_code_sums(qw)[None, :]
    assert np.array_equal(acc, split)


def test_asymmetric_layer_approximates_the_float_layer():
    """End to end on one-sided inputs with a common offset (post-GELU-like rows keep a large mean after the rotation only in
    column 0; the affine grid absorbs it): the asymmetric layer's error against X W^T + b is below the symmetric layer's."""
    rng = np.random.default_rng(14)
    M, N, K = 48, 40, 256
    X = np.abs(rng.standard_normal((M, K))) + 0.5
    W = rng.standard_normal((N, K)) * 0.05
    b = rng.standard_normal(N) * 0.1
    prep = oracle.prepare_weights(W, oracle.rotated_col_absmax(X))
    ref = X @ W.T + b
    ys = oracle.linear(X, prep, b).y
    _, ya, acc, u, zp, dx = oracle.linear_asym(X, prep, b)
    es, ea = np.linalg.norm(ys - ref) / np.linalg.norm(ref), np.linalg.norm(ya - ref) / np.linalg.norm(ref)
    assert ea < es and ea < 0.2
    # the integer accumulators reproduce the dequantized product exactly
    Xs = oracle.scale_columns(oracle.rotate(X), prep.c_hat, inverse=True)
    rec = dx[:, None] * (u.astype(np.float64) - zp[:, None])
    assert np.all(np.abs(Xs - rec) <= dx[:, None] / 2 * (1 + 1e-9))
    assert np.allclose(ya - b, (rec @ (prep.qw.astype(np.float64) * prep.dw[:, None]).T), rtol=1e-12, atol=1e-12)


def test_mixed_widths_order_the_error():
    """Mixed precision (appendix, further settings): each operand has its own width; widening either one lowers the layer's
    error against the float product, and widening the activations alone leaves the weight codes untouched."""
    rng = np.random.default_rng(15)
    M, N, K = 64, 48, 256
    X = rng.standard_t(3, (M, K))
    W = rng.standard_normal((N, K)) * 0.05
    ref = X @ W.T
    a = oracle.rotated_col_absmax(X)
    err = {}
    for wb in (4, 8):
        prep = oracle.prepare_weights(W, a, bits=wb)
        assert np.abs(prep.qw).max() == (1 << (wb - 1)) - 1
        for ab in (4, 8):
            r = oracle.linear(X, prep, bits=ab)
            assert np.abs(r.qx).max() == (1 << (ab - 1)) - 1
            err[wb, ab] = np.linalg.norm(r.y - ref) / np.linalg.norm(ref)
    assert err[8, 8] < err[4, 8] < err[4, 4] and err[8, 8] < err[8, 4] < err[4, 4]


def test_four_bit_codes_are_e2m3_numbers():
    """What the 6-bit floating-point matrix path rests on, from the format's definition (1 sign, 2 exponent bits with bias 1,
    3 mantissa bits, exponent 0 subnormal): every code of a dynamic 4-bit quantizer (-7 .. 7) is an E2M3 number, and so is
    every half-integer -7.5 .. 7.5 (a code of the full range -8 .. 7 or 0 .. 15 stored half a step up); -8 and 8 are not.
    Products of such values with integer codes are multiples of 1/2 (1/4 for two shifted operands, never used) and a row sum
    over K = 8192 stays below 2^23, so float32 holds it exactly in any order of addition."""
    values = set()
    for e in range(4):
        for m in range(8):
            mag = m / 8.0 if e == 0 else 2.0 ** (e - 1) * (1 + m / 8.0)
            values.update((mag, -mag))
    assert len(values) == 63 and max(values) == 7.5                       # +0 and -0 coincide
    assert all(float(q) in values for q in range(-7, 8))
    assert all(q + 0.5 in values for q in range(-8, 8))
    assert -8.0 not in values and 8.0 not in values
    worst = 7.5 * 7 * 8192                                                # |shifted code| * |weight code| * K
    assert 2 * worst < 2 ** 23 and np.float32(worst) == worst and np.float32(worst - 0.5) == worst - 0.5
    # and in integers: 49 * 8192 < 2^24
    assert 49 * 8192 < 2 ** 24
