"""GPU parity of fc2's kernel 1 with the preceding GELU fused in (qvggt_gelu_rotate_smooth_quant, _e2m3) against the oracle's
GELU followed by its rotate_smooth_quant, and of the chain fc1 -> GELU -> fc2 with no activation pass in between."""
import numpy as np
import pytest
import torch

import oracle
import synth
from synth import f32_to_bf16_bits
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

# The activation is rounded to bf16 before the rotation on both sides, and the kernel takes that rounded value from a table of
# correctly rounded results (every bf16 input has its own entry or an exact rule), so the rotation sees the same bf16 tensor as
# the oracle's: the standard bars of kernel 1 apply (a code off by one on at most 1e-4 of the elements, steps within 1e-5).


def _fc1_output_like(rows, K, seed):
    """What fc1 hands on: roughly unit-scale, heavy-tailed, a few strong channels, a few strong tokens, both signs."""
    rng = np.random.default_rng(seed)
    x = rng.standard_t(4, (rows, K)).astype(np.float32) * 1.5
    x[:, rng.choice(K, max(1, K // 200), replace=False)] *= 8
    x[: min(3, rows)] *= 6
    return f32_to_bf16_bits(x)


def _check(codes, got, qx, dx, what):
    frac = G.check_codes(codes, qx, what)
    G.check_scales(got, dx, what)
    return frac


def _gpu_gelu_rsq(Xd, sd, invd):
    M, K = Xd.shape
    Xq = torch.full((M, K // 2), 0xA5, dtype=torch.uint8, device=G.DEV)
    sx = torch.empty(M, dtype=torch.float32, device=G.DEV)
    G.q.qvggt_gelu_rotate_smooth_quant(Xd, sd, invd, G.gelu_table(), Xq, sx)
    return Xq, sx


def test_gelu_table_is_the_correctly_rounded_activation():
    """Every entry of the device-built table against the oracle's float64 GELU rounded to bf16, bit for bit; and the rules
    the kernel applies outside the table's window, checked on the oracle side for every bf16 input they cover."""
    tab = G.gelu_table().cpu().numpy().view(np.uint16)
    assert tab.size == 8192
    e = np.arange(8192)
    bits = (((e >> 12) << 15) | (0x3580 + (e & 0xFFF))).astype(np.uint16)
    want = oracle.bf16_from_f64(oracle.gelu(bits, round_to_bf16=False))
    assert np.array_equal(tab, want)
    allbits = np.arange(65536, dtype=np.uint32)
    allbits = allbits[(allbits & 0x7FFF) < 0x7F80]                            # finite inputs
    mag = allbits & 0x7FFF
    finite = np.ones(allbits.size, dtype=bool)
    act = oracle.bf16_from_f64(oracle.gelu(allbits.astype(np.uint16), round_to_bf16=False)).astype(np.uint32)
    tiny = finite & (mag < 0x3580)
    half = oracle.bf16_from_f64(0.5 * oracle.to_f64(allbits.astype(np.uint16))).astype(np.uint32)
    assert np.array_equal(act[tiny], half[tiny])                              # |x| < 2^-20: x / 2
    big = finite & (mag >= 0x4580)
    assert np.array_equal(act[big & (allbits < 0x8000)], allbits[big & (allbits < 0x8000)])      # x >= 2^12: x
    assert np.all(act[big & (allbits >= 0x8000)] == 0x8000)                   # x <= -2^12: -0


@pytest.mark.parametrize("K,rows", [(1024, 1031), (2048, 300), (4096, 203), (4096, 1)])
def test_gelu_rotate_quant(K, rows):
    X = _fc1_output_like(rows, K, 900 + K + rows)
    rng = np.random.default_rng(K + 9)
    signs = (rng.integers(0, 2, K) * 2 - 1).astype(np.int8)
    c_hat = np.exp(rng.uniform(-1, 1, K))
    inv = (1.0 / (np.sqrt(K) * c_hat)).astype(np.float32)
    act = oracle.gelu(X)
    dx, qx, _ = oracle.rotate_smooth_quant(act, 1.0 / (inv.astype(np.float64) * np.sqrt(K)), pre_signs=signs)
    Xd, sd, invd = G.to_dev(X), G.to_dev(signs), G.to_dev(inv)
    Xq, sx = _gpu_gelu_rsq(Xd, sd, invd)
    frac = _check(G.gpu_unpack(Xq, K), sx.cpu().numpy().astype(np.float64), qx, dx, f"K={K}")
    G.report("gelu_rotate_quant", K=K, rows=rows, code_mismatch_fraction=frac)
    # the E2M3 output: the same steps and, decoded, the same codes
    Xf = torch.full((G.q.qvggt_e2m3_bytes(rows, K),), 0xA5, dtype=torch.uint8, device=G.DEV)
    sxf = torch.empty(rows, dtype=torch.float32, device=G.DEV)
    G.q.qvggt_gelu_rotate_smooth_quant_e2m3(Xd, sd, invd, G.gelu_table(), Xf, sxf)
    assert torch.equal(sx, sxf)
    conv = torch.full_like(Xf, 0xA5)
    G.codes_to_e2m3(Xq, rows, K, conv)
    assert np.array_equal(G.decode_e2m3_rows(Xf.cpu().numpy(), rows, K), G.decode_e2m3_rows(conv.cpu().numpy(), rows, K))


def test_gelu_rotate_quant_special_values():
    """Zeros stay zeros (step 0, codes 0); large negative inputs vanish, large positive ones pass unchanged; no signs, no smoothing."""
    K, rows = 1024, 9
    x = np.zeros((rows, K), dtype=np.float32)
    x[1] = -30.0
    x[2] = 25.0
    x[3, ::2] = -12.0
    x[3, 1::2] = 3.0
    x[4:] = np.random.default_rng(4).standard_normal((rows - 4, K)) * 0.01          # the linear regime around zero: y ~ x / 2
    X = f32_to_bf16_bits(x)
    dx, qx, _ = oracle.rotate_smooth_quant(oracle.gelu(X))
    Xq, sx = _gpu_gelu_rsq(G.to_dev(X), None, None)
    codes, got = G.gpu_unpack(Xq, K), sx.cpu().numpy().astype(np.float64)
    assert got[0] == 0.0 and not codes[0].any()
    assert got[1] == 0.0 and dx[1] == 0.0 and not codes[1].any()
    _check(codes[2:], got[2:], qx[2:], dx[2:], "special rows")


def test_gelu_outputs_at_the_bottom_of_the_fp32_range():
    """x around -13 gives activations around 1e-38: rows of them land on either side of the smallest step (2^-126) and must agree
    with the oracle on which; nothing overflows to infinity or NaN on the way."""
    K = 1024
    x = np.zeros((6, K), dtype=np.float32)
    x[0] = -13.0
    x[1] = -12.0
    x[2, ::2], x[2, 1::2] = -12.5, -13.25
    x[3] = -14.0                                        # rounds to -0 in bf16: a zero row
    x[4, :8] = -11.0
    x[5] = -13.5
    X = f32_to_bf16_bits(x)
    dx, qx, _ = oracle.rotate_smooth_quant(oracle.gelu(X))
    assert (dx == 0).any() and (dx > 0).any()
    Xq, sx = _gpu_gelu_rsq(G.to_dev(X), None, None)
    codes, got = G.gpu_unpack(Xq, K), sx.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    assert np.array_equal(got == 0, dx == 0)
    _check(codes, got, qx, dx, "tiny activations")


def test_gelu_rotate_quant_every_input_value():
    """All finite bf16 values as inputs: every exponent, both signs, subnormals, zeros, and the values outside the table's window.
    A row holds 1024 consecutive magnitudes (eight binades) with random signs, so its step is set by values of its own size; three
    arrangements shifted against each other put every value among the largest of some row.  Rows whose rotated values leave the
    float32 range the kernel computes in (|.| < 1e-30 or > 1e37) are run but not compared."""
    K = 1024
    mags = np.arange(0x7F80, dtype=np.uint32)                                 # finite magnitudes, ascending
    rng = np.random.default_rng(77)
    rows_list = []
    for shift in (0, 384, 768):
        m = mags[shift: shift + (mags.size - shift) // K * K].reshape(-1, K)
        sign = rng.integers(0, 2, m.shape).astype(np.uint32) << 15
        rows_list.append((m | sign).astype(np.uint16))
    X = np.concatenate(rows_list)
    mod = f32_to_bf16_bits((rng.standard_normal((64, K)) * 2).astype(np.float32))      # ordinary rows with tiny values and zeros sprinkled in
    mod[:, ::97] = rng.choice(mags[:0x3600].astype(np.uint16), (64, len(range(0, K, 97))))
    X = np.concatenate([X, mod])
    act = oracle.gelu(X)
    top = np.abs(oracle.rotate(act)).max(axis=1)
    ok = (top > 1e-30) & (top < 1e37)
    assert ok.sum() > 120
    dx, qx, _ = oracle.rotate_smooth_quant(act[ok])
    Xq, sx = _gpu_gelu_rsq(G.to_dev(X), None, None)
    codes, got = G.gpu_unpack(Xq, K)[ok], sx.cpu().numpy().astype(np.float64)[ok]
    frac = _check(codes, got, qx, dx, "every input value")
    G.report("gelu_every_input_value", rows=int(ok.sum()), code_mismatch_fraction=frac)


def test_mlp_chain_without_an_activation_pass():
    """Config 3 on two frames: fc1 (bf16 out) -> fc2 whose kernel 1 applies the GELU on load, on the E2M3 path, against the
    oracle's chain fc1 -> GELU -> fc2.  Both sides run their own chain from the same X; the fc2 statistic is calibrated on
    each side's own first frame."""
    s1, s2 = synth.layer_spec(3, "fc1"), synth.layer_spec(3, "fc2")
    X = synth.make_activation_frames(s1, [0, 1])
    M = X.shape[0]
    signs1, signs2 = synth.make_signs(s1), synth.make_signs(s2)
    W1, W2, b1, b2 = synth.make_weights(s1), synth.make_weights(s2), synth.make_bias(s1), synth.make_bias(s2)
    a1 = oracle.rotated_col_absmax(synth.make_calibration(s1), pre_signs=signs1)
    p1 = oracle.prepare_weights(W1, a1, pre_signs=signs1)
    h = oracle.linear(X, p1, bias=b1, pre_signs=signs1).Y
    act = oracle.gelu(h)
    p2 = oracle.prepare_weights(W2, oracle.rotated_col_absmax(act[:1374], pre_signs=signs2), pre_signs=signs2)
    want = oracle.linear(act, p2, bias=b2, pre_signs=signs2)
    # GPU chain: fc1 through the whole-path entry point, then fc2's two kernels with the GELU inside the first
    g1 = G.gpu_prep(W1, synth.make_calibration(s1), signs1)
    hd = G.gpu_linear(G.to_dev(X), g1, G.to_dev(b1))
    cal = torch.nn.functional.gelu(hd[:1374].float()).to(torch.bfloat16)          # calibration input only (offline side)
    g2 = G.gpu_prep(W2, G.bf16_bits(cal), signs2)
    Wf = torch.empty(G.q.qvggt_e2m3_bytes(s2.N, s2.K), dtype=torch.uint8, device=G.DEV)
    G.codes_to_e2m3(g2["Wq"], s2.N, s2.K, Wf)
    Xf = torch.empty(G.q.qvggt_e2m3_bytes(M, s2.K), dtype=torch.uint8, device=G.DEV)
    sx = torch.empty(M, dtype=torch.float32, device=G.DEV)
    G.q.qvggt_gelu_rotate_smooth_quant_e2m3(hd, g2["signs"], g2["inv"], G.gelu_table(), Xf, sx)
    Y = torch.empty(M, s2.N, dtype=torch.bfloat16, device=G.DEV)
    G.q.qvggt_e2m3_gemm(Xf, sx, Wf, g2["sw"], G.to_dev(b2), M, s2.N, s2.K, Y, None)
    # the whole-path entry point and the convenience object run the same two kernels
    ws = torch.empty(G.q.qvggt_workspace_bytes_e2m3(M, s2.N, s2.K), dtype=torch.uint8, device=G.DEV)
    Yl = torch.full_like(Y, float("nan"))
    G.q.qvggt_gelu_linear_e2m3(hd, g2["signs"], g2["inv"], G.gelu_table(), Wf, g2["sw"], G.to_dev(b2), Yl, ws)
    assert torch.equal(Y, Yl)
    import paper_2509_21302_amd as q
    layer = q.DsfqLinear(G.to_dev(W2), G.to_dev(b2), G.to_dev(signs2), cal, alpha=0.5, bits=4, pre_gelu=True)
    assert torch.equal(layer(hd), Y)
    err = G.rel_fro(G.bf16_bits(Y), want.Y)
    assert err <= G.Y_REL_FRO, err          # two quantized layers in sequence at the stated bar (all 8 frames: tests/test_gpu_config3_chain.py)
    # and the fused kernel equals the unfused sequence on the GPU's own fc1 output up to the bf16 rounding flips of the activation
    actd = torch.nn.functional.gelu(hd.float()).to(torch.bfloat16)
    Y2 = G.gpu_linear(actd, g2, G.to_dev(b2))
    assert G.rel_fro(G.bf16_bits(Y), G.bf16_bits(Y2)) <= G.Y_REL_FRO


def test_gelu_rotate_quant_full_size():
    """137400 x 4096 (fc2 of the benchmark's config, its synthetic input standing in for fc1's output) in the launch configuration
    bench.py times: a seeded sample of rows against the oracle, and the E2M3 output against the packed one through the GEMM
    (equal codes give equal sums, whatever sign a zero carries)."""
    s = synth.layer_spec(5, "fc2")
    rng = np.random.default_rng(58)
    rows = np.unique(np.concatenate([np.arange(synth.SPECIAL_TOKENS), np.arange(s.M - 64, s.M), rng.choice(s.M, 250, replace=False)]))
    signs = synth.make_signs(s)
    inv = (1.0 / (np.sqrt(s.K) * np.exp(rng.uniform(-1, 1, s.K)))).astype(np.float32)
    X = synth.make_activation_frames(s)
    Xd, sd, invd = G.to_dev(X), G.to_dev(signs), G.to_dev(inv)
    Xs = X[rows]
    del X
    dx, qx, _ = oracle.rotate_smooth_quant(oracle.gelu(Xs), 1.0 / (inv.astype(np.float64) * np.sqrt(s.K)), pre_signs=signs)
    Xq, sx = _gpu_gelu_rsq(Xd, sd, invd)
    idx = torch.from_numpy(rows).to(G.DEV)
    _check(G.gpu_unpack(Xq[idx].contiguous(), s.K), sx[idx].cpu().numpy().astype(np.float64), qx, dx, "full size")
    Xf = torch.empty(G.q.qvggt_e2m3_bytes(s.M, s.K), dtype=torch.uint8, device=G.DEV)
    sxf = torch.empty_like(sx)
    G.q.qvggt_gelu_rotate_smooth_quant_e2m3(Xd, sd, invd, G.gelu_table(), Xf, sxf)
    assert torch.equal(sx, sxf)
    del Xd
    N = 256
    Wq = G.gpu_pack(rng.integers(-7, 8, (N, s.K)).astype(np.int8))
    Wf = torch.empty(G.q.qvggt_e2m3_bytes(N, s.K), dtype=torch.uint8, device=G.DEV)
    G.codes_to_e2m3(Wq, N, s.K, Wf)
    sw = torch.full((N,), 1e-3, dtype=torch.float32, device=G.DEV)
    Y1 = torch.empty(s.M, N, dtype=torch.bfloat16, device=G.DEV)
    G.q.qvggt_e2m3_gemm(Xf, sx, Wf, sw, None, s.M, N, s.K, Y1, None)
    G.codes_to_e2m3(Xq, s.M, s.K, Xf)
    Y2 = torch.empty_like(Y1)
    G.q.qvggt_e2m3_gemm(Xf, sx, Wf, sw, None, s.M, N, s.K, Y2, None)
    assert torch.equal(Y1, Y2)
