"""GPU parity of the GEMM on the 6-bit floating-point matrix path: 4-bit codes written as E2M3 numbers, the integer sums
exact in fp32.  Accumulators bit-exact against the oracle's integer product, Y against its epilogue, and identical to the
int8-path kernel on the same codes."""
import numpy as np
import pytest
import torch

import oracle
from synth import f32_to_bf16_bits
from tests import gpu_util as G

pytestmark = pytest.mark.gpu


def _e2m3(codes_np):
    """natural-order int8 codes -> packed rows (library order) -> E2M3 rows"""
    packed = G.gpu_pack(codes_np)
    rows, K = codes_np.shape
    out = torch.full((G.q.qvggt_e2m3_bytes(rows, K),), 0xA5, dtype=torch.uint8, device=G.DEV)        # pad rows keep the fill
    G.codes_to_e2m3(packed, rows, K, out)
    return packed, out


_decode_e2m3_rows = G.decode_e2m3_rows


def test_codes_to_e2m3_layout_and_values():
    K, rows = 256, 300
    rng = np.random.default_rng(0)
    codes = rng.integers(-7, 8, (rows, K)).astype(np.int8)
    codes[0] = np.resize(np.arange(-7, 8), K)
    packed, out = _e2m3(codes)
    pk = packed.cpu().numpy()
    nib = np.stack([pk & 15, pk >> 4], axis=2).reshape(rows, K).astype(np.int16)          # position p = byte p / 2, nibble p % 2
    at_position = np.where(nib >= 8, nib - 16, nib)
    assert np.array_equal(_decode_e2m3_rows(out.cpu().numpy(), rows, K), at_position.astype(np.float64))
    assert np.array_equal(np.sort(at_position, axis=1), np.sort(codes, axis=1))            # the library order is a permutation of a row


def test_codes_to_e2m3_counts_what_it_cannot_carry():
    """-8 has no E2M3 value: the converter writes -7 there and says how many times it did, so a caller cannot mistake the buffer
    for a faithful copy (a static weight step below the channel's own produces such codes)."""
    K, rows = 1024, 130
    rng = np.random.default_rng(5)
    codes = rng.integers(-8, 8, (rows, K)).astype(np.int8)
    n_lost = int((codes == -8).sum())
    assert n_lost > 1000
    packed = G.gpu_pack(codes)
    out = torch.zeros(G.q.qvggt_e2m3_bytes(rows, K), dtype=torch.uint8, device=G.DEV)
    assert G.codes_to_e2m3(packed, rows, K, out, expect_clean=False) == n_lost
    pk = packed.cpu().numpy()
    nib = np.stack([pk & 15, pk >> 4], axis=2).reshape(rows, K).astype(np.int16)
    at_position = np.where(nib >= 8, nib - 16, nib)
    assert np.array_equal(_decode_e2m3_rows(out.cpu().numpy(), rows, K), np.maximum(at_position, -7).astype(np.float64))
    # the counter accumulates: a second call adds to it
    cnt = torch.zeros(1, dtype=torch.int32, device=G.DEV)
    G.q.qvggt_codes_to_e2m3(packed, rows, K, out, cnt)
    G.q.qvggt_codes_to_e2m3(packed, rows, K, out, cnt)
    assert int(cnt.item()) == 2 * n_lost


def _run(qx, qw, dx, dw, bias_bits, debug=True):
    M, K = qx.shape
    N = qw.shape[0]
    (Xq, Xf), (Wq, Wf) = _e2m3(qx), _e2m3(qw)
    Y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=G.DEV)
    acc = torch.full((M, N), 12345, dtype=torch.int32, device=G.DEV) if debug else None
    G.q.qvggt_e2m3_gemm(Xf, G.to_dev(dx), Wf, G.to_dev(dw), G.to_dev(bias_bits), M, N, K, Y, acc)
    Y8 = torch.empty_like(Y)
    G.q.qvggt_w4a4_gemm(Xq, G.to_dev(dx), Wq, G.to_dev(dw), G.to_dev(bias_bits), M, N, K, Y8)
    return acc, Y, Y8


@pytest.mark.parametrize("M,N,K", [(64, 128, 128), (1, 16, 128), (300, 384, 256), (129, 144, 1024), (1374, 3072, 1024),
                                   (257, 1024, 4096), (33, 48, 8192), (500, 1040, 768)])
@pytest.mark.parametrize("with_bias", [True, False])
def test_e2m3_gemm_bit_exact(M, N, K, with_bias):
    rng = np.random.default_rng(M * 7 + N + K)
    qx = rng.integers(-7, 8, (M, K)).astype(np.int8)
    qw = rng.integers(-7, 8, (N, K)).astype(np.int8)
    dx = np.exp(rng.uniform(-3, 1, M)).astype(np.float32)
    dw = np.exp(rng.uniform(-5, -2, N)).astype(np.float32)
    bias_bits = f32_to_bf16_bits((rng.standard_normal(N) * 0.02).astype(np.float32)) if with_bias else None
    acc, Y, Y8 = _run(qx, qw, dx, dw, bias_bits)
    want = oracle.int_gemm(qx, qw)
    assert np.array_equal(acc.cpu().numpy(), want)
    Yo = oracle.dequant_bias(want, dx, dw, None if bias_bits is None else oracle.to_f64(bias_bits))
    ulp_off = np.abs(G.bf16_bits(Y).astype(np.int32) - Yo.astype(np.int32))
    assert ulp_off.max() <= 1 and (ulp_off != 0).mean() < 5e-3
    assert torch.equal(Y, Y8)                                    # the int8-path kernel gives the same bits


def test_e2m3_gemm_extreme_sums():
    """Every product +49 or -49 over the longest row: |acc| = 49 * 8192 needs 19 bits, exact in fp32 whatever the order."""
    M, N, K = 40, 32, 8192
    qx = np.full((M, K), 7, dtype=np.int8)
    qx[1::2] = -7
    qw = np.full((N, K), 7, dtype=np.int8)
    qw[::3] = -7
    qw[5, ::2] = 0
    acc, Y, Y8 = _run(qx, qw, np.ones(M, np.float32), np.ones(N, np.float32), None)
    assert np.array_equal(acc.cpu().numpy(), oracle.int_gemm(qx, qw))
    assert torch.equal(Y, Y8)


@pytest.mark.parametrize("M,N,K", [(66000, 512, 256), (65700, 768, 128), (16500, 4096, 1024)])
def test_e2m3_gemm_large_shapes(M, N, K):
    """Several rounds of 256 x 256 tiles with a ragged last tile row (the smaller shapes above run the 128 x 128 configuration):
    sampled rows (around the last full round, the last rows, random ones) bit-exact; every row written."""
    tiles_n = (N + 255) // 256
    seam = ((M + 255) // 256 * tiles_n // 256 * 256 // tiles_n) * 256
    assert 0 < seam < M
    gen = torch.Generator(device="cpu").manual_seed(M)
    qx = torch.randint(-7, 8, (M, K), generator=gen, dtype=torch.int8).numpy()
    qw = torch.randint(-7, 8, (N, K), generator=gen, dtype=torch.int8).numpy()
    rng = np.random.default_rng(M)
    dx = np.exp(rng.uniform(-3, 1, M)).astype(np.float32)
    dw = np.exp(rng.uniform(-8, -4, N)).astype(np.float32)
    acc, Y, Y8 = _run(qx, qw, dx, dw, None)
    rows = np.unique(np.concatenate([np.arange(0, 8), np.arange(seam - 300, min(seam + 300, M)), np.arange(M - 200, M),
                                     rng.choice(M, 200, replace=False)]))
    idx = torch.from_numpy(rows).to(G.DEV)
    want = oracle.int_gemm(qx[rows], qw)
    assert np.array_equal(acc[idx].cpu().numpy(), want)
    Yo = oracle.dequant_bias(want, dx[rows], dw, None)
    ulp_off = np.abs(G.bf16_bits(Y[idx]).astype(np.int32) - Yo.astype(np.int32))
    assert ulp_off.max() <= 1 and (ulp_off != 0).mean() < 5e-3
    assert not torch.isnan(Y.float()).any().item()
    assert torch.equal(Y, Y8)


def _position_of_element(K):
    """Where natural channel e sits in a row of codes, from the layout's statement in include/qvggt.h: identity except for
    K = 1024, 2048, 4096, where e = 128 hb + 32 nt + c goes to position c (K / 32) + nt + 4 hb' (hb' = hb, with bits 3 and 4
    of hb swapped at K = 4096)."""
    e = np.arange(K)
    if K not in (1024, 2048, 4096):
        return e
    c, nt, hb = e & 31, (e >> 5) & 3, e >> 7
    if K == 4096:
        hb = (hb & ~0x18) | ((hb & 8) << 1) | ((hb & 16) >> 1)
    return c * (K // 32) + nt + 4 * hb


def _heavy_bf16(rows, K, seed):
    import synth
    rng = np.random.default_rng(seed)
    x = rng.standard_t(3, (rows, K)).astype(np.float32)
    x[:, rng.choice(K, max(1, K // 100), replace=False)] *= 50
    x[: min(5, rows)] *= 20
    return synth.f32_to_bf16_bits(x)


@pytest.mark.parametrize("K,rows", [(1024, 1031), (2048, 300), (4096, 203)])
def test_rotate_quant_e2m3_is_kernel_1_in_another_format(K, rows):
    """Kernel 1 writing E2M3 blocks directly: decoded values equal the oracle's codes at the library's positions to the usual
    bar, equal the converted output of the packed-code kernel exactly, and the steps are the same floats."""
    X = _heavy_bf16(rows, K, 900 + K)
    X[7] = 0
    rng = np.random.default_rng(K + 1)
    signs = (rng.integers(0, 2, K) * 2 - 1).astype(np.int8)
    c_hat = np.exp(rng.uniform(-1, 1, K))
    inv = (1.0 / (np.sqrt(K) * c_hat)).astype(np.float32)
    Xd, sd, invd = G.to_dev(X), G.to_dev(signs), G.to_dev(inv)
    Xq, sx = G.gpu_rsq(Xd, sd, invd)
    Xf = torch.full((G.q.qvggt_e2m3_bytes(rows, K),), 0xA5, dtype=torch.uint8, device=G.DEV)
    sxf = torch.empty(rows, dtype=torch.float32, device=G.DEV)
    G.q.qvggt_rotate_smooth_quant_e2m3(Xd, sd, invd, Xf, sxf)
    assert torch.equal(sx, sxf)
    got = _decode_e2m3_rows(Xf.cpu().numpy(), rows, K)
    conv = torch.full_like(Xf, 0xA5)
    G.codes_to_e2m3(Xq, rows, K, conv)
    assert np.array_equal(got, _decode_e2m3_rows(conv.cpu().numpy(), rows, K))           # -0 and 0 compare equal
    assert not got[7].any()
    # directly against the oracle, with no other kernel in between: decode the E2M3 blocks (numpy, from the format's definition),
    # bring the positions of a row back to natural channel order (the permutation as the header states it), compare element-wise
    dx, qx, _ = oracle.rotate_smooth_quant(X, 1.0 / (inv.astype(np.float64) * np.sqrt(K)), pre_signs=signs)
    G.check_scales(sxf.cpu().numpy(), dx)
    natural = got[:, _position_of_element(K)]
    assert np.array_equal(natural, np.rint(natural)) and np.abs(natural).max() <= 7
    frac = G.check_codes(natural.astype(np.int8), qx, f"E2M3 blocks decoded, K={K}")
    G.report("rotate_quant_e2m3_direct", K=K, rows=rows, code_mismatch_fraction=frac)
    G.check_codes(G.gpu_unpack(Xq, K), qx)                       # and the packed kernel beside it


@pytest.mark.parametrize("name,M", [("fc1", 3000), ("fc2", 700)])
def test_linear_e2m3_matches_the_oracle_and_the_int8_path(name, M):
    """Whole online path through the 6-bit matrix instructions against the oracle's layer; bit-identical to qvggt_linear."""
    import synth
    s = synth.layer_spec(5, name)
    K, N = s.K, s.N
    rng = np.random.default_rng(M)
    X = _heavy_bf16(M, K, 40 + M)
    W = synth.make_weights(s)
    bias = synth.make_bias(s)
    signs = synth.make_signs(s)
    cal = X[:512]
    po = oracle.prepare_weights(W, oracle.rotated_col_absmax(cal, pre_signs=signs), pre_signs=signs)
    want = oracle.linear(X, po, bias=bias, pre_signs=signs)
    pg = G.gpu_prep(W, cal, signs)
    Wf = torch.empty(G.q.qvggt_e2m3_bytes(N, K), dtype=torch.uint8, device=G.DEV)
    G.codes_to_e2m3(pg["Wq"], N, K, Wf)
    Y = torch.empty(M, N, dtype=torch.bfloat16, device=G.DEV)
    ws = torch.empty(G.q.qvggt_workspace_bytes_e2m3(M, N, K), dtype=torch.uint8, device=G.DEV)
    G.q.qvggt_linear_e2m3(G.to_dev(X), pg["signs"], pg["inv"], Wf, pg["sw"], G.to_dev(bias), Y, ws)
    assert G.rel_fro(G.bf16_bits(Y), want.Y) <= G.Y_REL_FRO
    assert torch.equal(Y, G.gpu_linear(G.to_dev(X), pg, G.to_dev(bias)))


def test_layernorm_rotate_quant_e2m3_equals_the_packed_variant():
    """LayerNorm fused in front, E2M3 output: the same steps and, decoded, the same codes as the packed-code variant (whose
    parity against the oracle is tests/test_gpu_rotate_quant.py::test_layernorm_rotate_quant)."""
    K, rows, eps = 1024, 1031, 1e-5
    X = _heavy_bf16(rows, K, 77)
    rng = np.random.default_rng(5)
    signs = (rng.integers(0, 2, K) * 2 - 1).astype(np.int8)
    inv = (1.0 / (np.sqrt(K) * np.exp(rng.uniform(-1, 1, K)))).astype(np.float32)
    gamma = np.exp(rng.normal(0, 0.3, K)).astype(np.float32)
    beta = rng.normal(0, 0.1, K).astype(np.float32)
    Xd, sd, invd, gd, bd = (G.to_dev(v) for v in (X, signs, inv, gamma, beta))
    Xq, sx = G.gpu_ln_rsq(Xd, gd, bd, eps, sd, invd)
    Xf = torch.full((G.q.qvggt_e2m3_bytes(rows, K),), 0xA5, dtype=torch.uint8, device=G.DEV)
    sxf = torch.empty(rows, dtype=torch.float32, device=G.DEV)
    G.q.qvggt_layernorm_rotate_smooth_quant_e2m3(Xd, gd, bd, eps, sd, invd, Xf, sxf)
    assert torch.equal(sx, sxf)
    conv = torch.full_like(Xf, 0xA5)
    G.codes_to_e2m3(Xq, rows, K, conv)
    assert np.array_equal(_decode_e2m3_rows(Xf.cpu().numpy(), rows, K), _decode_e2m3_rows(conv.cpu().numpy(), rows, K))


def _shifted_setup(K, rows, N, seed, one_sided):
    rng = np.random.default_rng(seed)
    X = _heavy_bf16(rows, K, seed)
    if one_sided:
        X = f32_to_bf16_bits(np.abs(oracle.to_f64(X)).astype(np.float32))
    W = rng.standard_normal((N, K)).astype(np.float32) * 0.03
    bias = f32_to_bf16_bits(rng.normal(0, 0.1, N).astype(np.float32))
    signs = (rng.integers(0, 2, K) * 2 - 1).astype(np.int8)
    pg = G.gpu_prep(W, X, signs)
    Wf = torch.empty(G.q.qvggt_e2m3_bytes(N, K), dtype=torch.uint8, device=G.DEV)
    G.codes_to_e2m3(pg["Wq"], N, K, Wf)
    return X, W, bias, signs, pg, Wf, G.gpu_code_sums(pg["Wq"], N, K)


@pytest.mark.parametrize("K,rows,N", [(1024, 1031, 512), (4096, 600, 1024), (2048, 203, 256)])
def test_asymmetric_codes_on_the_e2m3_path(K, rows, N):
    """Affine activation codes stored as u - 7.5: decoded + 7.5 they are the packed kernel's u (whose parity against the oracle
    is tests/test_gpu_asym.py), same steps and zero points; the layer's Y equals the int8-instruction path's bit for bit and is
    within the usual bar of the oracle's asymmetric layer."""
    X, W, bias, signs, pg, Wf, wsum = _shifted_setup(K, rows, N, 50 + K, True)
    Xd = G.to_dev(X)
    Xq, sx, zx = G.gpu_rsq_asym(Xd, pg["signs"], pg["inv"])
    Xf = torch.full((G.q.qvggt_e2m3_bytes(rows, K),), 0xA5, dtype=torch.uint8, device=G.DEV)
    sxf, zxf = torch.empty_like(sx), torch.empty_like(zx)
    G.q.qvggt_rotate_smooth_quant_asym_e2m3(Xd, pg["signs"], pg["inv"], Xf, sxf, zxf)
    assert torch.equal(sx, sxf) and torch.equal(zx, zxf)
    pk = Xq.cpu().numpy()
    nib = np.stack([pk & 15, pk >> 4], axis=2).reshape(rows, K).astype(np.int16)
    at_position = np.where(nib >= 8, nib - 16, nib)                                        # u - 8 at the library's positions
    assert np.array_equal(_decode_e2m3_rows(Xf.cpu().numpy(), rows, K), at_position + 0.5)
    Y = torch.empty(rows, N, dtype=torch.bfloat16, device=G.DEV)
    G.q.qvggt_e2m3_gemm_shifted(Xf, sxf, zxf, Wf, pg["sw"], wsum, G.to_dev(bias), rows, N, K, Y)
    Y8 = torch.empty_like(Y)
    G.q.qvggt_w4a4_gemm_asym(Xq, sx, zx, pg["Wq"], pg["sw"], wsum, G.to_dev(bias), rows, N, K, Y8)
    assert torch.equal(Y, Y8)
    po = oracle.prepare_weights(W, oracle.rotated_col_absmax(X, pre_signs=signs), pre_signs=signs)
    want = oracle.linear_asym(X, po, bias, pre_signs=signs)[0]
    assert G.rel_fro(G.bf16_bits(Y), want) <= G.Y_REL_FRO


@pytest.mark.parametrize("K,rows,N,per_token", [(1024, 1031, 512, 1), (4096, 300, 256, 0), (2048, 203, 256, 1)])
def test_static_step_codes_on_the_e2m3_path(K, rows, N, per_token):
    """A given step (codes reach -8) stored as code + 0.5 with zero = 8: decoded - 0.5 they are the packed kernel's codes, and Y
    equals the int8-instruction path's bit for bit."""
    X, W, bias, signs, pg, Wf, wsum = _shifted_setup(K, rows, N, 60 + K, False)
    Xd = G.to_dev(X)
    _, sdyn = G.gpu_rsq(Xd, pg["signs"], pg["inv"])
    rng = np.random.default_rng(K)
    dyn = sdyn.cpu().numpy()
    step = (dyn * rng.uniform(0.2, 1.5, rows)).astype(np.float32) if per_token else np.array([np.median(dyn) * 0.5], dtype=np.float32)
    Xq, sx = G.gpu_rsq_static(Xd, pg["signs"], pg["inv"], G.to_dev(step), per_token)
    codes = G.gpu_unpack(Xq, K)
    assert (codes == -8).any() and (codes == 7).any()
    Xf = torch.full((G.q.qvggt_e2m3_bytes(rows, K),), 0xA5, dtype=torch.uint8, device=G.DEV)
    sxf, zxf = torch.empty_like(sx), torch.empty_like(sx)
    G.q.qvggt_rotate_smooth_quant_static_e2m3(Xd, pg["signs"], pg["inv"], G.to_dev(step), per_token, Xf, sxf, zxf)
    assert torch.equal(sx, sxf) and (zxf == 8).all().item()
    pk = Xq.cpu().numpy()
    nib = np.stack([pk & 15, pk >> 4], axis=2).reshape(rows, K).astype(np.int16)
    at_position = np.where(nib >= 8, nib - 16, nib)
    assert np.array_equal(_decode_e2m3_rows(Xf.cpu().numpy(), rows, K), at_position + 0.5)
    Y = torch.empty(rows, N, dtype=torch.bfloat16, device=G.DEV)
    G.q.qvggt_e2m3_gemm_shifted(Xf, sxf, zxf, Wf, pg["sw"], wsum, G.to_dev(bias), rows, N, K, Y)
    Y8 = torch.empty_like(Y)
    G.q.qvggt_w4a4_gemm(Xq, sx, pg["Wq"], pg["sw"], G.to_dev(bias), rows, N, K, Y8)
    assert torch.equal(Y, Y8)


@pytest.mark.parametrize("M", [1, 5, 130])
@pytest.mark.parametrize("K,N", [(1024, 48), (4096, 272)])
def test_linear_e2m3_few_rows(M, K, N):
    """Fewer rows than a 128-row block of the operand format (the rest of the block is never written and holds a fill here):
    the same bits as qvggt_linear."""
    rng = np.random.default_rng(M + K)
    X = _heavy_bf16(M, K, M + K)
    W = rng.standard_normal((N, K)).astype(np.float32) * 0.05
    signs = (rng.integers(0, 2, K) * 2 - 1).astype(np.int8)
    pg = G.gpu_prep(W, X, signs)
    Wf = torch.full((G.q.qvggt_e2m3_bytes(N, K),), 0xFF, dtype=torch.uint8, device=G.DEV)
    G.codes_to_e2m3(pg["Wq"], N, K, Wf)
    Y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=G.DEV)
    ws = torch.full((G.q.qvggt_workspace_bytes_e2m3(M, N, K),), 0xFF, dtype=torch.uint8, device=G.DEV)
    G.q.qvggt_linear_e2m3(G.to_dev(X), pg["signs"], pg["inv"], Wf, pg["sw"], None, Y, ws)
    assert torch.equal(Y, G.gpu_linear(G.to_dev(X), pg, None))
    want = oracle.linear(X, oracle.prepare_weights(W, oracle.rotated_col_absmax(X, pre_signs=signs), pre_signs=signs), pre_signs=signs)
    assert G.rel_fro(G.bf16_bits(Y), want.Y) <= G.Y_REL_FRO
