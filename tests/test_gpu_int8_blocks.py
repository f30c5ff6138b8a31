"""GPU parity of the int8-code path on blocked operands ("int8 blocks"): the same codes, integer sums and outputs as the
qvggt_*_i8 entry points, whose parity against the oracle is tests/test_gpu_int8_path.py; accumulators also directly against the
oracle's integer product."""
import numpy as np
import pytest
import torch

import oracle
import synth
from synth import f32_to_bf16_bits
from tests import gpu_util as G

pytestmark = pytest.mark.gpu


def _blocks(codes_np):
    lib = G.gpu_layout_int8(codes_np, 1)
    rows, K = codes_np.shape
    out = torch.full((G.q.qvggt_i8b_bytes(rows, K),), 0x5A, dtype=torch.uint8, device=G.DEV).view(torch.int8)
    G.q.qvggt_int8_to_blocks(lib, rows, K, out)
    return lib, out


def test_int8_to_blocks_layout():
    rows, K = 300, 256
    codes = np.random.default_rng(0).integers(-128, 128, (rows, K)).astype(np.int8)
    lib, out = _blocks(codes)
    L, B = lib.cpu().numpy(), out.cpu().numpy()
    r = np.arange(rows)
    for kt in range(K // 64):
        for ch in range(4):
            slot = ch ^ ((r % 16) >> 2)
            start = ((r // 128) * (K // 64) + kt) * 8192 + (r % 128) * 64 + slot * 16
            got = B[start[:, None] + np.arange(16)[None, :]]
            assert np.array_equal(got, L[:, kt * 64 + ch * 16: kt * 64 + ch * 16 + 16])


@pytest.mark.parametrize("M,N,K", [(64, 128, 128), (1, 16, 128), (300, 384, 256), (1374, 3072, 1024), (257, 1024, 4096), (33, 48, 8192),
                                   (500, 1040, 768)])
def test_i8b_gemm_bit_exact(M, N, K):
    rng = np.random.default_rng(M + N + K)
    qx = rng.integers(-128, 128, (M, K)).astype(np.int8)
    qw = rng.integers(-128, 128, (N, K)).astype(np.int8)
    dx = np.exp(rng.uniform(-3, 1, M)).astype(np.float32)
    dw = np.exp(rng.uniform(-8, -4, N)).astype(np.float32)
    bias_bits = f32_to_bf16_bits((rng.standard_normal(N) * 0.02).astype(np.float32))
    (Xl, Xb), (Wl, Wb) = _blocks(qx), _blocks(qw)
    Y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=G.DEV)
    acc = torch.full((M, N), 12345, dtype=torch.int32, device=G.DEV)
    G.q.qvggt_i8b_gemm(Xb, G.to_dev(dx), Wb, G.to_dev(dw), G.to_dev(bias_bits), M, N, K, Y, acc)
    assert np.array_equal(acc.cpu().numpy(), oracle.int_gemm(qx, qw))
    Y8 = torch.empty_like(Y)
    G.q.qvggt_i8_gemm(Xl, G.to_dev(dx), Wl, G.to_dev(dw), G.to_dev(bias_bits), M, N, K, Y8, None)
    assert torch.equal(Y, Y8)


@pytest.mark.parametrize("M,N,K", [(66000, 512, 256), (33000, 1024, 512)])
def test_i8b_gemm_both_tile_shapes(M, N, K):
    """Whole rounds of big tiles plus a remainder in the small configuration: every row equals the row-major kernel's."""
    gen = torch.Generator(device="cpu").manual_seed(M)
    qx = torch.randint(-128, 128, (M, K), generator=gen, dtype=torch.int8).numpy()
    qw = torch.randint(-128, 128, (N, K), generator=gen, dtype=torch.int8).numpy()
    rng = np.random.default_rng(M)
    dx = np.exp(rng.uniform(-3, 1, M)).astype(np.float32)
    dw = np.exp(rng.uniform(-8, -4, N)).astype(np.float32)
    (Xl, Xb), (Wl, Wb) = _blocks(qx), _blocks(qw)
    Y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=G.DEV)
    G.q.qvggt_i8b_gemm(Xb, G.to_dev(dx), Wb, G.to_dev(dw), None, M, N, K, Y, None)
    Y8 = torch.empty_like(Y)
    G.q.qvggt_i8_gemm(Xl, G.to_dev(dx), Wl, G.to_dev(dw), None, M, N, K, Y8, None)
    assert torch.equal(Y, Y8)
    rows = np.unique(np.concatenate([np.arange(0, 8), np.arange(M - 200, M), rng.choice(M, 200, replace=False)]))
    acc = torch.full((M, N), 12345, dtype=torch.int32, device=G.DEV)
    G.q.qvggt_i8b_gemm(Xb, G.to_dev(dx), Wb, G.to_dev(dw), None, M, N, K, Y, acc)
    assert np.array_equal(acc[torch.from_numpy(rows).to(G.DEV)].cpu().numpy(), oracle.int_gemm(qx[rows], qw))


@pytest.mark.parametrize("K,rows", [(1024, 1031), (2048, 300), (4096, 203)])
@pytest.mark.parametrize("bits", [8, 6])
def test_rotate_quant_i8b_equals_the_row_major_kernel(K, rows, bits):
    rng = np.random.default_rng(K + bits)
    x = rng.standard_t(3, (rows, K)).astype(np.float32)
    x[:, rng.choice(K, K // 100, replace=False)] *= 50
    X = f32_to_bf16_bits(x)
    signs = (rng.integers(0, 2, K) * 2 - 1).astype(np.int8)
    inv = (1.0 / (np.sqrt(K) * np.exp(rng.uniform(-1, 1, K)))).astype(np.float32)
    Xd, sd, invd = G.to_dev(X), G.to_dev(signs), G.to_dev(inv)
    Xq, sx = G.gpu_rsq_i8(Xd, sd, invd, bits)
    want = torch.full((G.q.qvggt_i8b_bytes(rows, K),), 0x5A, dtype=torch.uint8, device=G.DEV).view(torch.int8)
    G.q.qvggt_int8_to_blocks(Xq, rows, K, want)
    got = torch.full_like(want, 0x5A)
    sxb = torch.empty_like(sx)
    G.q.qvggt_rotate_smooth_quant_i8b(Xd, sd, invd, bits, got, sxb)
    assert torch.equal(sx, sxb) and torch.equal(got, want)


@pytest.mark.parametrize("name,M,bits", [("fc1", 3000, 8), ("fc2", 700, 8), ("fc1", 130, 6)])
def test_linear_i8b(name, M, bits):
    s = synth.layer_spec(5, name)
    K, N = s.K, s.N
    rng = np.random.default_rng(M)
    x = rng.standard_t(3, (M, K)).astype(np.float32)
    X = f32_to_bf16_bits(x)
    W, bias, signs = synth.make_weights(s), synth.make_bias(s), synth.make_signs(s)
    pg = G.gpu_prep_i8(W, X[:512], signs, bits)
    Wb = torch.empty(G.q.qvggt_i8b_bytes(N, K), dtype=torch.int8, device=G.DEV)
    G.q.qvggt_int8_to_blocks(pg["Wq"], N, K, Wb)
    Y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=G.DEV)
    ws = torch.empty(G.q.qvggt_workspace_bytes_i8b(M, N, K), dtype=torch.uint8, device=G.DEV)
    G.q.qvggt_linear_i8b(G.to_dev(X), pg["signs"], pg["inv"], bits, Wb, pg["sw"], G.to_dev(bias), Y, ws)
    assert torch.equal(Y, G.gpu_linear_i8(G.to_dev(X), pg, G.to_dev(bias)))
    po = oracle.prepare_weights(W, oracle.rotated_col_absmax(X[:512], pre_signs=signs), pre_signs=signs, bits=bits)
    want = oracle.linear(X, po, bias=bias, pre_signs=signs, bits=bits)
    assert G.rel_fro(G.bf16_bits(Y), want.Y) <= G.Y_REL_FRO


@pytest.mark.parametrize("name,n_random", [("fc1", 600), ("fc2", 300)])
def test_linear_i8b_full_size(name, n_random):
    """The benchmark's shapes (137400 tokens) in the launch configuration bench.py times: every element of Y equals the row-major
    path's, and a seeded sample of rows is within the output bound of the oracle's."""
    s = synth.layer_spec(5, name)
    rng = np.random.default_rng(len(name) + 8)
    rows = np.unique(np.concatenate([np.arange(synth.SPECIAL_TOKENS), np.arange(s.M - 64, s.M), rng.choice(s.M, n_random, replace=False)]))
    signs = synth.make_signs(s)
    W, Xc, bias = synth.make_weights(s), synth.make_calibration(s), synth.make_bias(s)
    po = oracle.prepare_weights(W, oracle.rotated_col_absmax(Xc, pre_signs=signs), pre_signs=signs, alpha=0.5, bits=8)
    pg = G.gpu_prep_i8(W, Xc, signs, 8)
    X = synth.make_activation_frames(s)
    Xd = G.to_dev(X)
    want = oracle.linear(X[rows], po, bias=bias, pre_signs=signs, bits=8)
    del X
    Wb = torch.empty(G.q.qvggt_i8b_bytes(s.N, s.K), dtype=torch.int8, device=G.DEV)
    G.q.qvggt_int8_to_blocks(pg["Wq"], s.N, s.K, Wb)
    Y = torch.full((s.M, s.N), float("nan"), dtype=torch.bfloat16, device=G.DEV)
    ws = torch.empty(G.q.qvggt_workspace_bytes_i8b(s.M, s.N, s.K), dtype=torch.uint8, device=G.DEV)
    G.q.qvggt_linear_i8b(Xd, pg["signs"], pg["inv"], 8, Wb, pg["sw"], G.to_dev(bias), Y, ws)
    idx = torch.from_numpy(rows).to(G.DEV)
    err = G.rel_fro(G.bf16_bits(Y[idx]), want.Y)
    assert err <= G.Y_REL_FRO, err
    assert torch.equal(Y, G.gpu_linear_i8(Xd, pg, G.to_dev(bias)))
